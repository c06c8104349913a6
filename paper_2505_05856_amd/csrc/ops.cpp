// Standalone operator entry points and diagnostics of dpstage's C ABI: the kernels the stage
// step uses, callable one at a time for operator-level parity tests and microbenchmarks.
#include "stage_internal.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>

using namespace dpi;

extern "C" {

// ---------------------------------------------------------------- standalone ops
size_t dp_op_workspace_bytes(int32_t rows, int32_t cols) {
  return std::max(dp::reduce_ws_bytes(rows, cols), (size_t)rows * (size_t)cols * sizeof(float));
}

static dp_status op_done(hipError_t e, const char *what) {
  return e == hipSuccess ? DP_OK : fail(DP_E_HIP, "%s: %s", what, hipGetErrorString(e));
}
static bool bad_dtype(int32_t d) { return d != DP_F32 && d != DP_BF16; }

static dp_status norm_fwd(bool rms, int32_t dtype, int32_t rows, int32_t cols, float eps, const void *x,
                          const void *gamma, const void *beta, void *y, float *stats, void *hip_stream) {
  if (!bad_dtype(dtype) && rows == 0) return DP_OK;   // nothing to do; the row pointers may be null
  if (bad_dtype(dtype) || rows < 0 || !x || !gamma || !beta) return fail(DP_E_INVAL, "norm_fwd: bad argument");
  if (!dp::ln_supported(dtype, cols)) return fail(DP_E_UNSUPPORTED, "norm: cols must be a multiple of 8, <= 8192");
  return op_done(dp::launch_ln_fwd(dtype, rows, cols, eps, x, gamma, beta, y, stats, (hipStream_t)hip_stream, rms),
                 "norm_fwd");
}

static dp_status norm_bwd(bool rms, int32_t dtype, int32_t rows, int32_t cols, const void *dy, const void *x,
                          const float *stats, const void *gamma, const void *dres, void *dx, void *dgamma, void *dbeta,
                          void *dx_colsum, void *ws, void *hip_stream) {
  if (bad_dtype(dtype) || rows < 0 || !dgamma || !dbeta || (rows > 0 && (!dy || !x || !stats || !gamma || !dx || !ws)))
    return fail(DP_E_INVAL, "norm_bwd: bad argument");   // (no rows: only the sums, which become zero, are touched)
  if (!dp::ln_supported(dtype, cols)) return fail(DP_E_UNSUPPORTED, "norm: cols must be a multiple of 8, <= 8192");
  return op_done(dp::launch_ln_bwd(dtype, rows, cols, dy, x, stats, gamma, dres, dx, dgamma, dbeta, dx_colsum, ws,
                                   (hipStream_t)hip_stream, nullptr, rms), "norm_bwd");
}

dp_status dp_op_layernorm_fwd(int32_t dtype, int32_t rows, int32_t cols, float eps, const void *x, const void *gamma,
                              const void *beta, void *y, float *stats, void *hip_stream) {
  return norm_fwd(false, dtype, rows, cols, eps, x, gamma, beta, y, stats, hip_stream);
}
dp_status dp_op_layernorm_bwd(int32_t dtype, int32_t rows, int32_t cols, const void *dy, const void *x,
                              const float *stats, const void *gamma, const void *dres, void *dx, void *dgamma,
                              void *dbeta, void *dx_colsum, void *ws, void *hip_stream) {
  return norm_bwd(false, dtype, rows, cols, dy, x, stats, gamma, dres, dx, dgamma, dbeta, dx_colsum, ws, hip_stream);
}
dp_status dp_op_rmsnorm_fwd(int32_t dtype, int32_t rows, int32_t cols, float eps, const void *x, const void *gamma,
                            const void *beta, void *y, float *stats, void *hip_stream) {
  return norm_fwd(true, dtype, rows, cols, eps, x, gamma, beta, y, stats, hip_stream);
}
dp_status dp_op_rmsnorm_bwd(int32_t dtype, int32_t rows, int32_t cols, const void *dy, const void *x,
                            const float *stats, const void *gamma, const void *dres, void *dx, void *dgamma,
                            void *dbeta, void *dx_colsum, void *ws, void *hip_stream) {
  return norm_bwd(true, dtype, rows, cols, dy, x, stats, gamma, dres, dx, dgamma, dbeta, dx_colsum, ws, hip_stream);
}

dp_status dp_op_gelu_fwd(int32_t dtype, int32_t gelu_kind, size_t n, const void *x, void *y, void *hip_stream) {
  if (bad_dtype(dtype) || (n > 0 && (!x || !y)) || (gelu_kind < 0 || gelu_kind > 2)) return fail(DP_E_INVAL, "gelu_fwd: bad argument");
  if (n % 8) return fail(DP_E_UNSUPPORTED, "gelu: n must be a multiple of 8");
  return op_done(dp::launch_gelu_fwd(dtype, gelu_kind, n, x, y, (hipStream_t)hip_stream), "gelu_fwd");
}

dp_status dp_op_gelu_bwd(int32_t dtype, int32_t gelu_kind, int32_t rows, int32_t cols, const void *dy, const void *x,
                         void *dx, void *dbias, void *ws, void *hip_stream) {
  if (bad_dtype(dtype) || rows < 0 || cols <= 0 || !dbias || (rows > 0 && (!x || !dy || !dx || !ws)) ||
      (gelu_kind < 0 || gelu_kind > 2))
    return fail(DP_E_INVAL, "gelu_bwd: bad argument");
  if (cols % 8) return fail(DP_E_UNSUPPORTED, "gelu: cols must be a multiple of 8");
  return op_done(dp::launch_gelu_bwd_colsum(dtype, gelu_kind, rows, cols, dy, x, dx, dbias, ws,
                                            (hipStream_t)hip_stream), "gelu_bwd");
}

dp_status dp_op_gemm(int32_t dtype, int32_t mode, int32_t M, int32_t N, int32_t K, const void *A, const void *B,
                     const void *bias, const void *res, void *C, void *hip_stream) {
  if (bad_dtype(dtype) || (mode != 0 && mode != 1) || M < 0 || N < 0 || K < 0)
    return fail(DP_E_INVAL, "gemm: bad argument");
  if (M == 0 || N == 0) return DP_OK;                        // no output element
  if (!C || (K > 0 && (!A || !B))) return fail(DP_E_INVAL, "gemm: null operand");   // (K = 0: C = bias + res)
  dp::GemmArgs a{mode, M, N, K, A, B, bias, res, C};
  const bool simple = !env_mfma_enabled();
  if (dtype == DP_BF16 && !simple && dp::gemm_mfma_supported(a))
    return op_done(dp::launch_gemm_mfma(a, (hipStream_t)hip_stream), "gemm");
  return op_done(dp::launch_gemm_simple(dtype, a, (hipStream_t)hip_stream), "gemm");
}

dp_status dp_op_colsum(int32_t dtype, int32_t rows, int32_t cols, const void *x, void *out, void *ws,
                       void *hip_stream) {
  if (bad_dtype(dtype) || rows < 0 || cols <= 0 || !out || (rows > 0 && (!x || !ws))) return fail(DP_E_INVAL, "colsum: bad argument");
  if (cols % 8) return fail(DP_E_UNSUPPORTED, "colsum: cols must be a multiple of 8");
  return op_done(dp::launch_colsum(dtype, rows, cols, x, out, ws, (hipStream_t)hip_stream), "colsum");
}

dp_status dp_op_colsum_static(int32_t dtype, int32_t rows, int32_t cols, const void *x, void *out, void *hip_stream) {
  if (bad_dtype(dtype) || rows < 0 || cols <= 0 || !out || (rows > 0 && !x)) return fail(DP_E_INVAL, "colsum_static: bad argument");
  if (cols % 8) return fail(DP_E_UNSUPPORTED, "colsum: cols must be a multiple of 8");
  const size_t need = dp::colsum_static_needed_bytes(rows, cols);
  if (need > dp::colsum_static_max_bytes())
    return fail(DP_E_UNSUPPORTED, "colsum_static: [%d, %d] needs %zu bytes of partial sums, the library's static scratch "
                "array holds %zu (use dp_op_colsum with a workspace)", rows, cols, need, dp::colsum_static_max_bytes());
  return op_done(dp::launch_colsum_static(dtype, rows, cols, x, out, (hipStream_t)hip_stream), "colsum_static");
}

dp_status dp_op_attention_fwd(int32_t dtype, int32_t B, int32_t S, int32_t nh, int32_t dh, int32_t causal,
                              const void *qkv, void *o, float *lse, void *hip_stream) {
  if (bad_dtype(dtype) || B < 0 || S < 0 || nh <= 0 || dh <= 0 || ((long)B * S > 0 && !qkv)) return fail(DP_E_INVAL, "attention_fwd: bad argument");
  if (dh % 8) return fail(DP_E_UNSUPPORTED, "attention: head_dim must be a multiple of 8");
  const bool simple = !env_mfma_enabled();
  if (dtype == DP_BF16 && !simple && dp::attn_mfma_supported(S, dh))
    return op_done(dp::launch_attn_fwd_mfma(B, S, nh, dh, causal, qkv, o, lse, (hipStream_t)hip_stream), "attention_fwd");
  if (S > 4096) return fail(DP_E_UNSUPPORTED, "attention: seq > 4096 needs the MFMA path");
  return op_done(dp::launch_attn_fwd_simple(dtype, B, S, nh, dh, causal, qkv, o, lse, (hipStream_t)hip_stream),
                 "attention_fwd");
}

dp_status dp_op_attention_bwd(int32_t dtype, int32_t B, int32_t S, int32_t nh, int32_t dh, int32_t causal,
                              const void *qkv, const void *o, const float *lse, const void *d_o, void *dqkv, void *ws,
                              void *hip_stream) {
  if (bad_dtype(dtype) || B < 0 || S < 0 || nh <= 0 || dh <= 0 || ((long)B * S > 0 && (!qkv || !o || !lse || !d_o || !dqkv || !ws)))
    return fail(DP_E_INVAL, "attention_bwd: bad argument");
  if (dh % 8) return fail(DP_E_UNSUPPORTED, "attention: head_dim must be a multiple of 8");
  const bool simple = !env_mfma_enabled();
  if (dtype == DP_BF16 && !simple && dp::attn_mfma_supported(S, dh))
    return op_done(dp::launch_attn_bwd_mfma(B, S, nh, dh, causal, qkv, o, lse, d_o, dqkv, (float *)ws,
                                            (hipStream_t)hip_stream), "attention_bwd");
  if (S > 4096) return fail(DP_E_UNSUPPORTED, "attention: seq > 4096 needs the MFMA path");
  return op_done(dp::launch_attn_bwd_simple(dtype, B, S, nh, dh, causal, qkv, o, lse, d_o, dqkv, (float *)ws,
                                            (hipStream_t)hip_stream), "attention_bwd");
}

// ---- dropout forms of the standalone operations
static dp_status drop_args_of(const dp_dropout *d, int site, dp::DropArgs *out) {
  if (d == nullptr) return fail(DP_E_INVAL, "dropout description is null");
  if (!(d->p >= 0.f && d->p < 1.f)) return fail(DP_E_INVAL, "dropout rate must be in [0, 1)");
  if (d->layer < 0) return fail(DP_E_INVAL, "dropout layer must be >= 0");
  *out = dp::make_drop_args(d->seed, d->micro_batch, d->layer, site, d->p);
  return DP_OK;
}

dp_status dp_op_dropout(int32_t dtype, size_t n, const void *x, const void *res, void *y, const dp_dropout *drop,
                        int32_t site, void *hip_stream) {
  if (bad_dtype(dtype) || !x || !y || (site != dp::kSiteProj && site != dp::kSiteFc2 && site != dp::kSiteCrossProj))
    return fail(DP_E_INVAL, "dropout: bad argument");
  if (n % 8 || n >= ((size_t)1 << 32)) return fail(DP_E_UNSUPPORTED, "dropout: n must be a multiple of 8 below 2^32");
  dp::DropArgs a;
  const dp_status s = drop_args_of(drop, site, &a);
  if (s != DP_OK) return s;
  return op_done(dp::launch_dropout(dtype, n, x, res, y, a, (hipStream_t)hip_stream), "dropout");
}

dp_status dp_op_attention_dropout_fwd(int32_t dtype, int32_t B, int32_t S, int32_t nh, int32_t dh, int32_t causal,
                                      const void *qkv, void *o, float *lse, const dp_dropout *drop, void *hip_stream) {
  if (bad_dtype(dtype) || B < 0 || S < 0 || nh <= 0 || dh <= 0 || ((long)B * S > 0 && !qkv)) return fail(DP_E_INVAL, "attention_fwd: bad argument");
  if (dh % 8) return fail(DP_E_UNSUPPORTED, "attention: head_dim must be a multiple of 8");
  if ((long)S * S >= (1L << 32)) return fail(DP_E_UNSUPPORTED, "attention dropout needs seq*seq < 2^32");
  dp::DropArgs a;
  const dp_status st = drop_args_of(drop, dp::kSiteAttn, &a);
  if (st != DP_OK) return st;
  const bool simple = !env_mfma_enabled();
  if (dtype == DP_BF16 && !simple && dp::attn_mfma_supported(S, dh))
    return op_done(dp::launch_attn_fwd_mfma(B, S, nh, dh, causal, qkv, o, lse, (hipStream_t)hip_stream, &a),
                   "attention_fwd");
  if (S > 4096) return fail(DP_E_UNSUPPORTED, "attention: seq > 4096 needs the MFMA path");
  return op_done(dp::launch_attn_fwd_simple(dtype, B, S, nh, dh, causal, qkv, o, lse, (hipStream_t)hip_stream, &a),
                 "attention_fwd");
}

dp_status dp_op_attention_dropout_bwd(int32_t dtype, int32_t B, int32_t S, int32_t nh, int32_t dh, int32_t causal,
                                      const void *qkv, const void *o, const float *lse, const void *d_o, void *dqkv,
                                      void *ws, const dp_dropout *drop, void *hip_stream) {
  if (bad_dtype(dtype) || B < 0 || S < 0 || nh <= 0 || dh <= 0 || ((long)B * S > 0 && (!qkv || !o || !lse || !d_o || !dqkv || !ws)))
    return fail(DP_E_INVAL, "attention_bwd: bad argument");
  if (dh % 8) return fail(DP_E_UNSUPPORTED, "attention: head_dim must be a multiple of 8");
  if ((long)S * S >= (1L << 32)) return fail(DP_E_UNSUPPORTED, "attention dropout needs seq*seq < 2^32");
  dp::DropArgs a;
  const dp_status st = drop_args_of(drop, dp::kSiteAttn, &a);
  if (st != DP_OK) return st;
  const bool simple = !env_mfma_enabled();
  if (dtype == DP_BF16 && !simple && dp::attn_mfma_supported(S, dh))
    return op_done(dp::launch_attn_bwd_mfma(B, S, nh, dh, causal, qkv, o, lse, d_o, dqkv, (float *)ws,
                                            (hipStream_t)hip_stream, &a), "attention_bwd");
  if (S > 4096) return fail(DP_E_UNSUPPORTED, "attention: seq > 4096 needs the MFMA path");
  return op_done(dp::launch_attn_bwd_simple(dtype, B, S, nh, dh, causal, qkv, o, lse, d_o, dqkv, (float *)ws,
                                            (hipStream_t)hip_stream, &a), "attention_bwd");
}


// ---- cross-attention: queries from one tensor, keys and values from another
static dp_status cross_args(const char *what, int32_t dtype, int32_t B, int32_t Sq, int32_t Sk, int32_t nh, int32_t dh,
                            const dp_dropout *drop, dp::DropArgs *a, bool *dropping) {
  if (bad_dtype(dtype) || B < 0 || Sq < 0 || Sk < 0 || nh <= 0 || dh <= 0) return fail(DP_E_INVAL, "%s: bad argument", what);
  if (dh % 8) return fail(DP_E_UNSUPPORTED, "attention: head_dim must be a multiple of 8");
  if ((long)B * Sq > 0 && Sk == 0) return fail(DP_E_INVAL, "%s: a softmax over no keys is undefined", what);
  *dropping = drop != nullptr;
  if (drop != nullptr) {
    if ((long)Sq * Sk >= (1L << 32)) return fail(DP_E_UNSUPPORTED, "attention dropout needs Sq*Sk < 2^32");
    return drop_args_of(drop, dp::kSiteCross, a);
  }
  return DP_OK;
}

dp_status dp_op_cross_attention_fwd(int32_t dtype, int32_t B, int32_t Sq, int32_t Sk, int32_t nh, int32_t dh,
                                    const void *q, const void *kv, void *o, float *lse, const dp_dropout *drop,
                                    void *hip_stream) {
  dp::DropArgs a;
  bool dropping = false;
  const dp_status st = cross_args("cross_attention_fwd", dtype, B, Sq, Sk, nh, dh, drop, &a, &dropping);
  if (st != DP_OK) return st;
  if ((long)B * Sq == 0) return DP_OK;
  if (!q || !kv) return fail(DP_E_INVAL, "cross_attention_fwd: null operand");
  const long H = (long)nh * dh;
  const char *kvp = (const char *)kv;
  const dp::AttnView v{q, kvp, kvp + (size_t)H * dp::dtype_size(dtype), nullptr, nullptr, nullptr, H, 2 * H, Sq, Sk};
  const bool simple = !env_mfma_enabled();
  if (dtype == DP_BF16 && !simple && dp::attn_mfma_supported(Sk, dh))
    return op_done(dp::launch_attn_fwd_mfma_view(B, nh, dh, 0, v, o, lse, (hipStream_t)hip_stream, dropping ? &a : nullptr),
                   "cross_attention_fwd");
  if (Sq > 4096 || Sk > 4096) return fail(DP_E_UNSUPPORTED, "attention: more than 4096 rows needs the MFMA path");
  return op_done(dp::launch_attn_fwd_simple_view(dtype, B, nh, dh, 0, v, o, lse, (hipStream_t)hip_stream,
                                                 dropping ? &a : nullptr), "cross_attention_fwd");
}

dp_status dp_op_cross_attention_bwd(int32_t dtype, int32_t B, int32_t Sq, int32_t Sk, int32_t nh, int32_t dh,
                                    const void *q, const void *kv, const void *o, const float *lse, const void *d_o,
                                    void *dq, void *dkv, void *ws, const dp_dropout *drop, void *hip_stream) {
  dp::DropArgs a;
  bool dropping = false;
  const dp_status st = cross_args("cross_attention_bwd", dtype, B, Sq, Sk, nh, dh, drop, &a, &dropping);
  if (st != DP_OK) return st;
  if ((long)B * Sq > 0 && (!q || !o || !lse || !d_o || !dq || !ws)) return fail(DP_E_INVAL, "cross_attention_bwd: null operand");
  if ((long)B * Sk > 0 && (!kv || !dkv)) return fail(DP_E_INVAL, "cross_attention_bwd: null operand");
  const long H = (long)nh * dh;
  const size_t hb = (size_t)H * dp::dtype_size(dtype);
  const char *kvp = (const char *)kv;
  char *dkvp = (char *)dkv;
  const dp::AttnView v{q, kvp, kvp ? kvp + hb : nullptr, dq, dkvp, dkvp ? dkvp + hb : nullptr, H, 2 * H, Sq, Sk};
  const bool simple = !env_mfma_enabled();
  if (dtype == DP_BF16 && !simple && dp::attn_mfma_supported(std::max(Sk, 1), dh))
    return op_done(dp::launch_attn_bwd_mfma_view(B, nh, dh, 0, v, o, lse, d_o, (float *)ws, (hipStream_t)hip_stream,
                                                 dropping ? &a : nullptr), "cross_attention_bwd");
  if (Sq > 4096 || Sk > 4096) return fail(DP_E_UNSUPPORTED, "attention: more than 4096 rows needs the MFMA path");
  return op_done(dp::launch_attn_bwd_simple_view(dtype, B, nh, dh, 0, v, o, lse, d_o, (float *)ws, (hipStream_t)hip_stream,
                                                 dropping ? &a : nullptr), "cross_attention_bwd");
}


dp_status dp_probe_mfma(const void *data_bf16, size_t n_elems, int32_t iters, float *tflops, float *shader_mhz,
                        void *hip_stream) {
  if (!data_bf16 || n_elems < 8 || n_elems % 8 || iters < 1 || !tflops || !shader_mhz)
    return fail(DP_E_INVAL, "probe_mfma: bad argument");
  int dev = 0, cus = 0;
  HIP_TRY(hipGetDevice(&dev), DP_E_HIP);
  HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev), DP_E_HIP);
  *tflops = 0.f; *shader_mhz = 0.f;
  return op_done(dp::run_mfma_probe(data_bf16, n_elems, iters, cus, tflops, shader_mhz, (hipStream_t)hip_stream),
                 "probe_mfma");
}

}  // extern "C"
