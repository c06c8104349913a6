// Internal launcher interface between the step executor and the HIP kernels.
// Every launcher enqueues on `s` and returns hipGetLastError(); none waits.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace dp {

// ---- dropout masks ------------------------------------------------------------
// What a kernel needs to draw one site's mask (the generator is described in common.h).
// thr == 0 keeps everything.
struct DropArgs {
  uint32_t base;    // of (seed, micro-batch, layer, site)
  uint32_t thr;     // floor(p * 2^32)
  float scale;      // 1 / (1 - p)
};
// (up to eight sites a layer: the key chain takes 8 * layer + site)
enum DropSite { kSiteAttn = 0, kSiteProj = 1, kSiteFc2 = 2, kSiteCross = 3, kSiteCrossProj = 4 };
inline uint32_t drop_mix_host(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
inline DropArgs make_drop_args(uint64_t seed, uint64_t mb, int layer, int site, float p) {
  uint32_t s = drop_mix_host((uint32_t)seed ^ 0x9e3779b9u);
  s = drop_mix_host(s ^ (uint32_t)(seed >> 32));
  s = drop_mix_host(s ^ (uint32_t)mb);
  s = drop_mix_host(s ^ (uint32_t)(mb >> 32));
  s = drop_mix_host(s ^ (uint32_t)(8 * layer + site));
  DropArgs a;
  a.base = s;
  a.thr = (uint32_t)((double)p * 4294967296.0);   // p < 1: the product is below 2^32; the cast truncates
  a.scale = 1.0f / (1.0f - p);
  return a;
}


enum { kF32 = 0, kBF16 = 1 };
enum { kGemmNT = 0, kGemmTN = 1 };

inline size_t dtype_size(int dtype) { return dtype == kBF16 ? 2 : 4; }

// Upper bound of row-blocks used by the two-pass column reductions.
constexpr int kMaxRowBlocks = 512;
// Row blocks of a two-pass column reduction: at least `min_rows` rows a block, at
// most kMaxRowBlocks blocks.  Returns the block count, *rpb = rows per block.
inline int row_blocks(int rows, int min_rows, int *rpb) {
  int nb = (rows + min_rows - 1) / min_rows;
  if (nb > kMaxRowBlocks) nb = kMaxRowBlocks;
  if (nb < 1) nb = 1;
  *rpb = (rows + nb - 1) / nb;
  return (rows + *rpb - 1) / *rpb;
}
// Bytes of fp32 partials a column reduction over [rows, cols] needs (x3: LayerNorm
// backward reduces up to three vectors at once).
inline size_t reduce_ws_bytes(int rows, int cols) {
  int rpb;
  return (size_t)row_blocks(rows, 8, &rpb) * 3 * (size_t)cols * sizeof(float);
}

struct GemmArgs {
  int mode;            // kGemmNT: A [M,K], B [N,K];  kGemmTN: A [K,M], B [K,N]
  int M, N, K;
  const void *A, *B;
  const void *bias;    // [N] or null
  const void *res;     // [M,N] or null, added after bias
  void *C;             // [M,N]
  // optional second output (MFMA path only): C2[m,n] = gelu(C[m,n] as stored), gelu_kind 0 erf / 1 tanh
  void *C2 = nullptr;
  int gelu_kind = 0;
};

// ---- shape support (host checks; the launchers assume they passed) ----------
bool ln_supported(int dtype, int cols);                 // cols % 8 == 0, cols <= 8192
bool gemm_mfma_supported(const GemmArgs &a);            // bf16 MFMA path preconditions
bool attn_mfma_supported(int S, int dh);

// ---- elementwise / reductions ----------------------------------------------
// Second pass of a two-pass column reduction: out[j / seg][j % seg] = sum over the nb
// partial rows of part[.][j], j < width, in a fixed order.  The launchers below run it
// themselves unless they are handed a ReduceJob to fill in: then the caller runs it later
// with launch_reduce_jobs (several jobs in one launch; same arithmetic, same bits).
struct ReduceJob {
  const float *part;
  int nb, width, seg;
  void *out0, *out1, *out2;
  int accumulate = 0;   // add to what the outputs hold instead of overwriting (batched launch only)
};
constexpr int kMaxReduceJobs = 8;
hipError_t launch_reduce_jobs(int dtype, const ReduceJob *jobs, int n, hipStream_t s);

hipError_t launch_ln_fwd(int dtype, int rows, int cols, float eps, const void *x, const void *gamma,
                         const void *beta, void *y, float *stats, hipStream_t s, bool rms = false);
// dxsum (nullable): receives the column sums of the stored dx
hipError_t launch_ln_bwd(int dtype, int rows, int cols, const void *dy, const void *x, const float *stats,
                         const void *gamma, const void *dres, void *dx, void *dgamma, void *dbeta, void *dxsum,
                         void *ws, hipStream_t s, ReduceJob *job = nullptr, bool rms = false);
// (rms: RMSNorm, i.e. no mean is subtracted; same kernels, see elementwise.hip)
// dx = dy * gelu'(x) over [rows, cols] and dbias = column sums of the stored dx
hipError_t launch_gelu_bwd_colsum(int dtype, int kind, int rows, int cols, const void *dy, const void *x, void *dx,
                                  void *dbias, void *ws, hipStream_t s, ReduceJob *job = nullptr);
// y = (res ? res : 0) + keep * scale * x, n a multiple of 8 and below 2^32; x and res may be y
hipError_t launch_dropout(int dtype, size_t n, const void *x, const void *res, void *y, const DropArgs &a,
                          hipStream_t s);
hipError_t launch_gelu_fwd(int dtype, int kind, size_t n, const void *x, void *y, hipStream_t s);
hipError_t launch_colsum(int dtype, int rows, int cols, const void *x, void *out, void *ws, hipStream_t s,
                         ReduceJob *job = nullptr);
// The same with the partial sums in a device array of the library's own (no workspace, no
// allocation); the caller checks colsum_static_needed_bytes(...) <= colsum_static_max_bytes().
size_t colsum_static_max_bytes();
size_t colsum_static_needed_bytes(int rows, int cols);
hipError_t launch_colsum_static(int dtype, int rows, int cols, const void *x, void *out, hipStream_t s);
// dst[c, r] = src[r, c]
hipError_t launch_transpose(int dtype, int rows, int cols, const void *src, void *dst, hipStream_t s);
hipError_t launch_fill_u32(void *p, size_t n_words, uint32_t pattern, hipStream_t s);

// ---- GEMM -------------------------------------------------------------------
hipError_t launch_gemm_simple(int dtype, const GemmArgs &a, hipStream_t s);
hipError_t launch_gemm_mfma(const GemmArgs &a, hipStream_t s);   // bf16 only
// kernels with LDS-direct operand loads; launch_gemm_mfma routes to them when the shape is supported
bool gemm_dma_supported(const GemmArgs &a);
hipError_t launch_gemm_dma(const GemmArgs &a, hipStream_t s);

// ---- attention ----------------------------------------------------------------
// qkv [T,3H]; o [T,H] (nullable); lse [B,nh,S] fp32 (nullable); drop: dropout of the
// probabilities (null or thr == 0: none; needs S*S < 2^32)
hipError_t launch_attn_fwd_simple(int dtype, int B, int S, int nh, int dh, int causal, const void *qkv, void *o,
                                  float *lse, hipStream_t s, const DropArgs *drop = nullptr);
// ws: fp32 [T, nh] row dots D_i = <dO_i, O_i>
hipError_t launch_attn_bwd_simple(int dtype, int B, int S, int nh, int dh, int causal, const void *qkv,
                                  const void *o, const float *lse, const void *d_o, void *dqkv, float *ws,
                                  hipStream_t s, const DropArgs *drop = nullptr);
hipError_t launch_attn_fwd_mfma(int B, int S, int nh, int dh, int causal, const void *qkv, void *o, float *lse,
                                hipStream_t s, const DropArgs *drop = nullptr);
hipError_t launch_attn_bwd_mfma(int B, int S, int nh, int dh, int causal, const void *qkv, const void *o,
                                const float *lse, const void *d_o, void *dqkv, float *ws, hipStream_t s,
                                const DropArgs *drop = nullptr);

// Where an attention call's operands live.  Each is a row-major matrix with one row per token
// and head h's dh columns at column h*dh; sample b's rows start at row b*Sq (queries, O, dO,
// dQ, and [B,nh,Sq] for lse) or b*Sk (keys, values, dK, dV).  Self-attention over a packed
// [T,3H] tensor is the case k = q + H, v = q + 2H, ldq = ldkv = 3H, Sq = Sk; cross-attention
// takes its queries from one tensor and keys and values from another of a different length.
struct AttnView {
  const void *q, *k, *v;
  void *dq, *dk, *dv;   // backward only; laid out like q, k, v
  long ldq, ldkv;       // row strides in elements
  int Sq, Sk;
};
inline AttnView attn_self_view(const void *qkv, void *dqkv, int S, int H, size_t esz) {
  const char *p = (const char *)qkv;
  char *g = (char *)dqkv;
  const size_t h = (size_t)H * esz;
  return AttnView{p, p ? p + h : nullptr, p ? p + 2 * h : nullptr, g, g ? g + h : nullptr, g ? g + 2 * h : nullptr,
                  3L * H, 3L * H, S, S};
}
// The same kernels on a view; causal needs Sq == Sk.  Dropout positions are query*Sk + key.
hipError_t launch_attn_fwd_simple_view(int dtype, int B, int nh, int dh, int causal, const AttnView &v, void *o,
                                       float *lse, hipStream_t s, const DropArgs *drop = nullptr);
hipError_t launch_attn_bwd_simple_view(int dtype, int B, int nh, int dh, int causal, const AttnView &v, const void *o,
                                       const float *lse, const void *d_o, float *ws, hipStream_t s,
                                       const DropArgs *drop = nullptr);
hipError_t launch_attn_fwd_mfma_view(int B, int nh, int dh, int causal, const AttnView &v, void *o, float *lse,
                                     hipStream_t s, const DropArgs *drop = nullptr);
hipError_t launch_attn_bwd_mfma_view(int B, int nh, int dh, int causal, const AttnView &v, const void *o,
                                     const float *lse, const void *d_o, float *ws, hipStream_t s,
                                     const DropArgs *drop = nullptr);

// ---- diagnostics --------------------------------------------------------------
// Matrix-core issue rate with operand fragments taken from `data` (bf16, n_elems >= 8); waits.
hipError_t run_mfma_probe(const void *data, size_t n_elems, int iters, int n_cus, float *tflops, float *shader_mhz,
                          hipStream_t s);

}  // namespace dp
