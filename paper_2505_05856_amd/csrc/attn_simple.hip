// Plain softmax attention on the vector ALUs, one wavefront per query row
// (forward, dQ) or per key row (dK, dV).  This is the fp32 debug mode's
// attention and the fallback for shapes the MFMA kernels do not take.
// Scores of one row live in LDS (4 bytes x S per wave), so S <= 4096.
// Operands come through an AttnView: Sq queries from one tensor, Sk keys and values from
// another (the same packed tensor for self-attention).
// Dropout (da.thr != 0): element (i, j) of head (b, h) is kept when
// drop_bits(i*Sk + j, keys of unit b*nh + h) >= da.thr; kept probabilities are scaled by
// da.scale after the softmax, and the backward masks and scales dP the same way.
#include "common.h"
#include "kernels.h"

namespace dp {

template <typename T>
__device__ __forceinline__ float dot_row(const float *__restrict__ qs, const T *__restrict__ p, int dh) {
  float s = 0.f;
  for (int d = 0; d < dh; d += 8) {
    float v[8];
    load8(p + d, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) s += qs[d + i] * v[i];
  }
  return s;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_simple_kernel(AttnView av, T *__restrict__ o,
                                                              float *__restrict__ lse, int B, int nh, int dh,
                                                              int causal, float scale, DropArgs da) {
  extern __shared__ float smem[];
  const int Sq = av.Sq, S = av.Sk;   // S: the key count
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float *sc = smem + (size_t)wave * (S + dh);
  float *qs = sc + S;
  long row_id = (long)blockIdx.x * 4 + wave;  // (b, h, i)
  const bool active = row_id < (long)B * nh * Sq;  // inactive waves still reach every barrier
  if (!active) row_id = 0;
  const int i = (int)(row_id % Sq);
  const int h = (int)((row_id / Sq) % nh);
  const int b = (int)(row_id / ((long)Sq * nh));
  const int H = nh * dh;
  const size_t ldq = (size_t)av.ldq, ld = (size_t)av.ldkv;
  const T *qrow = (const T *)av.q + ((size_t)b * Sq + i) * ldq + (size_t)h * dh;
  const T *kbase = (const T *)av.k + (size_t)b * S * ld + (size_t)h * dh;
  const T *vbase = (const T *)av.v + (size_t)b * S * ld + (size_t)h * dh;
  for (int d = lane; d < dh; d += 64) qs[d] = ldf(qrow + d);
  __syncthreads();
  const int jn = !active ? 0 : causal ? i + 1 : S;
  float m = -INFINITY;
  for (int j = lane; j < jn; j += 64) {
    const float s = scale * dot_row(qs, kbase + (size_t)j * ld, dh);
    sc[j] = s;
    m = fmaxf(m, s);
  }
  m = wave_max(m);
  float l = 0.f;
  for (int j = lane; j < jn; j += 64) {
    const float p = expf(sc[j] - m);
    sc[j] = p;
    l += p;
  }
  l = wave_sum(l);
  if (da.thr != 0) {
    const DropKeys keys = drop_keys(da.base, (uint32_t)(b * nh + h));
    for (int j = lane; j < jn; j += 64)
      if (drop_bits((uint32_t)i * (uint32_t)S + (uint32_t)j, keys.k0, keys.k1) < da.thr) sc[j] = 0.f;
  }
  __syncthreads();
  if (!active) return;
  if (lse != nullptr && lane == 0) lse[((size_t)b * nh + h) * Sq + i] = m + logf(l);
  if (o == nullptr) return;
  const float inv = da.scale / l;
  for (int d = lane; d < dh; d += 64) {
    float acc = 0.f;
    const T *v = vbase + d;
    for (int j = 0; j < jn; ++j) acc += sc[j] * ldf(v + (size_t)j * ld);
    stf(o + ((size_t)b * Sq + i) * H + (size_t)h * dh + d, acc * inv);
  }
}

// Per query row i: D_i = <dO_i, O_i>; dS_ij = P_ij (dP_ij - D_i); dQ_i = scale * sum_j dS_ij K_j.
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_simple_kernel(AttnView av, const T *__restrict__ o,
                                                                 const float *__restrict__ lse,
                                                                 const T *__restrict__ d_o,
                                                                 float *__restrict__ drow, int B, int nh,
                                                                 int dh, int causal, float scale, DropArgs da) {
  extern __shared__ float smem[];
  const int Sq = av.Sq, S = av.Sk;   // S: the key count
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float *sc = smem + (size_t)wave * (S + 2 * dh);
  float *qs = sc + S;
  float *dos = qs + dh;
  long row_id = (long)blockIdx.x * 4 + wave;
  const bool active = row_id < (long)B * nh * Sq;
  if (!active) row_id = 0;
  const int i = (int)(row_id % Sq);
  const int h = (int)((row_id / Sq) % nh);
  const int b = (int)(row_id / ((long)Sq * nh));
  const int H = nh * dh;
  const size_t ldq = (size_t)av.ldq, ld = (size_t)av.ldkv;
  const size_t qoff = ((size_t)b * Sq + i) * ldq + (size_t)h * dh;
  const T *kbase = (const T *)av.k + (size_t)b * S * ld + (size_t)h * dh;
  const T *vbase = (const T *)av.v + (size_t)b * S * ld + (size_t)h * dh;
  const size_t orow = ((size_t)b * Sq + i) * H + (size_t)h * dh;
  float dsum = 0.f;
  for (int d = lane; d < dh; d += 64) {
    qs[d] = ldf((const T *)av.q + qoff + d);
    const float g = ldf(d_o + orow + d);
    dos[d] = g;
    dsum += g * ldf(o + orow + d);
  }
  dsum = wave_sum(dsum);
  __syncthreads();
  const float L = lse[((size_t)b * nh + h) * Sq + i];
  if (active && lane == 0) drow[((size_t)b * nh + h) * Sq + i] = dsum;
  const int jn = !active ? 0 : causal ? i + 1 : S;
  const DropKeys keys = drop_keys(da.base, (uint32_t)(b * nh + h));
  for (int j = lane; j < jn; j += 64) {
    const float p = expf(scale * dot_row(qs, kbase + (size_t)j * ld, dh) - L);
    float dp = dot_row(dos, vbase + (size_t)j * ld, dh);
    if (da.thr != 0)
      dp = drop_bits((uint32_t)i * (uint32_t)S + (uint32_t)j, keys.k0, keys.k1) >= da.thr ? dp * da.scale : 0.f;
    sc[j] = p * (dp - dsum);
  }
  __syncthreads();
  if (!active) return;
  for (int d = lane; d < dh; d += 64) {
    float acc = 0.f;
    const T *k = kbase + d;
    for (int j = 0; j < jn; ++j) acc += sc[j] * ldf(k + (size_t)j * ld);
    stf((T *)av.dq + qoff + d, acc * scale);
  }
}

// Per key row j: dV_j = sum_i P_ij dO_i; dK_j = scale * sum_i dS_ij Q_i.
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_simple_kernel(AttnView av,
                                                                  const float *__restrict__ lse,
                                                                  const T *__restrict__ d_o,
                                                                  const float *__restrict__ drow,
                                                                  int B, int nh, int dh,
                                                                  int causal, float scale, DropArgs drop) {
  extern __shared__ float smem[];
  const int S = av.Sq, Sk = av.Sk;   // S: the query count, which bounds the loops over i below
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float *pa = smem + (size_t)wave * (2 * S + 2 * dh);
  float *da = pa + S;
  float *ks = da + S;
  float *vs = ks + dh;
  long row_id = (long)blockIdx.x * 4 + wave;
  const bool active = row_id < (long)B * nh * Sk;
  if (!active) row_id = 0;
  const int j = (int)(row_id % Sk);
  const int h = (int)((row_id / Sk) % nh);
  const int b = (int)(row_id / ((long)Sk * nh));
  const int H = nh * dh;
  const size_t ld = (size_t)av.ldq, ldkv = (size_t)av.ldkv;
  const T *base = (const T *)av.q + (size_t)b * S * ld + (size_t)h * dh;
  const T *dob = d_o + (size_t)b * S * H + (size_t)h * dh;
  const size_t koff = ((size_t)b * Sk + j) * ldkv + (size_t)h * dh;
  for (int d = lane; d < dh; d += 64) {
    ks[d] = ldf((const T *)av.k + koff + d);
    vs[d] = ldf((const T *)av.v + koff + d);
  }
  __syncthreads();
  const int i0 = !active ? S : causal ? j : 0;
  const float *Lr = lse + ((size_t)b * nh + h) * S;
  const float *Dr = drow + ((size_t)b * nh + h) * S;
  const DropKeys keys = drop_keys(drop.base, (uint32_t)(b * nh + h));
  for (int i = i0 + lane; i < S; i += 64) {
    const float p = expf(scale * dot_row(ks, base + (size_t)i * ld, dh) - Lr[i]);
    float dp = dot_row(vs, dob + (size_t)i * H, dh);
    float pv = p;   // what multiplied V in the forward
    if (drop.thr != 0) {
      const bool keep = drop_bits((uint32_t)i * (uint32_t)Sk + (uint32_t)j, keys.k0, keys.k1) >= drop.thr;
      pv = keep ? p * drop.scale : 0.f;
      dp = keep ? dp * drop.scale : 0.f;
    }
    pa[i] = pv;
    da[i] = p * (dp - Dr[i]);
  }
  __syncthreads();
  if (!active) return;
  for (int d = lane; d < dh; d += 64) {
    float acc_v = 0.f, ak = 0.f;
    for (int i = i0; i < S; ++i) {
      acc_v += pa[i] * ldf(dob + (size_t)i * H + d);
      ak += da[i] * ldf(base + (size_t)i * ld + d);
    }
    stf((T *)av.dk + koff + d, ak * scale);
    stf((T *)av.dv + koff + d, acc_v);
  }
}

template <typename T>
static hipError_t fwd_t(int B, int nh, int dh, int causal, const AttnView &v, void *o, float *lse, const DropArgs &da,
                        hipStream_t s) {
  const long rows = (long)B * nh * v.Sq;
  const size_t smem = 4 * (size_t)(v.Sk + dh) * sizeof(float);
  hipLaunchKernelGGL((attn_fwd_simple_kernel<T>), dim3((unsigned)((rows + 3) / 4)), dim3(256), smem, s, v, (T *)o, lse,
                     B, nh, dh, causal, 1.0f / sqrtf((float)dh), da);
  return hipGetLastError();
}

hipError_t launch_attn_fwd_simple_view(int dtype, int B, int nh, int dh, int causal, const AttnView &v, void *o,
                                       float *lse, hipStream_t s, const DropArgs *drop) {
  if (causal && v.Sq != v.Sk) return hipErrorInvalidValue;
  if ((long)B * v.Sq * nh == 0) return hipSuccess;
  const DropArgs da = drop != nullptr && drop->thr != 0 ? *drop : DropArgs{0u, 0u, 1.f};
  return dtype == kBF16 ? fwd_t<bf16>(B, nh, dh, causal, v, o, lse, da, s)
                        : fwd_t<float>(B, nh, dh, causal, v, o, lse, da, s);
}

template <typename T>
static hipError_t bwd_t(int B, int nh, int dh, int causal, const AttnView &v, const void *o, const float *lse,
                        const void *d_o, float *ws, const DropArgs &da, hipStream_t s) {
  const long qrows = (long)B * nh * v.Sq, krows = (long)B * nh * v.Sk;
  const float scale = 1.0f / sqrtf((float)dh);
  const dim3 block(256);
  if (qrows > 0 && v.Sk > 0) {
    hipLaunchKernelGGL((attn_bwd_dq_simple_kernel<T>), dim3((unsigned)((qrows + 3) / 4)), block,
                       4 * (size_t)(v.Sk + 2 * dh) * sizeof(float), s, v, (const T *)o, lse, (const T *)d_o, ws, B, nh,
                       dh, causal, scale, da);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (krows > 0)   // (no queries: dK = dV = 0 is still written)
    hipLaunchKernelGGL((attn_bwd_dkv_simple_kernel<T>), dim3((unsigned)((krows + 3) / 4)), block,
                       4 * (size_t)(2 * v.Sq + 2 * dh) * sizeof(float), s, v, lse, (const T *)d_o, ws, B, nh, dh, causal,
                       scale, da);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_simple_view(int dtype, int B, int nh, int dh, int causal, const AttnView &v, const void *o,
                                       const float *lse, const void *d_o, float *ws, hipStream_t s,
                                       const DropArgs *drop) {
  if (causal && v.Sq != v.Sk) return hipErrorInvalidValue;
  if ((long)B * nh == 0) return hipSuccess;
  const DropArgs da = drop != nullptr && drop->thr != 0 ? *drop : DropArgs{0u, 0u, 1.f};
  return dtype == kBF16 ? bwd_t<bf16>(B, nh, dh, causal, v, o, lse, d_o, ws, da, s)
                        : bwd_t<float>(B, nh, dh, causal, v, o, lse, d_o, ws, da, s);
}

hipError_t launch_attn_fwd_simple(int dtype, int B, int S, int nh, int dh, int causal, const void *qkv, void *o,
                                  float *lse, hipStream_t s, const DropArgs *drop) {
  return launch_attn_fwd_simple_view(dtype, B, nh, dh, causal, attn_self_view(qkv, nullptr, S, nh * dh, dtype_size(dtype)),
                                     o, lse, s, drop);
}

hipError_t launch_attn_bwd_simple(int dtype, int B, int S, int nh, int dh, int causal, const void *qkv,
                                  const void *o, const float *lse, const void *d_o, void *dqkv, float *ws,
                                  hipStream_t s, const DropArgs *drop) {
  return launch_attn_bwd_simple_view(dtype, B, nh, dh, causal, attn_self_view(qkv, dqkv, S, nh * dh, dtype_size(dtype)),
                                     o, lse, d_o, ws, s, drop);
}

}  // namespace dp
