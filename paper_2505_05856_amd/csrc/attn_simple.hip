// Plain softmax attention on the vector ALUs, one wavefront per query row
// (forward, dQ) or per key row (dK, dV).  This is the fp32 debug mode's
// attention and the fallback for shapes the MFMA kernels do not take.
// Scores of one row live in LDS (4 bytes x S per wave), so S <= 4096.
// Dropout (da.thr != 0): element (i, j) of head (b, h) is kept when
// drop_bits(i*S + j, keys of unit b*nh + h) >= da.thr; kept probabilities are scaled by
// da.scale after the softmax, and the backward masks and scales dP the same way.
#include "common.h"
#include "kernels.h"

namespace dp {

// qkv row t: [Q(0..H) | K(H..2H) | V(2H..3H)], head h at columns h*dh.
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
__global__ __launch_bounds__(256) void attn_fwd_simple_kernel(const T *__restrict__ qkv, T *__restrict__ o,
                                                              float *__restrict__ lse, int B, int S, int nh, int dh,
                                                              int causal, float scale, DropArgs da) {
  extern __shared__ float smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float *sc = smem + (size_t)wave * (S + dh);
  float *qs = sc + S;
  long row_id = (long)blockIdx.x * 4 + wave;  // (b, h, i)
  const bool active = row_id < (long)B * nh * S;  // inactive waves still reach every barrier
  if (!active) row_id = 0;
  const int i = (int)(row_id % S);
  const int h = (int)((row_id / S) % nh);
  const int b = (int)(row_id / ((long)S * nh));
  const int H = nh * dh;
  const size_t ld = 3 * (size_t)H;
  const T *base = qkv + (size_t)b * S * ld + (size_t)h * dh;
  for (int d = lane; d < dh; d += 64) qs[d] = ldf(base + (size_t)i * ld + d);
  __syncthreads();
  const int jn = !active ? 0 : causal ? i + 1 : S;
  float m = -INFINITY;
  for (int j = lane; j < jn; j += 64) {
    const float s = scale * dot_row(qs, base + (size_t)j * ld + H, dh);
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
  if (lse != nullptr && lane == 0) lse[((size_t)b * nh + h) * S + i] = m + logf(l);
  if (o == nullptr) return;
  const float inv = da.scale / l;
  for (int d = lane; d < dh; d += 64) {
    float acc = 0.f;
    const T *v = base + 2 * (size_t)H + d;
    for (int j = 0; j < jn; ++j) acc += sc[j] * ldf(v + (size_t)j * ld);
    stf(o + ((size_t)b * S + i) * H + (size_t)h * dh + d, acc * inv);
  }
}

// Per query row i: D_i = <dO_i, O_i>; dS_ij = P_ij (dP_ij - D_i); dQ_i = scale * sum_j dS_ij K_j.
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_simple_kernel(const T *__restrict__ qkv, const T *__restrict__ o,
                                                                 const float *__restrict__ lse,
                                                                 const T *__restrict__ d_o, T *__restrict__ dqkv,
                                                                 float *__restrict__ drow, int B, int S, int nh,
                                                                 int dh, int causal, float scale, DropArgs da) {
  extern __shared__ float smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float *sc = smem + (size_t)wave * (S + 2 * dh);
  float *qs = sc + S;
  float *dos = qs + dh;
  long row_id = (long)blockIdx.x * 4 + wave;
  const bool active = row_id < (long)B * nh * S;
  if (!active) row_id = 0;
  const int i = (int)(row_id % S);
  const int h = (int)((row_id / S) % nh);
  const int b = (int)(row_id / ((long)S * nh));
  const int H = nh * dh;
  const size_t ld = 3 * (size_t)H;
  const T *base = qkv + (size_t)b * S * ld + (size_t)h * dh;
  const size_t orow = ((size_t)b * S + i) * H + (size_t)h * dh;
  float dsum = 0.f;
  for (int d = lane; d < dh; d += 64) {
    qs[d] = ldf(base + (size_t)i * ld + d);
    const float g = ldf(d_o + orow + d);
    dos[d] = g;
    dsum += g * ldf(o + orow + d);
  }
  dsum = wave_sum(dsum);
  __syncthreads();
  const float L = lse[((size_t)b * nh + h) * S + i];
  if (active && lane == 0) drow[((size_t)b * nh + h) * S + i] = dsum;
  const int jn = !active ? 0 : causal ? i + 1 : S;
  const DropKeys keys = drop_keys(da.base, (uint32_t)(b * nh + h));
  for (int j = lane; j < jn; j += 64) {
    const float p = expf(scale * dot_row(qs, base + (size_t)j * ld + H, dh) - L);
    float dp = dot_row(dos, base + (size_t)j * ld + 2 * (size_t)H, dh);
    if (da.thr != 0)
      dp = drop_bits((uint32_t)i * (uint32_t)S + (uint32_t)j, keys.k0, keys.k1) >= da.thr ? dp * da.scale : 0.f;
    sc[j] = p * (dp - dsum);
  }
  __syncthreads();
  if (!active) return;
  for (int d = lane; d < dh; d += 64) {
    float acc = 0.f;
    const T *k = base + H + d;
    for (int j = 0; j < jn; ++j) acc += sc[j] * ldf(k + (size_t)j * ld);
    stf(dqkv + ((size_t)b * S + i) * ld + (size_t)h * dh + d, acc * scale);
  }
}

// Per key row j: dV_j = sum_i P_ij dO_i; dK_j = scale * sum_i dS_ij Q_i.
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_simple_kernel(const T *__restrict__ qkv,
                                                                  const float *__restrict__ lse,
                                                                  const T *__restrict__ d_o,
                                                                  const float *__restrict__ drow,
                                                                  T *__restrict__ dqkv, int B, int S, int nh, int dh,
                                                                  int causal, float scale, DropArgs drop) {
  extern __shared__ float smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float *pa = smem + (size_t)wave * (2 * S + 2 * dh);
  float *da = pa + S;
  float *ks = da + S;
  float *vs = ks + dh;
  long row_id = (long)blockIdx.x * 4 + wave;
  const bool active = row_id < (long)B * nh * S;
  if (!active) row_id = 0;
  const int j = (int)(row_id % S);
  const int h = (int)((row_id / S) % nh);
  const int b = (int)(row_id / ((long)S * nh));
  const int H = nh * dh;
  const size_t ld = 3 * (size_t)H;
  const T *base = qkv + (size_t)b * S * ld + (size_t)h * dh;
  const T *dob = d_o + (size_t)b * S * H + (size_t)h * dh;
  for (int d = lane; d < dh; d += 64) {
    ks[d] = ldf(base + (size_t)j * ld + H + d);
    vs[d] = ldf(base + (size_t)j * ld + 2 * (size_t)H + d);
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
      const bool keep = drop_bits((uint32_t)i * (uint32_t)S + (uint32_t)j, keys.k0, keys.k1) >= drop.thr;
      pv = keep ? p * drop.scale : 0.f;
      dp = keep ? dp * drop.scale : 0.f;
    }
    pa[i] = pv;
    da[i] = p * (dp - Dr[i]);
  }
  __syncthreads();
  if (!active) return;
  for (int d = lane; d < dh; d += 64) {
    float av = 0.f, ak = 0.f;
    for (int i = i0; i < S; ++i) {
      av += pa[i] * ldf(dob + (size_t)i * H + d);
      ak += da[i] * ldf(base + (size_t)i * ld + d);
    }
    stf(dqkv + ((size_t)b * S + j) * ld + H + (size_t)h * dh + d, ak * scale);
    stf(dqkv + ((size_t)b * S + j) * ld + 2 * (size_t)H + (size_t)h * dh + d, av);
  }
}

template <typename T>
static hipError_t fwd_t(int B, int S, int nh, int dh, int causal, const void *qkv, void *o, float *lse,
                        const DropArgs &da, hipStream_t s) {
  const long rows = (long)B * nh * S;
  const size_t smem = 4 * (size_t)(S + dh) * sizeof(float);
  hipLaunchKernelGGL((attn_fwd_simple_kernel<T>), dim3((unsigned)((rows + 3) / 4)), dim3(256), smem, s,
                     (const T *)qkv, (T *)o, lse, B, S, nh, dh, causal, 1.0f / sqrtf((float)dh), da);
  return hipGetLastError();
}

hipError_t launch_attn_fwd_simple(int dtype, int B, int S, int nh, int dh, int causal, const void *qkv, void *o,
                                  float *lse, hipStream_t s, const DropArgs *drop) {
  if ((long)B * S * nh == 0) return hipSuccess;
  const DropArgs da = drop != nullptr && drop->thr != 0 ? *drop : DropArgs{0u, 0u, 1.f};
  return dtype == kBF16 ? fwd_t<bf16>(B, S, nh, dh, causal, qkv, o, lse, da, s)
                        : fwd_t<float>(B, S, nh, dh, causal, qkv, o, lse, da, s);
}

template <typename T>
static hipError_t bwd_t(int B, int S, int nh, int dh, int causal, const void *qkv, const void *o, const float *lse,
                        const void *d_o, void *dqkv, float *ws, const DropArgs &da, hipStream_t s) {
  const long rows = (long)B * nh * S;
  const float scale = 1.0f / sqrtf((float)dh);
  const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
  hipLaunchKernelGGL((attn_bwd_dq_simple_kernel<T>), grid, block, 4 * (size_t)(S + 2 * dh) * sizeof(float), s,
                     (const T *)qkv, (const T *)o, lse, (const T *)d_o, (T *)dqkv, ws, B, S, nh, dh, causal, scale, da);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_bwd_dkv_simple_kernel<T>), grid, block, 4 * (size_t)(2 * S + 2 * dh) * sizeof(float), s,
                     (const T *)qkv, lse, (const T *)d_o, ws, (T *)dqkv, B, S, nh, dh, causal, scale, da);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_simple(int dtype, int B, int S, int nh, int dh, int causal, const void *qkv,
                                  const void *o, const float *lse, const void *d_o, void *dqkv, float *ws,
                                  hipStream_t s, const DropArgs *drop) {
  if ((long)B * S * nh == 0) return hipSuccess;
  const DropArgs da = drop != nullptr && drop->thr != 0 ? *drop : DropArgs{0u, 0u, 1.f};
  return dtype == kBF16 ? bwd_t<bf16>(B, S, nh, dh, causal, qkv, o, lse, d_o, dqkv, ws, da, s)
                        : bwd_t<float>(B, S, nh, dh, causal, qkv, o, lse, d_o, dqkv, ws, da, s);
}

}  // namespace dp
