// Plain LDS-tiled GEMM on the vector ALUs with fp32 accumulation.  This is the
// fp32 debug mode's GEMM and the fallback for shapes the MFMA kernels do not
// take; it handles any M, N, K through guarded loads.
#include "common.h"
#include "kernels.h"

namespace dp {

// C[m,n] = sum_k A(m,k) B(k,n) + bias[n] + res[m,n]
//   A(m,k) = A[m*sam + k*sak],  B(k,n) = B[k*sbk + n*sbn]
template <typename T>
__global__ __launch_bounds__(256) void gemm_simple_kernel(const T *__restrict__ A, const T *__restrict__ B,
                                                          const T *__restrict__ bias, const T *__restrict__ res,
                                                          T *__restrict__ C, int M, int N, int K, long sam,
                                                          long sak, long sbk, long sbn) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;  // 16 x 16 threads, 4x4 outputs each
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  // which of A/B index runs fastest in memory decides the load mapping
  const bool a_k_fast = sak == 1, b_k_fast = sbk == 1;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256;  // 0..1023
      int am, ak, bn, bk;
      if (a_k_fast) { ak = e & 15; am = e >> 4; } else { am = e & 63; ak = e >> 6; }
      if (b_k_fast) { bk = e & 15; bn = e >> 4; } else { bn = e & 63; bk = e >> 6; }
      const int gm = m0 + am, gka = k0 + ak, gn = n0 + bn, gkb = k0 + bk;
      As[ak][am] = (gm < M && gka < K) ? ldf(A + gm * sam + gka * sak) : 0.f;
      Bs[bk][bn] = (gn < N && gkb < K) ? ldf(B + gkb * sbk + gn * sbn) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j];
      if (bias != nullptr) v += ldf(bias + n);
      if (res != nullptr) v += ldf(res + (size_t)m * N + n);
      stf(C + (size_t)m * N + n, v);
    }
  }
}

hipError_t launch_gemm_simple(int dtype, const GemmArgs &a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  long sam, sak, sbk, sbn;
  if (a.mode == kGemmNT) { sam = a.K; sak = 1; sbk = 1; sbn = a.K; }
  else { sam = 1; sak = a.M; sbk = a.N; sbn = 1; }
  const dim3 grid((a.N + 63) / 64, (a.M + 63) / 64), block(256);
  if (dtype == kBF16)
    hipLaunchKernelGGL((gemm_simple_kernel<bf16>), grid, block, 0, s, (const bf16 *)a.A, (const bf16 *)a.B,
                       (const bf16 *)a.bias, (const bf16 *)a.res, (bf16 *)a.C, a.M, a.N, a.K, sam, sak, sbk, sbn);
  else
    hipLaunchKernelGGL((gemm_simple_kernel<float>), grid, block, 0, s, (const float *)a.A, (const float *)a.B,
                       (const float *)a.bias, (const float *)a.res, (float *)a.C, a.M, a.N, a.K, sam, sak, sbk, sbn);
  return hipGetLastError();
}

}  // namespace dp
