// Diagnostic: what the matrix cores sustain when nothing else limits them.  Every wave keeps 16
// independent 32x32 accumulators and issues v_mfma_f32_32x32x16_bf16 back to back on operand
// fragments held in registers; the operands are taken from a caller's buffer, because the
// clock the chip holds under this load depends on the data (all-zero operands run at the
// nominal clock, random mantissas draw more power and the clock drops).  Reports the rate and
// the shader clock over the loop (cycle counter against the constant 100 MHz counter).
#include "common.h"
#include "kernels.h"

namespace dp {
namespace {

typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void mfma_issue_kernel(const probe_bf16x8 *__restrict__ in, size_t n8, float *out,
                                                         int iters, unsigned long long *clk) {
  const size_t tid = threadIdx.x + (size_t)blockIdx.x * 256;
  probe_bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { a[i] = in[(tid * 8 + i) % n8]; b[i] = in[(tid * 8 + 4 + i) % n8]; }
  probe_f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  const unsigned long long c0 = __builtin_readcyclecounter(), r0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  const unsigned long long c1 = __builtin_readcyclecounter(), r1 = wall_clock64();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) s += acc[i][j][e];
  out[tid] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) { clk[0] = c1 - c0; clk[1] = r1 - r0; }
}

}  // namespace

// One workgroup of 4 waves per CU (the accumulators leave room for one wave a SIMD).
hipError_t run_mfma_probe(const void *data, size_t n_elems, int iters, int n_cus, float *tflops, float *shader_mhz,
                          hipStream_t s) {
  float *out = nullptr;
  unsigned long long *clk = nullptr, host_clk[2] = {0, 0};
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipMalloc(&out, (size_t)n_cus * 256 * sizeof(float));
  if (e == hipSuccess) e = hipMalloc(&clk, 2 * sizeof(unsigned long long));
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  float ms = 0.f;
  for (int rep = 0; rep < 2 && e == hipSuccess; ++rep) {   // the first launch warms the clocks up
    e = hipEventRecord(e0, s);
    if (e != hipSuccess) break;
    hipLaunchKernelGGL(mfma_issue_kernel, dim3(n_cus), dim3(256), 0, s, (const probe_bf16x8 *)data, n_elems / 8, out,
                       iters, clk);
    e = hipGetLastError();
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  }
  if (e == hipSuccess) e = hipMemcpy(host_clk, clk, sizeof host_clk, hipMemcpyDeviceToHost);
  if (e == hipSuccess && ms > 0.f && host_clk[1] > 0) {
    *tflops = (float)((double)n_cus * 4 * iters * 16 * 32768.0 / ((double)ms * 1e-3) / 1e12);
    *shader_mhz = (float)((double)host_clk[0] * 100.0 / (double)host_clk[1]);
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (out) (void)hipFree(out);
  if (clk) (void)hipFree(clk);
  return e;
}

}  // namespace dp
