// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32
// accumulation, fused bias / residual epilogue, bf16 output.
//
//   NT: C[M,N] = A[M,K] * B[N,K]^T   both operands contraction-contiguous
//       (forward with the transposed weight copy; dX = dY * W^T with W as stored)
//   TN: C[M,N] = A[K,M]^T * B[K,N]   contraction over the leading dimension
//       (dW = X^T * dY); tiles are staged in LDS as loaded and handed to the
//       matrix cores through the LDS transpose read (ds_read_b64_tr_b16).
//
// A block of WGM x WGN waves owns a BM x BN tile of C; every wave owns
// (BM/WGM) x (BN/WGN) of it as 32x32 MFMA accumulators.  K advances in steps of
// 64 through a double-buffered LDS stage with two k-steps of global loads in
// flight, one barrier per step.  No split-K, so the summation order is fixed
// and results do not depend on scheduling.
#include "common.h"
#include "kernels.h"

#include <cstdlib>
#include <cstring>
#include <type_traits>

namespace dp {

namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;


// LDS row strides in elements.  NT rows hold BK (+8) contraction elements: the
// 144-byte stride spreads the 16-byte fragment reads of 8 consecutive rows over
// all banks.  TN rows hold BM/BN (+16) elements: the 32-byte skew does the same
// for the four rows one transpose read touches.
template <int BMN, bool TN, int BK> struct Lds {
  static constexpr int kStride = TN ? BMN + 16 : BK + 8;
  static constexpr int kRows = TN ? BK : BMN;
  static constexpr int kElems = kStride * kRows;
};

__device__ __forceinline__ uint4 ld16(const bf16 *p) { return *reinterpret_cast<const uint4 *>(p); }

// ---- explicitly counted global loads ----------------------------------------------
// The main loop keeps two k-steps of global loads in flight.  Written as ordinary loads
// the compiler's wait-count insertion drains all of them at every loop back-edge, so the
// loads are issued as inline asm (invisible to that pass) and waited for with explicit
// s_waitcnt vmcnt(n): the counter retires in order, so "at most n outstanding" means every
// load older than the n youngest has landed.  touch() makes the registers look rewritten
// by the wait, which pins their consumers behind it.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void gload16(u32x4 &d, unsigned byte_off, const void *uniform_base) {
  asm volatile("global_load_dwordx4 %0, %1, %2" : "=&v"(d) : "v"(byte_off), "s"(uniform_base));
}
template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N)); }
__device__ __forceinline__ void touch(u32x4 &d) { asm volatile("" : "+v"(d)); }

// Global -> registers for one operand tile.  NT: tile is [BMN rows][BK], row r
// of the operand at p + r*ld.  TN: tile is [BK][BMN], contraction row k at
// p + k*ld.  Out-of-range chunks read as zero.
// FULL: the whole tile lies inside the operand, so the loads carry no guard at all (a
// guard's select would sit right behind its load and make the wave wait for it at once,
// which would undo the prefetch).  Otherwise out-of-range chunks read as zero.
template <int BMN, bool TN, bool FULL, int BK, int NTHR>
__device__ __forceinline__ void load_tile(uint4 (&st)[BMN * BK / 8 / NTHR], const bf16 *__restrict__ p, long ld,
                                          int row0, int rows, int k0, int K, int tid) {
  constexpr int NCH = BMN * BK / 8 / NTHR;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = tid + i * NTHR;
    int r, kk;
    if (TN) { kk = c / (BMN / 8); r = (c % (BMN / 8)) * 8; }
    else { r = c / (BK / 8); kk = (c % (BK / 8)) * 8; }
    const int gr = row0 + r, gk = k0 + kk;
    const long off = TN ? (long)gk * ld + gr : (long)gr * ld + gk;
    if (FULL) st[i] = ld16(p + off);
    else st[i] = (gr < rows && gk < K) ? ld16(p + off) : make_uint4(0, 0, 0, 0);
  }
}

template <int BMN, bool TN, int BK, int NTHR, typename V>
__device__ __forceinline__ void store_tile(bf16 *lds, const V (&st)[BMN * BK / 8 / NTHR], int tid) {
  constexpr int NCH = BMN * BK / 8 / NTHR;
  constexpr int S = Lds<BMN, TN, BK>::kStride;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = tid + i * NTHR;
    int off;
    if (TN) off = (c / (BMN / 8)) * S + (c % (BMN / 8)) * 8;
    else off = (c / (BK / 8)) * S + (c % (BK / 8)) * 8;
    *reinterpret_cast<V *>(lds + off) = st[i];
  }
}

// One 32 x 16 MFMA operand fragment: row (lane%32) of the 32-row block at
// `row0`, contraction elements k16 + 8*(lane/32) .. +7.
template <int BMN, bool TN, int BK>
__device__ __forceinline__ bf16x8 load_frag(const bf16 *lds, int row0, int k16, int lane) {
  constexpr int S = Lds<BMN, TN, BK>::kStride;
  if (!TN) return *reinterpret_cast<const bf16x8 *>(lds + (row0 + (lane & 31)) * S + k16 + 8 * (lane >> 5));
  // transpose read: a 16-lane group fetches 4 contraction rows x 16 columns; lane i of
  // the group supplies the address of row i/4, columns 4*(i%4).. and receives column i
  // of all four rows.
  const int i = lane & 15;
  const bf16 *p = lds + (k16 + 8 * (lane >> 5) + (i >> 2)) * S + row0 + 16 * ((lane >> 4) & 1) + 4 * (i & 3);
  union { s16x4 h[2]; bf16x8 v; } u;
  u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
  u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * S));
  return u.v;
}

template <int BM, int BN, bool TN, int BK, int WPE, int WGM, int WGN>
__global__ __launch_bounds__(64 * WGM * WGN) __attribute__((amdgpu_waves_per_eu(WPE, WPE))) void gemm_mfma_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ B,
                                                           const bf16 *__restrict__ bias,
                                                           const bf16 *__restrict__ res, bf16 *__restrict__ C,
                                                           bf16 *__restrict__ C2, int gelu_kind, int M,
                                                           int N, int K, int tiles_m, int tiles_n) {
  constexpr int NTHR = 64 * WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN, FM = WM / 32, FN = WN / 32;
  constexpr int AE = Lds<BM, TN, BK>::kElems, BE = Lds<BN, TN, BK>::kElems;
  // One LDS array addressed by integer offsets: stage s holds A at s*(AE+BE) and B
  // right after it.  (Picking a stage through an array of pointers turns the LDS
  // pointers generic, and the fragment reads then compile to flat loads that wait on
  // the global-load counter as well.)
  extern __shared__ __attribute__((aligned(16))) bf16 smem[];
  constexpr int STAGE = AE + BE;

  // Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous run
  // of tiles, and walk tiles in groups of 8 tile-rows so that a run shares A and B
  // panels in that XCD's L2.
  const int nt = tiles_m * tiles_n;
  int pid = blockIdx.x;
  {
    const int xcd = pid & 7, idx = pid >> 3, base = nt >> 3, rem = nt & 7;
    pid = xcd * base + (xcd < rem ? xcd : rem) + idx;
  }
  constexpr int GM = 8;
  const int group = pid / (GM * tiles_n);
  const int first_m = group * GM;
  const int gsz = min(tiles_m - first_m, GM);
  const int tm = first_m + (pid % (GM * tiles_n)) % gsz;
  const int tn = (pid % (GM * tiles_n)) / gsz;
  // Ragged last tiles are shifted back inside the matrix (they overlap their neighbour; each
  // element is still stored once, by the tile whose unshifted position covers it) whenever the matrix is at least one tile tall/wide: then no
  // load of the fast path needs a guard.  Smaller matrices keep their origin and take the
  // guarded path below.
  const bool interior = M >= BM && N >= BN;
  const int m0 = interior ? min(tm * BM, M - BM) : tm * BM, n0 = interior ? min(tn * BN, N - BN) : tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;
  const long lda = TN ? M : K, ldb = TN ? N : K;

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // multiply the LDS stage at element offset `cur` into the accumulators
  auto compute = [&](int cur) {
    bf16x8 a[2][FM], b[2][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) a[0][i] = load_frag<BM, TN, BK>(smem + cur, wm + i * 32, 0, lane);
#pragma unroll
    for (int j = 0; j < FN; ++j) b[0][j] = load_frag<BN, TN, BK>(smem + cur + AE, wn + j * 32, 0, lane);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int c = ks & 1;
      if (ks + 1 < BK / 16) {   // fragments of the next 16-slice are fetched under this slice's MFMAs
#pragma unroll
        for (int i = 0; i < FM; ++i) a[c ^ 1][i] = load_frag<BM, TN, BK>(smem + cur, wm + i * 32, (ks + 1) * 16, lane);
#pragma unroll
        for (int j = 0; j < FN; ++j)
          b[c ^ 1][j] = load_frag<BN, TN, BK>(smem + cur + AE, wn + j * 32, (ks + 1) * 16, lane);
      }
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c][i], b[c][j], acc[i][j], 0, 0, 0);
      // keep the next slice's LDS reads under this slice's MFMAs: MFMA, read, MFMA, read, ...
#pragma unroll
      for (int g = 0; g < FM * FN; ++g) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, TN ? 2 : 1, 0);
      }
    }
  };
  constexpr int NA = BM * BK / 8 / NTHR, NB = BN * BK / 8 / NTHR;

  if (K % BK == 0 && interior) {
    // ---- two-deep software pipeline with explicitly counted loads -----------------
    u32x4 ra0[NA], rb0[NB], ra1[NA], rb1[NB];
    // A thread's NA (NB) chunks of a tile sit a fixed, uniform distance apart, so one VGPR
    // byte offset per operand plus uniform (SGPR) base pointers address all of them.
    constexpr int RA = TN ? NTHR / (BM / 8) : NTHR / (BK / 8);   // rows between a thread's consecutive chunks
    constexpr int RB = TN ? NTHR / (BN / 8) : NTHR / (BK / 8);
    const unsigned offa = TN ? (unsigned)(((tid / (BM / 8)) * lda + (tid % (BM / 8)) * 8) * 2)
                             : (unsigned)(((tid / (BK / 8)) * lda + (tid % (BK / 8)) * 8) * 2);
    const unsigned offb = TN ? (unsigned)(((tid / (BN / 8)) * ldb + (tid % (BN / 8)) * 8) * 2)
                             : (unsigned)(((tid / (BK / 8)) * ldb + (tid % (BK / 8)) * 8) * 2);
    const bf16 *pa = TN ? A + m0 : A + (long)m0 * lda;   // uniform: advanced one k-step per issue
    const bf16 *pb = TN ? B + n0 : B + (long)n0 * ldb;
    const long step_a = TN ? (long)BK * lda : BK, step_b = TN ? (long)BK * ldb : BK;
    const long gap_a = (long)RA * lda, gap_b = (long)RB * ldb;
    auto issue_a = [&](u32x4 (&xa)[NA]) {
#pragma unroll
      for (int i = 0; i < NA; ++i) gload16(xa[i], offa, pa + i * gap_a);
      pa += step_a;
    };
    auto issue_b = [&](u32x4 (&xb)[NB]) {
#pragma unroll
      for (int i = 0; i < NB; ++i) gload16(xb[i], offb, pb + i * gap_b);
      pb += step_b;
    };
    auto issue = [&](u32x4 (&xa)[NA], u32x4 (&xb)[NB]) { issue_a(xa); issue_b(xb); };
    auto landed = [&](u32x4 (&xa)[NA], u32x4 (&xb)[NB]) {
#pragma unroll
      for (int i = 0; i < NA; ++i) touch(xa[i]);
#pragma unroll
      for (int i = 0; i < NB; ++i) touch(xb[i]);
    };
    const int nk = K / BK;
    issue(ra0, rb0);
    if (nk > 1) { issue(ra1, rb1); wait_vmcnt<NA + NB>(); } else { wait_vmcnt<0>(); }
    landed(ra0, rb0);
    store_tile<BM, TN, BK, NTHR>(smem, ra0, tid);
    store_tile<BN, TN, BK, NTHR>(smem + AE, rb0, tid);
    __syncthreads();
    // k-step kt: request tile kt+2 into (la, lb), multiply stage `cur`, then move tile kt+1
    // (requested one step ago, in (sa, sb)) into the other stage
    auto step = [&](int kt, int cur, u32x4 (&la)[NA], u32x4 (&lb)[NB], u32x4 (&sa)[NA], u32x4 (&sb)[NB]) {
      // The requests for tile kt+2 go out in two bursts, A before and B after the multiply:
      // a wave sits in the issue stage until the texture path has taken its requests
      // (16 clocks per 1 KB request, every wave of the CU queueing at once), so a burst
      // half as long at the top of the step leaves the MFMA pipes idle half as long.
      const bool more = kt + 2 < nk;
      if (more) issue_a(la);
      compute(cur);
      if (more) issue_b(lb);
      if (kt + 1 < nk) {
        if (more) wait_vmcnt<NA + NB>(); else wait_vmcnt<0>();
        landed(sa, sb);
        store_tile<BM, TN, BK, NTHR>(smem + (STAGE - cur), sa, tid);
        store_tile<BN, TN, BK, NTHR>(smem + (STAGE - cur) + AE, sb, tid);
      }
      __syncthreads();
    };
    for (int kt = 0; kt < nk; kt += 2) {
      step(kt, 0, ra0, rb0, ra1, rb1);
      if (kt + 1 < nk) step(kt + 1, STAGE, ra1, rb1, ra0, rb0);
    }
  } else {
    // ---- K tail present: guarded loads (zero-filled), one k-step of prefetch ------
    uint4 ra[NA], rb[NB];
    const int nk = (K + BK - 1) / BK;
    load_tile<BM, TN, false, BK, NTHR>(ra, A, lda, m0, M, 0, K, tid);
    load_tile<BN, TN, false, BK, NTHR>(rb, B, ldb, n0, N, 0, K, tid);
    store_tile<BM, TN, BK, NTHR>(smem, ra, tid);
    store_tile<BN, TN, BK, NTHR>(smem + AE, rb, tid);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      const int cur = (kt & 1) * STAGE;
      if (kt + 1 < nk) {
        load_tile<BM, TN, false, BK, NTHR>(ra, A, lda, m0, M, (kt + 1) * BK, K, tid);
        load_tile<BN, TN, false, BK, NTHR>(rb, B, ldb, n0, N, (kt + 1) * BK, K, tid);
      }
      compute(cur);
      if (kt + 1 < nk) {
        store_tile<BM, TN, BK, NTHR>(smem + (STAGE - cur), ra, tid);
        store_tile<BN, TN, BK, NTHR>(smem + (STAGE - cur) + AE, rb, tid);
      }
      __syncthreads();
    }
  }

  // epilogue: accumulator element e of lane l is C[8*(e/4) + 4*(l/32) + e%4][l%32] of its 32x32 block
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    const int col = n0 + wn + j * 32 + (lane & 31);
    if (col >= N || col < tn * BN) continue;   // a shifted tile leaves its neighbour's part alone
    const float bv = bias != nullptr ? (float)bias[col] : 0.f;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = m0 + wm + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        if (row >= M || row < tm * BM) continue;
        float v = acc[i][j][e] + bv;
        if (res != nullptr) v += (float)res[(long)row * N + col];
        const bf16 stored = (bf16)v;
        C[(long)row * N + col] = stored;
        // fused activation: computed from the value as stored, so that a later standalone
        // GELU of C gives the same bits
        if (C2 != nullptr) C2[(long)row * N + col] = (bf16)gelu_f((float)stored, gelu_kind);
      }
    }
  }
}

template <int BM, int BN, bool TN, int BK = 64, int WPE = (BM * BN > 128 * 128 ? 1 : 2), int WGM = 2, int WGN = 2>
hipError_t launch_cfg(const GemmArgs &a, hipStream_t s) {
  constexpr size_t smem = 2 * (size_t)(Lds<BM, TN, BK>::kElems + Lds<BN, TN, BK>::kElems) * sizeof(bf16);
  static bool attr_set = false;
  auto kern = gemm_mfma_kernel<BM, BN, TN, BK, WPE, WGM, WGN>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(64 * WGM * WGN), smem, s, (const bf16 *)a.A, (const bf16 *)a.B,
                     (const bf16 *)a.bias, (const bf16 *)a.res, (bf16 *)a.C, (bf16 *)a.C2, a.gelu_kind, a.M, a.N, a.K,
                     tiles_m, tiles_n);
  return hipGetLastError();
}

template <bool TN>
hipError_t launch_mode(const GemmArgs &a, hipStream_t s) {
  auto tiles = [&](int bm, int bn) { return (long)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn); };
  // Tile choice: 256x256 (8 waves, 128x64 a wave) halves the L1/L2 traffic per flop of
  // 128x128 and is taken whenever it still gives nearly every CU a workgroup; below that
  // the largest tile that does.  DPSTAGE_GEMM_TILE=256x256|128x128|64x64 overrides
  // the choice (tuning aid).
  static const char *force = getenv("DPSTAGE_GEMM_TILE");
  if (force != nullptr) {
    if (!strcmp(force, "256x256")) return launch_cfg<256, 256, TN, 64, 2, 4, 2>(a, s);
    if (!strcmp(force, "128x128")) return launch_cfg<128, 128, TN>(a, s);
    if (!strcmp(force, "64x64")) return launch_cfg<64, 64, TN>(a, s);
  }
  if (tiles(256, 256) >= 240) return launch_cfg<256, 256, TN, 64, 2, 4, 2>(a, s);
  if (tiles(128, 128) >= 256) return launch_cfg<128, 128, TN>(a, s);
  if (tiles(64, 128) >= 256) return launch_cfg<64, 128, TN>(a, s);
  return launch_cfg<64, 64, TN>(a, s);
}

}  // namespace

bool gemm_mfma_supported(const GemmArgs &a) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return false;
  const bool aligned = (((uintptr_t)a.A | (uintptr_t)a.B) & 15) == 0;
  if (a.mode == kGemmNT) return aligned && a.K % 8 == 0;
  return aligned && a.M % 8 == 0 && a.N % 8 == 0;   // TN: rows of A and B are M and N long
}

hipError_t launch_gemm_mfma(const GemmArgs &a, hipStream_t s) {
  // DPSTAGE_GEMM_NT=reg / DPSTAGE_GEMM_TN=reg keep that form on the register-staged kernel of this file (tuning aid)
  static const char *nt = getenv("DPSTAGE_GEMM_NT"), *tn = getenv("DPSTAGE_GEMM_TN");
  const char *keep = a.mode == kGemmNT ? nt : tn;
  if (gemm_dma_supported(a) && !(keep != nullptr && !strcmp(keep, "reg"))) return launch_gemm_dma(a, s);
  return a.mode == kGemmNT ? launch_mode<false>(a, s) : launch_mode<true>(a, s);
}

}  // namespace dp
