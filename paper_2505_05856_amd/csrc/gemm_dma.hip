// bf16 NT GEMM on the gfx950 matrix cores with operand tiles brought into LDS by the
// load unit itself (global_load_lds_dwordx4): no staging registers, no LDS store
// instructions, and the requests can be spread between the MFMAs of a k-step.
//
//   C[M,N] = A[M,K] * B[N,K]^T (+ bias, + residual), fp32 accumulation, bf16 out.
//
// Preconditions (checked by gemm_dma_supported): K % 64 == 0, M >= BM, N >= BN for the
// tile chosen, 16-byte aligned operands.  Ragged edge tiles are shifted back inside the
// matrix, so no load is ever guarded.  No split-K: the summation order is fixed.
//
// LDS layout.  A stage holds the A tile [BM rows][64 k] and the B tile [BN rows][64 k]
// as 128-byte rows without padding (the load unit writes the 64 lanes of a request to
// 1 KB of consecutive LDS, i.e. 8 whole rows).  Bank conflicts of the 16-byte fragment
// reads are avoided by a swizzle instead: the 16-byte chunk c of row r sits at chunk
// position c ^ ((r >> 1) & 7), which spreads any 16 consecutive rows of one logical
// chunk over all 16 chunk positions of the 256-byte bank period.  The swizzle costs
// nothing on the way in: a lane simply fetches the global chunk that belongs at its
// fixed LDS position.
#include "common.h"
#include "kernels.h"

#include <cstdlib>
#include <cstring>
#include <type_traits>

namespace dp {

namespace {

constexpr int kBK = 64;          // contraction elements per stage
constexpr int kRowBytes = 128;   // one LDS row: 64 bf16

// One request: lane l fetches 16 bytes from uniform_base + byte_off and the unit stores
// them at LDS byte lds_base + 16*l.  Invisible to the compiler's wait-count pass; the
// kernel counts them itself (vmcnt retires in order).  M0 is reserved by the compiler (never
// allocated), and nothing else in this file makes it emit an M0 user, so it is simply overwritten.
__device__ __forceinline__ void dma16(unsigned lds_base, unsigned byte_off, const void *uniform_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_base), "v"(byte_off), "s"(uniform_base));
}
template <int N> __device__ __forceinline__ void wait_vmcnt_mem() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
__device__ __forceinline__ const char *uniform_ptr(const char *p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const char *)(((uint64_t)hi << 32) | lo);
}

template <int BM, int BN, int WGM, int WGN, int STAGES, bool ACT>
__global__ __launch_bounds__(64 * WGM * WGN) __attribute__((amdgpu_waves_per_eu(WGM * WGN / 4, WGM * WGN / 4))) void gemm_dma_nt_kernel(
    const bf16 *__restrict__ A, const bf16 *__restrict__ B, const bf16 *__restrict__ bias,
    const bf16 *__restrict__ res, bf16 *__restrict__ C, bf16 *__restrict__ C2, int gelu_kind, int M, int N, int K,
    int tiles_m, int tiles_n) {
  constexpr int NW = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN, FM = WM / 32, FN = WN / 32;
  constexpr int A_BYTES = BM * kRowBytes, B_BYTES = BN * kRowBytes, STAGE_BYTES = A_BYTES + B_BYTES;
  constexpr int NIA = BM / 8 / NW, NIB = BN / 8 / NW;   // requests per wave per stage
  static_assert(NIA % 2 == 0 && NIB % 2 == 0, "a wave's row groups must start on an even group");
  constexpr int NI = NIA + NIB;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

  // tile order: each XCD gets a contiguous run of tiles, walked in groups of 8 tile rows
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
  const int m0 = min(tm * BM, M - BM), n0 = min(tn * BN, N - BN);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;

  // ---- request addressing -------------------------------------------------------------
  // Request j of this wave for operand A fills LDS rows 8*(wave*NIA + j) .. +7; lane l is
  // row l/8, chunk position l%8 of them and fetches logical chunk (l%8) ^ swizzle(row).
  // Even and odd row groups differ in swizzle bit 2, hence two lane offsets.
  const int r8 = lane >> 3, pc = lane & 7;
  const unsigned ldk = (unsigned)K * 2u;   // bytes per operand row
  unsigned voff_even = (unsigned)r8 * ldk + (unsigned)((pc ^ (r8 >> 1)) << 4);
  unsigned voff_odd = (unsigned)r8 * ldk + (unsigned)((pc ^ (r8 >> 1) ^ 4) << 4);
  const char *pa[NIA], *pb[NIB];
#pragma unroll
  for (int j = 0; j < NIA; ++j)
    pa[j] = uniform_ptr((const char *)A + (size_t)(m0 + 8 * (wave * NIA + j)) * ldk);
#pragma unroll
  for (int j = 0; j < NIB; ++j)
    pb[j] = uniform_ptr((const char *)B + (size_t)(n0 + 8 * (wave * NIB + j)) * ldk);
  const unsigned lds_a = (unsigned)(wave * NIA) * 1024u, lds_b = (unsigned)A_BYTES + (unsigned)(wave * NIB) * 1024u;

  // request i (0 .. NI-1) of this wave for the stage at LDS byte `sb`
  auto request = [&](int i, unsigned sb) {
    if (i < NIA) dma16(sb + lds_a + (unsigned)i * 1024u, (i & 1) ? voff_odd : voff_even, pa[i]);
    else dma16(sb + lds_b + (unsigned)(i - NIA) * 1024u, ((i - NIA) & 1) ? voff_odd : voff_even, pb[i - NIA]);
  };
  auto advance_k = [&]() { voff_even += kBK * 2; voff_odd += kBK * 2; };

  // ---- fragment addressing --------------------------------------------------------------
  // lane l reads row (l%32) of a 32-row block, logical chunk 2*ks + l/32 of slice ks; with
  // the swizzle that is byte ((row*128) + x0) ^ (ks << 5) of the tile.
  const unsigned x0 = (unsigned)(((lane >> 5) ^ ((lane >> 1) & 7)) << 4);
  const unsigned fa = (unsigned)(wm + (lane & 31)) * kRowBytes + x0;
  const unsigned fb = (unsigned)A_BYTES + (unsigned)(wn + (lane & 31)) * kRowBytes + x0;
  auto frag = [&](unsigned base, int blk, int ks) {
    // the block offset has no bits below 128, so it can stay outside the xor (an immediate of the read)
    return *reinterpret_cast<const bf16x8 *>(lds + ((base ^ (unsigned)(ks << 5)) + (unsigned)blk * 32u * kRowBytes));
  };

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = K / kBK;
  // prologue: stages 0 .. STAGES-2
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s) {
    if (s < nk) {
#pragma unroll
      for (int i = 0; i < NI; ++i) request(i, (unsigned)s * STAGE_BYTES);
      advance_k();
    }
  }

  int cur = 0;                 // ring slot of k-step kt
  int nxt = STAGES - 1;        // ring slot the requests of this step go to
  // One k-step.  MORE: k-step kt+STAGES-1 exists and is requested under this step's MFMAs.
  auto step = [&](auto more_tag) {
    constexpr bool MORE = decltype(more_tag)::value;
    // k-step kt must have landed: at most the requests of the later steps may be pending
    if (MORE) wait_vmcnt_mem<(STAGES - 2) * NI>(); else wait_vmcnt_mem<0>();
    __syncthreads();   // everyone's part of this stage is in, and everyone is done with the previous slot
    const unsigned sb = (unsigned)cur * STAGE_BYTES, nb = (unsigned)nxt * STAGE_BYTES;
    bf16x8 a[2][FM], b[2][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) a[0][i] = frag(sb + fa, i, 0);
#pragma unroll
    for (int j = 0; j < FN; ++j) b[0][j] = frag(sb + fb, j, 0);
    constexpr int KS = kBK / 16;
    constexpr int TOTAL = KS * FM * FN;       // MFMAs of the step
    static_assert(TOTAL % NI == 0, "requests are spread evenly between the MFMAs");
    constexpr int EVERY = TOTAL / NI;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int c = ks & 1;
      if (ks + 1 < KS) {   // fragments of the next 16-slice are fetched under this slice's MFMAs
#pragma unroll
        for (int i = 0; i < FM; ++i) a[c ^ 1][i] = frag(sb + fa, i, ks + 1);
#pragma unroll
        for (int j = 0; j < FN; ++j) b[c ^ 1][j] = frag(sb + fb, j, ks + 1);
      }
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c][i], b[c][j], acc[i][j], 0, 0, 0);
          const int g = (ks * FM + i) * FN + j;
          if (MORE && g % EVERY == EVERY - 1) request(g / EVERY, nb);
        }
    }
    if (MORE) advance_k();
    cur = cur + 1 == STAGES ? 0 : cur + 1;
    nxt = nxt + 1 == STAGES ? 0 : nxt + 1;
  };
  int kt = 0;
  for (; kt + STAGES - 1 < nk; ++kt) step(std::true_type{});
  for (; kt < nk; ++kt) step(std::false_type{});

  // epilogue: accumulator element e of lane l is C[8*(e/4) + 4*(l/32) + e%4][l%32] of its 32x32 block.
  // Addresses are a uniform pointer (scalar registers) per row plus one 32-bit lane offset, which
  // keeps the address arithmetic off the vector registers the accumulators fill.
  const unsigned lane_off = ((unsigned)(4 * (lane >> 5)) * (unsigned)N + (unsigned)(lane & 31)) * 2u;
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    const int col0 = n0 + wn + j * 32;
    const float bv = bias != nullptr ? (float)bias[col0 + (lane & 31)] : 0.f;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const size_t urow = (size_t)(m0 + wm + i * 32 + 8 * (e >> 2) + (e & 3));
        const size_t uoff = (urow * (size_t)N + (size_t)col0) * 2 + lane_off;
        float v = acc[i][j][e] + bv;
        if (res != nullptr) v += (float)*reinterpret_cast<const bf16 *>((const char *)res + uoff);
        const bf16 stored = (bf16)v;
        *reinterpret_cast<bf16 *>((char *)C + uoff) = stored;
        // fused activation: computed from the value as stored, so that a later standalone
        // GELU of C gives the same bits
        if (ACT) *reinterpret_cast<bf16 *>((char *)C2 + uoff) = (bf16)gelu_f((float)stored, gelu_kind);
      }
    }
  }
}

template <int BM, int BN, int WGM, int WGN, int STAGES, bool ACT>
hipError_t launch_dma_act(const GemmArgs &a, hipStream_t s) {
  constexpr size_t smem = (size_t)STAGES * (BM + BN) * kRowBytes;
  static_assert(smem <= 160 * 1024, "LDS of one CU");
  static bool attr_set = false;
  auto kern = gemm_dma_nt_kernel<BM, BN, WGM, WGN, STAGES, ACT>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(64 * WGM * WGN), smem, s, (const bf16 *)a.A,
                     (const bf16 *)a.B, (const bf16 *)a.bias, (const bf16 *)a.res, (bf16 *)a.C, (bf16 *)a.C2,
                     a.gelu_kind, a.M, a.N, a.K, tiles_m, tiles_n);
  return hipGetLastError();
}

template <int BM, int BN, int WGM, int WGN, int STAGES>
hipError_t launch_dma_cfg(const GemmArgs &a, hipStream_t s) {
  return a.C2 != nullptr ? launch_dma_act<BM, BN, WGM, WGN, STAGES, true>(a, s)
                         : launch_dma_act<BM, BN, WGM, WGN, STAGES, false>(a, s);
}

}  // namespace

bool gemm_dma_supported(const GemmArgs &a) {
  if (a.mode != kGemmNT || a.M < 128 || a.N < 128 || a.K <= 0 || a.K % kBK != 0) return false;
  if ((uint64_t)a.K * 2 * 8 + 4096 > 0xffffffffull) return false;   // lane offsets are 32-bit
  return (((uintptr_t)a.A | (uintptr_t)a.B) & 15) == 0;
}

hipError_t launch_gemm_dma(const GemmArgs &a, hipStream_t s) {
  auto tiles = [&](int bm, int bn) { return (long)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn); };
  static const char *force = getenv("DPSTAGE_GEMM_TILE");
  const bool big_ok = a.M >= 256 && a.N >= 256;
  if (force != nullptr) {
    if (!strcmp(force, "256x256") && big_ok) return launch_dma_cfg<256, 256, 4, 2, 2>(a, s);
    if (!strcmp(force, "128x128")) return launch_dma_cfg<128, 128, 2, 2, 4>(a, s);
  }
  if (big_ok && tiles(256, 256) >= 240) return launch_dma_cfg<256, 256, 4, 2, 2>(a, s);
  return launch_dma_cfg<128, 128, 2, 2, 4>(a, s);
}

}  // namespace dp
