// bf16 GEMM on the gfx950 matrix cores with operand tiles brought into LDS by the
// load unit itself (global_load_lds_dwordx4): no staging registers, no LDS store
// instructions, and the requests can be spread between the MFMAs of a k-step.
//
//   NT: C[M,N] = A[M,K] * B[N,K]^T (+ bias, + residual, optional second output gelu(C))
//   TN: C[M,N] = A[K,M]^T * B[K,N]
// fp32 accumulation, bf16 out.
//
// Preconditions (checked by gemm_dma_supported): K % 64 == 0, M >= BM, N >= BN for the
// tile chosen, 16-byte aligned operands and rows.  Ragged edge tiles are shifted back
// inside the matrix, so no load is ever guarded.  No split-K: the summation order is fixed.
//
// LDS layout.  The load unit writes the 64 lanes of a request to 1 KB of consecutive LDS,
// so rows cannot be padded; bank conflicts are avoided by swizzling 16-byte chunks
// instead, which costs nothing on the way in: a lane simply fetches the global chunk
// that belongs at its fixed LDS position.
//   NT: a stage holds the A tile [BM rows][64 k] and the B tile [BN rows][64 k] as
//       128-byte rows; chunk c of row r sits at chunk position c ^ ((r >> 1) & 7), which
//       spreads any 16 consecutive rows of one logical chunk (one 16-byte fragment read)
//       over all 16 chunk positions of the 256-byte bank period.
//   TN: a stage holds the tiles as loaded, [64 k rows][BM] and [64 k rows][BN]; fragments
//       come through the transpose read (ds_read_b64_tr_b16), one of which touches four
//       consecutive k rows x 64 bytes per half wave.  Chunk c of k row r sits at
//       c ^ ((r & 3) << 2): the four rows land in the four 64-byte quarters of the bank
//       period.
#include "common.h"
#include "kernels.h"

#include <cstdlib>
#include <cstring>
#include <type_traits>

namespace dp {

namespace {

constexpr int kKAlign = 64;      // K must be a multiple of this (every stage depth divides it)

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// One request: lane l fetches 16 bytes from uniform_base + byte_off and the unit stores
// them at LDS byte lds_base + 16*l.  Invisible to the compiler's wait-count pass; the
// kernel counts them itself (vmcnt retires in order).  M0 is reserved by the compiler (never
// allocated), and nothing else in this file makes it emit an M0 user, so it is simply overwritten.
__device__ __forceinline__ void dma16(unsigned lds_base, unsigned byte_off, const void *uniform_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_base), "v"(byte_off), "s"(uniform_base) : "m0", "memory");
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

// TN: chunk-position swizzle of k row r of a tile whose rows are ROWB bytes.  256- and
// 512-byte rows: the four rows of a transpose read go to the four 64-byte quarters of the
// bank period.  128-byte rows (two rows a period): rows r and r+2 swap 64-byte halves.
template <int ROWB> __device__ __forceinline__ constexpr int tn_swizzle(int r) {
  return ROWB == 128 ? ((r >> 1) & 1) << 2 : (r & 3) << 2;
}

template <int BM, int BN, int WGM, int WGN, int STAGES, bool ACT, bool TN, int BK, bool SPLIT>
__global__ __attribute__((amdgpu_waves_per_eu(WGM * WGN / 4, WGM * WGN / 4), amdgpu_flat_work_group_size(64 * WGM * WGN, 64 * WGM * WGN))) void gemm_dma_kernel(
    const bf16 *__restrict__ A, const bf16 *__restrict__ B, const bf16 *__restrict__ bias,
    const bf16 *__restrict__ res, bf16 *__restrict__ C, bf16 *__restrict__ C2, int gelu_kind, int M, int N, int K,
    int tiles_m, int tiles_n) {
  constexpr int NW = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN, FM = WM / 32, FN = WN / 32;
  static_assert(BK == 64 || BK == 32, "stage depth");
  constexpr int kRowBytes = BK * 2;                  // NT: one LDS row
  constexpr int CPR = BK / 8, RP = 16 / CPR;         // NT: chunks per row, rows per 256-byte bank period
  constexpr int A_BYTES = BM * kRowBytes, B_BYTES = BN * kRowBytes, STAGE_BYTES = A_BYTES + B_BYTES;
  constexpr int ROWB_A = BM * 2, ROWB_B = BN * 2;   // TN: bytes of one k row of a tile
  constexpr int NIA = A_BYTES / 1024 / NW, NIB = B_BYTES / 1024 / NW;   // requests per wave per stage
  static_assert(NIA >= 1 && NIB >= 1, "every wave issues requests for both operands");
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
  // Request j of this wave for operand A fills LDS bytes 1024*(wave*NIA + j) .. +1023 of
  // the A tile.  Consecutive requests alternate between two lane offsets ("even"/"odd"
  // request groups) wherever the swizzle depends on the group's parity.
  //   NT: a request is 8 operand rows x 128 bytes; lane l is row l/8, chunk position l%8
  //       and fetches logical chunk (l%8) ^ ((row >> 1) & 7).
  //   TN: a request is RPR = 1024/ROWB k rows of ROWB bytes; lane l is k row l/(64/RPR),
  //       chunk position l%(64/RPR) and fetches logical chunk position ^ ((krow & 3) << 2).
  const unsigned lda = (unsigned)(TN ? M : K) * 2u, ldb = (unsigned)(TN ? N : K) * 2u;   // operand row bytes
  unsigned voa[2], vob[2];
  if (!TN) {
    constexpr int RPQ = 64 / CPR;   // operand rows per request
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      const int r = lane / CPR, pc = lane % CPR;
      voa[v] = vob[v] = (unsigned)r * lda + (unsigned)((pc ^ (((RPQ * v + r) / RP) % CPR)) << 4);
    }
  } else {
    constexpr int RPA = 1024 / ROWB_A, RPB = 1024 / ROWB_B;
    static_assert(RPA == 2 || RPA == 4 || RPA == 8, "tile width 64, 128 or 256");
    static_assert(RPB == 2 || RPB == 4 || RPB == 8, "tile width 64, 128 or 256");
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      const int ka = lane / (64 / RPA), pa_ = lane % (64 / RPA);
      voa[v] = (unsigned)ka * lda + (unsigned)((pa_ ^ tn_swizzle<ROWB_A>(RPA * v + ka)) << 4);
      const int kb = lane / (64 / RPB), pb_ = lane % (64 / RPB);
      vob[v] = (unsigned)kb * ldb + (unsigned)((pb_ ^ tn_swizzle<ROWB_B>(RPB * v + kb)) << 4);
    }
  }
  const char *pa[NIA], *pb[NIB];
#pragma unroll
  for (int j = 0; j < NIA; ++j)
    pa[j] = TN ? uniform_ptr((const char *)A + (size_t)((1024 / ROWB_A) * (wave * NIA + j)) * lda + (size_t)m0 * 2)
               : uniform_ptr((const char *)A + (size_t)(m0 + (64 / CPR) * (wave * NIA + j)) * lda);
#pragma unroll
  for (int j = 0; j < NIB; ++j)
    pb[j] = TN ? uniform_ptr((const char *)B + (size_t)((1024 / ROWB_B) * (wave * NIB + j)) * ldb + (size_t)n0 * 2)
               : uniform_ptr((const char *)B + (size_t)(n0 + (64 / CPR) * (wave * NIB + j)) * ldb);
  const unsigned lds_a = (unsigned)(wave * NIA) * 1024u, lds_b = (unsigned)A_BYTES + (unsigned)(wave * NIB) * 1024u;

  // request i (0 .. NI-1) of this wave for the stage at LDS byte `sb`
  auto request = [&](int i, unsigned sb) {
    if (i < NIA) dma16(sb + lds_a + (unsigned)i * 1024u, voa[(wave * NIA + i) & 1], pa[i]);
    else dma16(sb + lds_b + (unsigned)(i - NIA) * 1024u, vob[(wave * NIB + i - NIA) & 1], pb[i - NIA]);
  };
  auto advance_k = [&]() {
    const unsigned da = TN ? BK * lda : BK * 2, db = TN ? BK * ldb : BK * 2;
    voa[0] += da; voa[1] += da; vob[0] += db; vob[1] += db;
  };

  // ---- fragment addressing --------------------------------------------------------------
  // NT: lane l reads row (l%32) of a 32-row block, logical chunk 2*ks + l/32 of slice ks; with
  //     the swizzle that is byte ((row*128) + x0) ^ (ks << 5) of the tile.
  // TN: a 16-lane group fetches 4 k rows x 16 columns per transpose read; lane i of the group
  //     supplies the address of k row i/4, columns 4*(i%4).. and receives column i of all
  //     four rows.  Lanes 16..31 take the next 16 columns, lanes 32..63 the k rows 8 further;
  //     a second read 4 rows on completes the 8 contraction elements of the operand.
  const unsigned x0 = (unsigned)(((lane >> 5) ^ (((lane & 31) / RP) % CPR)) << 4);
  const unsigned fa = (unsigned)(wm + (lane & 31)) * kRowBytes + x0;
  const unsigned fb = (unsigned)A_BYTES + (unsigned)(wn + (lane & 31)) * kRowBytes + x0;
  const int ti = lane & 15, tt = ti >> 2;                                    // TN: k row within the four
  const unsigned tlow = (unsigned)((2 * ((lane >> 4) & 1) + ((ti & 3) >> 1)) * 16 + (ti & 1) * 8);
  const unsigned trow = (unsigned)(8 * (lane >> 5) + tt);
  auto frag = [&](unsigned base, int blk, int ks, bool is_b) -> bf16x8 {
    if (!TN) {
      // the block offset has no bits below 128, so it can stay outside the xor (an immediate of the read)
      return *reinterpret_cast<const bf16x8 *>(lds + (((base + (is_b ? fb : fa)) ^ (unsigned)(ks << 5)) + (unsigned)blk * 32u * kRowBytes));
    }
    const unsigned rowb = is_b ? ROWB_B : ROWB_A;
    const unsigned cw = (unsigned)((is_b ? wn : wm) / 8 + blk * 4);        // first chunk of the 32-column block
    const unsigned sw = is_b ? (unsigned)tn_swizzle<ROWB_B>(tt) : (unsigned)tn_swizzle<ROWB_A>(tt);
    const unsigned off = base + (is_b ? (unsigned)A_BYTES : 0u) + trow * rowb + ((cw ^ sw) << 4) + tlow +
                         (unsigned)ks * 16u * rowb;
    union { s16x4 h[2]; bf16x8 v; } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(lds + off));
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(lds + off + 4u * rowb));
    return u.v;
  };

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = K / BK;
  constexpr int KS = BK / 16;                      // 16-deep MFMA slices of a k-step
  // The main loop is software-pipelined by hand over "slices" of SK MFMA k-slices: the
  // fragments of slice s+1 are read from LDS into the other half of a register double buffer
  // before the MFMAs of slice s are issued, so an LDS read has a whole slice of MFMAs (at
  // least four per wave) to complete.  Scheduling barriers pin that order: left alone, the
  // compiler reuses one set of fragment registers and waits for every read right before its
  // first MFMA.
  constexpr int SK = FM * FN >= 8 ? 1 : (FM * FN >= 4 ? 1 : 2);
  constexpr int NS = KS / SK;                      // slices of a k-step
  constexpr int MPS = SK * FM * FN;                // MFMAs of a slice
  static_assert(KS % SK == 0 && NS % 2 == 0, "the fragment double buffer keeps its parity across steps");
  bf16x8 a[2][SK][FM], b[2][SK][FN];
  // fragments of slice s of the tiles at LDS bytes base_a / base_b (frag adds A_BYTES for B)
  auto read_slice = [&](auto buf_tag, unsigned base_a, unsigned base_b, int s) {
    constexpr int BUF = decltype(buf_tag)::value;
#pragma unroll
    for (int q = 0; q < SK; ++q) {
#pragma unroll
      for (int i = 0; i < FM; ++i) a[BUF][q][i] = frag(base_a, i, s * SK + q, false);
#pragma unroll
      for (int j = 0; j < FN; ++j) b[BUF][q][j] = frag(base_b, j, s * SK + q, true);
    }
  };
  // the MFMAs of one slice; req(g) issues the operand requests that go behind MFMA g
  auto mfma_slice = [&](auto buf_tag, auto &&req) {
    constexpr int BUF = decltype(buf_tag)::value;
#pragma unroll
    for (int q = 0; q < SK; ++q)
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[BUF][q][i], b[BUF][q][j], acc[i][j], 0, 0, 0);
          req((q * FM + i) * FN + j);
        }
  };
  auto no_req = [](int) {};
  using Buf0 = std::integral_constant<int, 0>;
  using Buf1 = std::integral_constant<int, 1>;
  // One pass of the loop, for k-step kt, entered right behind the barrier that certified
  // stage kt (so no LDS read is in flight on entry, nor at the loop's back edge: the
  // compiler's wait-count pass only places exact partial waits inside straight-line code):
  //   read slice 0 of stage kt, under the MFMAs of the LAST slice of step kt-1, whose
  //     fragments are still in buffer 1 (not FIRST), with req_first's requests between them;
  //   slices 0 .. NS-2: read the next slice, then the MFMAs of this one, req_inner between them;
  //   every LDS read of stage kt has now been issued: wait for stage kt+1 and pass the
  //     barrier that certifies it and frees stage kt (NEXT); the MFMAs of slice NS-1 follow
  //     in the next pass (or behind the loop).
  auto pass = [&](auto first_tag, auto next_tag, unsigned base_a, unsigned base_b, auto &&wait_next,
                  auto &&req_first, auto &&req_inner) {
    constexpr bool FIRST = decltype(first_tag)::value, NEXT = decltype(next_tag)::value;
    read_slice(Buf0{}, base_a, base_b, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (!FIRST) {
      mfma_slice(Buf1{}, req_first);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int s = 0; s + 1 < NS; ++s) {
      if (s & 1) read_slice(Buf0{}, base_a, base_b, s + 1); else read_slice(Buf1{}, base_a, base_b, s + 1);
      __builtin_amdgcn_sched_barrier(0);
      if (s & 1) mfma_slice(Buf1{}, [&](int g) { req_inner(s * MPS + g); });
      else mfma_slice(Buf0{}, [&](int g) { req_inner(s * MPS + g); });
      __builtin_amdgcn_sched_barrier(0);
    }
    if (NEXT) {
      wait_next();
      __syncthreads();
    }
  };
  // a request pinned in place between the MFMAs around it
  auto pinned = [&](auto &&issue) {
    __builtin_amdgcn_sched_barrier(0);
    issue();
    __builtin_amdgcn_sched_barrier(0);
  };
  constexpr int INNER = (NS - 1) * MPS;   // MFMAs of a pass that can carry its spread-out requests
  using Yes = std::true_type;
  using No = std::false_type;
  if constexpr (SPLIT) {
    // ---- ring of five operand tiles ---------------------------------------------------
    // A 256x256 k-step fills 64 KB of LDS, so only two whole stages fit.  With the A and B
    // tiles as separate ring entries a fifth tile fits: slot (2k) % 5 holds A(k), slot
    // (2k+1) % 5 holds B(k).  Request order A0 B0 A1 B1 A2 | B2 A3 | B3 A4 ...: pass k asks
    // for B(k+1) right behind the barrier that freed A(k-1)'s slot, and for A(k+2), spread
    // over its inner slices, into the slot B(k-1) left; a B tile so has one step to land
    // and an A tile one to two.  (The launcher sends K < 3 * BK elsewhere.)
    static_assert(BM == BN, "the ring entries are of one size");
    constexpr unsigned TILE = A_BYTES;
    auto req_a = [&](int i, unsigned slot) {
        dma16(slot * TILE + lds_a + (unsigned)i * 1024u, voa[(wave * NIA + i) & 1], pa[i]);
    };
    auto req_b = [&](int i, unsigned slot) {
        dma16(slot * TILE + (lds_b - (unsigned)A_BYTES) + (unsigned)i * 1024u, vob[(wave * NIB + i) & 1], pb[i]);
    };
    const unsigned da = TN ? BK * lda : BK * 2, db = TN ? BK * ldb : BK * 2;
    auto adv_a = [&]() { voa[0] += da; voa[1] += da; };
    auto adv_b = [&]() { vob[0] += db; vob[1] += db; };
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int i = 0; i < NIA; ++i) req_a(i, 2u * t);
      adv_a();
#pragma unroll
      for (int i = 0; i < NIB; ++i) req_b(i, 2u * t + 1u);
      adv_b();
    }
    wait_vmcnt_mem<NIA + NIB>();
    __syncthreads();
    unsigned sa = 0, sbk = 1;   // slots of A(kt), B(kt)
    auto ring = [](unsigned s, unsigned d) { return s + d >= 5 ? s + d - 5 : s + d; };
    // MORE: k-step kt+2 exists (its A tile is requested in this pass)
    auto step = [&](auto first_tag, auto next_tag, auto more_tag) {
      constexpr bool FIRST = decltype(first_tag)::value, NEXT = decltype(next_tag)::value,
                     MORE = decltype(more_tag)::value;
      const unsigned to_b = ring(sbk, 2), to_a = ring(sa, 4);   // slots of B(kt+1), A(kt+2)
      pass(first_tag, next_tag, sa * TILE, sbk * TILE - (unsigned)A_BYTES,
           [&]() { if (MORE) wait_vmcnt_mem<NIA>(); else wait_vmcnt_mem<0>(); },
           [&](int g) {
             if (NEXT && g < NIB) pinned([&]() { req_b(g, to_b); });
           },
           [&](int p) {
             if (MORE) {
#pragma unroll
               for (int q = 0; q < NIA; ++q)
                 if (((q + 1) * INNER + NIA - 1) / NIA - 1 == p) pinned([&]() { req_a(q, to_a); });
             }
           });
      if (!FIRST && NEXT) adv_b();
      if (MORE) adv_a();
      sa = ring(sa, 2);
      sbk = ring(sbk, 2);
    };
    static_assert(NIB <= MPS, "the B requests of a pass ride the MFMAs of one slice");
    step(Yes{}, Yes{}, Yes{});
    int kt = 1;
    for (; kt + 2 < nk; ++kt) step(No{}, Yes{}, Yes{});
    step(No{}, Yes{}, No{});
    step(No{}, No{}, No{});
  } else {
    // ---- ring of STAGES whole stages ------------------------------------------------------
    // Stage k sits in slot k % STAGES.  Stages 0 .. STAGES-2 are requested up front; pass kt
    // asks for stage kt+STAGES-1, spread over its inner slices, into the slot the barrier
    // before it freed, so a stage has STAGES-2 steps and more to land.
    static_assert(STAGES >= 3, "the barrier of a step certifies the next stage");
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) {
      if (s < nk) {
#pragma unroll
        for (int i = 0; i < NI; ++i) request(i, (unsigned)s * STAGE_BYTES);
        advance_k();
      }
    }
    if (nk >= STAGES - 1) wait_vmcnt_mem<(STAGES - 2) * NI>(); else wait_vmcnt_mem<0>();
    __syncthreads();
    int cur = 0;                 // ring slot of k-step kt
    int nxt = STAGES - 1;        // ring slot the requests of this pass go to
    // MORE: k-step kt+STAGES-1 exists (requested in this pass; the stages before it then all
    // exist, so the wait for stage kt+1 may leave STAGES-2 stages pending)
    auto step = [&](auto first_tag, auto next_tag, auto more_tag) {
      constexpr bool MORE = decltype(more_tag)::value;
      const unsigned sb = (unsigned)cur * STAGE_BYTES, nb = (unsigned)nxt * STAGE_BYTES;
      pass(first_tag, next_tag, sb, sb,
           [&]() { if (MORE) wait_vmcnt_mem<(STAGES - 2) * NI>(); else wait_vmcnt_mem<0>(); },
           no_req,
           [&](int p) {
             if (MORE) {
#pragma unroll
               for (int q = 0; q < NI; ++q)
                 if (((q + 1) * INNER + NI - 1) / NI - 1 == p) pinned([&]() { request(q, nb); });
             }
           });
      if (MORE) advance_k();
      cur = cur + 1 == STAGES ? 0 : cur + 1;
      nxt = nxt + 1 == STAGES ? 0 : nxt + 1;
    };
    if (nk >= STAGES) step(Yes{}, Yes{}, Yes{});
    else if (nk > 1) step(Yes{}, Yes{}, No{});
    else step(Yes{}, No{}, No{});
    int kt = 1;
    for (; kt + STAGES - 1 < nk; ++kt) step(No{}, Yes{}, Yes{});
    for (; kt + 1 < nk; ++kt) step(No{}, Yes{}, No{});
    if (kt < nk) step(No{}, No{}, No{});
  }
  // the MFMAs of the last slice of the last k-step
  __builtin_amdgcn_sched_barrier(0);
  mfma_slice(Buf1{}, no_req);

  // ---- epilogue ---------------------------------------------------------------------------
  // Accumulator element e of lane l is C[8*(e/4) + 4*(l/32) + e%4][l%32] of its 32x32 block:
  // single elements per lane, 64 contiguous bytes per row and store.  Each wave therefore
  // turns its tile through LDS, 32 rows at a time (fp32, so that bias and residual are added
  // before the one rounding): written as held, read back as runs of four columns per lane,
  // so that the global accesses are 8 bytes a lane and 256..512 contiguous bytes a row.
  // Column c of row r sits at c ^ (32 * ((r >> 2) & 1)): rows r and r+4, which one write
  // instruction touches, land in different halves of the banks.
  constexpr int LPR = WN / 4;            // lanes per row on the way out
  constexpr int RPI = 64 / LPR;          // rows per read/store instruction
  constexpr int EPI_BYTES = 32 * WN * 4; // one wave's 32 x WN fp32 block
  constexpr unsigned ESW = WN >= 64 ? 32u : 0u;   // (a 32-column block has no second half to swap with)
  static_assert(NW * EPI_BYTES <= (SPLIT ? 5 * A_BYTES : STAGES * STAGE_BYTES), "the epilogue reuses the operand stages");
  __syncthreads();                       // every wave is done with the operand stages
  unsigned char *ew = lds + (unsigned)wave * EPI_BYTES;
  const int orow = lane / LPR, oc4 = (lane % LPR) * 4;
  const unsigned lane_off = ((unsigned)orow * (unsigned)N + (unsigned)oc4) * 2u;
  // A tile that was shifted back stores only the part its unshifted position covers: the rest
  // is its neighbour's (written once, so that C may also be the residual operand).
  const int skip_rows = tm * BM - m0;
  const bool col_owned = n0 + wn + oc4 >= tn * BN;
  float bv[4] = {0.f, 0.f, 0.f, 0.f};
  if (bias != nullptr) {
    const bf16x4 b4 = *reinterpret_cast<const bf16x4 *>(bias + n0 + wn + oc4);
#pragma unroll
    for (int q = 0; q < 4; ++q) bv[q] = (float)b4[q];
  }
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    // the residual of the 32 rows, asked for before the turn through LDS and first used after it
    // (every tile lies inside the matrix, so rows and columns the tile does not own are read too)
    bf16x4 r4[32 / RPI];
    if (res != nullptr) {
#pragma unroll
      for (int g = 0; g < 32 / RPI; ++g) {
        const size_t uoff = ((size_t)(m0 + wm + i * 32 + g * RPI) * (size_t)N + (size_t)(n0 + wn)) * 2 + lane_off;
        r4[g] = *reinterpret_cast<const bf16x4 *>((const char *)res + uoff);
      }
    }
    // write: element e of block j -> row 8*(e/4) + 4*(l/32) + e%4, column 32*j + l%32
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int r = 8 * (e >> 2) + (e & 3);            // + 4*(l/32)
        const unsigned rr = (unsigned)r + 4u * (unsigned)(lane >> 5);
        const unsigned cc = (unsigned)(32 * j + (lane & 31)) ^ (ESW * ((rr >> 2) & 1u));
        *reinterpret_cast<float *>(ew + (rr * WN + cc) * 4u) = acc[i][j][e];
      }
    // read back (all reads asked for before the first is used), then store
    f32x4 tb[32 / RPI];
#pragma unroll
    for (int g = 0; g < 32 / RPI; ++g) {
      const unsigned rr = (unsigned)(g * RPI + orow);
      const unsigned cc = (unsigned)oc4 ^ (ESW * ((rr >> 2) & 1u));
      tb[g] = *reinterpret_cast<const f32x4 *>(ew + (rr * WN + cc) * 4u);
    }
#pragma unroll
    for (int g = 0; g < 32 / RPI; ++g) {
      const f32x4 t = tb[g];
      const size_t uoff = ((size_t)(m0 + wm + i * 32 + g * RPI) * (size_t)N + (size_t)(n0 + wn)) * 2 + lane_off;
      if (!col_owned || wm + i * 32 + g * RPI + orow < skip_rows) continue;
      float v[4] = {t[0] + bv[0], t[1] + bv[1], t[2] + bv[2], t[3] + bv[3]};
      if (res != nullptr) {
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] += (float)r4[g][q];
      }
      bf16x4 o;
#pragma unroll
      for (int q = 0; q < 4; ++q) o[q] = (bf16)v[q];
      *reinterpret_cast<bf16x4 *>((char *)C + uoff) = o;
      if (ACT) {
        // fused activation: computed from the value as stored, so that a later standalone
        // GELU of C gives the same bits
        bf16x4 o2;
#pragma unroll
        for (int q = 0; q < 4; ++q) o2[q] = (bf16)gelu_f((float)o[q], gelu_kind);
        *reinterpret_cast<bf16x4 *>((char *)C2 + uoff) = o2;
      }
    }
  }
}

template <int BM, int BN, int WGM, int WGN, int STAGES, bool ACT, bool TN, int BK, bool SPLIT>
hipError_t launch_dma_act(const GemmArgs &a, hipStream_t s) {
  constexpr size_t smem = SPLIT ? (size_t)5 * BM * BK * 2 : (size_t)STAGES * (BM + BN) * BK * 2;
  static_assert(smem <= 160 * 1024, "LDS of one CU");
  static bool attr_set = false;
  auto kern = gemm_dma_kernel<BM, BN, WGM, WGN, STAGES, ACT, TN, BK, SPLIT>;
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

template <int BM, int BN, int WGM, int WGN, int STAGES, bool TN, int BK = 64, bool SPLIT = false>
hipError_t launch_dma_cfg(const GemmArgs &a, hipStream_t s) {
  if (TN) return launch_dma_act<BM, BN, WGM, WGN, STAGES, false, TN, BK, SPLIT>(a, s);   // no epilogue extras in this form
  return a.C2 != nullptr ? launch_dma_act<BM, BN, WGM, WGN, STAGES, true, false, BK, SPLIT>(a, s)
                         : launch_dma_act<BM, BN, WGM, WGN, STAGES, false, false, BK, SPLIT>(a, s);
}

template <bool TN>
hipError_t launch_dma_mode(const GemmArgs &a, hipStream_t s) {
  auto tiles = [&](int bm, int bn) { return (long)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn); };
  // DPSTAGE_GEMM_TILE overrides the tile choice (tuning aid)
  static const char *force = getenv("DPSTAGE_GEMM_TILE");
  const bool big_ok = a.M >= 256 && a.N >= 256;
  if (force != nullptr) {
    if (!strcmp(force, "256x256") && big_ok && a.K >= 192) return launch_dma_cfg<256, 256, 4, 2, 2, TN, 64, true>(a, s);
    if (!strcmp(force, "128x128")) return launch_dma_cfg<128, 128, 4, 2, 4, TN>(a, s);
    if (!strcmp(force, "128x128w4")) return launch_dma_cfg<128, 128, 2, 2, 4, TN>(a, s);
    if (!strcmp(force, "64x64")) return launch_dma_cfg<64, 64, 2, 2, 8, TN>(a, s);

  }
  // 256x256 (8 waves, 64x128 a wave, ring of five operand tiles) halves the L1 traffic per
  // flop of 128x128 and wins as soon as it gives two thirds of the CUs a workgroup (measured:
  // 175 tiles, the [1600 x 6400] weight gradients, 10-20 % faster than 650 tiles of 128x128;
  // 133 and 112 tiles slower); below that 128x128 with 8 waves and a four-stage ring.
  if (big_ok && a.K >= 192 && tiles(256, 256) >= 170) return launch_dma_cfg<256, 256, 4, 2, 2, TN, 64, true>(a, s);
  // a small output with a long contraction (the out-projection weight gradient) leaves most
  // CUs without a 128x128 tile: 64x64 tiles, several workgroups a CU, then run faster
  if (tiles(128, 128) <= 96) return launch_dma_cfg<64, 64, 2, 2, 8, TN>(a, s);
  return launch_dma_cfg<128, 128, 4, 2, 4, TN>(a, s);
}

}  // namespace

bool gemm_dma_supported(const GemmArgs &a) {
  if (a.M < 128 || a.N < 128 || a.K <= 0 || a.K % kKAlign != 0) return false;
  if ((((uintptr_t)a.A | (uintptr_t)a.B) & 15) != 0) return false;
  // the epilogue moves runs of four columns (8 bytes)
  if (a.N % 4 != 0 || (((uintptr_t)a.C | (uintptr_t)a.C2 | (uintptr_t)a.res | (uintptr_t)a.bias) & 7) != 0) return false;
  // lane offsets are 32-bit
  if (a.mode == kGemmNT) return (uint64_t)a.K * 2 * 9 + 4096 <= 0xffffffffull;
  if (a.M % 8 != 0 || a.N % 8 != 0) return false;   // 16-byte rows and tile origins
  const uint64_t ld = (uint64_t)(a.M > a.N ? a.M : a.N) * 2;
  return ((uint64_t)a.K + 4) * ld + 4096 <= 0xffffffffull;
}

hipError_t launch_gemm_dma(const GemmArgs &a, hipStream_t s) {
  return a.mode == kGemmNT ? launch_dma_mode<false>(a, s) : launch_dma_mode<true>(a, s);
}

}  // namespace dp
