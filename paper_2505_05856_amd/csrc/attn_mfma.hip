// Fused softmax attention on the gfx950 matrix cores (bf16 in, fp32 accumulate).
//
// Forward: a block owns 128 query rows of one (batch, head); each of its 4 waves
// owns 32 of them.  K/V tiles of 64 keys stream through a double-buffered LDS
// stage, brought in by the load unit itself (forward; the backward kernels still
// stage their tiles through registers).  A wave computes S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so that a
// lane holds one query row's logits for 16 keys of every 32-key block: the
// softmax row reductions are in-lane plus one exchange between the two half
// waves, and the probabilities already sit in the register layout the second
// MFMA (O^T = V^T P^T) wants as its B operand.  V^T fragments come from the V
// tile as loaded ([key][d]) through the LDS transpose read.  Only O and the
// per-row log-sum-exp leave the chip; no S x S tensor is ever stored.
//
// Backward recomputes P from Q, K and the log-sum-exp, in two kernels so that
// every output element has exactly one owner (no float atomics, fixed order):
//   dK/dV: block per 128 keys (32 per wave), loops over query tiles;
//   dQ:    block per 128 queries (32 per wave), loops over key tiles.
#include "common.h"
#include "kernels.h"

#include <type_traits>

namespace dp {

namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int BKV = 64;    // keys (forward, dQ) or queries (dK/dV) per LDS stage
constexpr int BROWS = 128; // rows a block owns (4 waves x 32)

__device__ __forceinline__ uint4 ld16(const bf16 *p) { return *reinterpret_cast<const uint4 *>(p); }
__device__ __forceinline__ bf16x8 as_frag(uint4 v) {
  union { uint4 u; bf16x8 f; } c;
  c.u = v;
  return c.f;
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// elements e0..e0+7 of an MFMA result as a bf16 operand fragment
__device__ __forceinline__ bf16x8 pack8(const f32x16 &v, int e0) {
  bf16x8 r;
#pragma unroll
  for (int t = 0; t < 8; ++t) r[t] = (bf16)v[e0 + t];
  return r;
}

// Workgroups are dealt to the 8 XCDs round-robin by launch index.  This maps the launch
// index to a work index so that each XCD gets one contiguous run of work items: the
// row tiles of one (batch, head) then share K/V (or Q/dO) in a single XCD's L2
// instead of being fetched from HBM once per XCD.
__device__ __forceinline__ int xcd_contiguous(int pid, int n) {
  const int xcd = pid & 7, idx = pid >> 3, base = n >> 3, rem = n & 7;
  return xcd * base + (xcd < rem ? xcd : rem) + idx;
}

// Row index, inside its 32-row block, of element e of a 32x32 MFMA result held by `lane`.
__device__ __forceinline__ int acc_row(int e, int lane) { return 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3); }

// ---- K/V (or Q/dO) tiles brought into LDS by the load unit itself ------------------------
// One request: lane l fetches 16 bytes from uniform_base + byte_off and the unit stores them at
// LDS byte lds_base + 16*l (global_load_lds_dwordx4): no staging registers, no LDS store
// instructions, nothing to wait for until the tile is needed.  Invisible to the compiler's
// wait-count pass: the kernels wait with s_waitcnt vmcnt(0) themselves before the barrier that
// publishes a tile.  M0 is reserved by the compiler and nothing else in this file uses it.
__device__ __forceinline__ void dma16(unsigned lds_base, unsigned byte_off, const void *uniform_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_base), "v"(byte_off), "s"(uniform_base) : "m0", "memory");
}
__device__ __forceinline__ void wait_dma() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ const char *uniform_ptr(const char *p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const char *)(((uint64_t)hi << 32) | lo);
}

// A [64 rows][DH] tile in LDS, laid out for fragments whose contraction runs ALONG a row
// (frag_rows_sw): DH/64 half-tiles of [64][64] with unpadded 128-byte rows; 16-byte chunk c of
// row r sits at chunk position c ^ ((r >> 1) & 7), which spreads the 16 rows one fragment read
// phase touches over all banks.  The load unit writes 1 KB of consecutive LDS a request, so a
// lane fetches the global chunk that belongs at its LDS position: request q of the tile is rows
// 8q..8q+7 of half-tile q / 8; lane l is row 8q + l/8, position l%8.  Rows past `nrows` repeat
// the last row (their logits are masked; as values they meet probabilities that are zero).
// `ldb`: row stride of the source in bytes.  Every wave issues its DH/32 requests of the tile.
template <int DH>
__device__ __forceinline__ void dma_tile_rows(unsigned lds_byte, const char *src_col0, unsigned ldb, int row0, int nrows,
                                              int wave, int lane) {
  constexpr int NREQ = DH / 32;   // per wave: 64 * DH * 2 bytes / 1 KB / 4 waves
#pragma unroll
  for (int i = 0; i < NREQ; ++i) {
    const int q = wave * NREQ + i, half = q >> 3, r = 8 * (q & 7) + (lane >> 3);
    const int rg = min(row0 + r, nrows - 1);
    const unsigned chunk = (unsigned)((lane & 7) ^ ((r >> 1) & 7));
    dma16(lds_byte + (unsigned)q * 1024u, (unsigned)rg * ldb + (unsigned)half * 128u + chunk * 16u, src_col0);
  }
}
// fragment (32 rows from row0, contraction elements k0..k0+15) of such a tile
__device__ __forceinline__ bf16x8 frag_rows_sw(const unsigned char *tile, int row0, int k0, int lane) {
  const unsigned r = (unsigned)(row0 + (lane & 31));
  const unsigned c = (unsigned)(((k0 & 63) >> 3) + (lane >> 5));
  return *reinterpret_cast<const bf16x8 *>(tile + (unsigned)(k0 >> 6) * 8192u + r * 128u + ((c ^ ((r >> 1) & 7u)) << 4));
}

// The same tile laid out as loaded, [64 rows][DH * 2 bytes], for fragments whose contraction
// runs DOWN the rows (through the transpose read, which touches four consecutive
// rows x 64 bytes per 16 lanes): chunk c of row r sits at c ^ swz(r), swz = (r & 3) << 2 for
// 256-byte rows (the four rows land in the four 64-byte quarters of the bank period) and
// ((r >> 1) & 1) << 2 for 128-byte rows (rows r and r+2 swap 64-byte halves).
template <int DH> __device__ __forceinline__ constexpr unsigned swz_cols(unsigned r) {
  return DH == 128 ? (r & 3u) << 2 : ((r >> 1) & 1u) << 2;
}
template <int DH>
__device__ __forceinline__ void dma_tile_cols(unsigned lds_byte, const char *src_col0, unsigned ldb, int row0, int nrows,
                                              int wave, int lane) {
  constexpr int NREQ = DH / 32, RPR = 1024 / (DH * 2), CPR = DH / 8;   // rows per request, chunks per row
#pragma unroll
  for (int i = 0; i < NREQ; ++i) {
    const int q = wave * NREQ + i, r = RPR * q + lane / CPR;
    const int rg = min(row0 + r, nrows - 1);
    const unsigned chunk = (unsigned)(lane % CPR) ^ swz_cols<DH>((unsigned)r);
    dma16(lds_byte + (unsigned)q * 1024u, (unsigned)rg * ldb + chunk * 16u, src_col0);
  }
}
// fragment: lane l gets column col0 + l%32 for the rows r0 + 4*(l/32) + {0,1,2,3} and those 8 further
// (the order in which a 32x32 MFMA result holds 16 consecutive rows of one column)
template <int DH>
__device__ __forceinline__ bf16x8 frag_cols_sw(const unsigned char *tile, int r0, int col0, int lane) {
  constexpr unsigned ROWB = DH * 2;
  const unsigned i = (unsigned)(lane & 15), tt = i >> 2;
  const unsigned row = (unsigned)r0 + 4u * (unsigned)(lane >> 5) + tt;
  const unsigned cw = (unsigned)(col0 >> 3) + 2u * (unsigned)((lane >> 4) & 1) + ((i & 3u) >> 1);
  const unsigned char *p = tile + row * ROWB + ((cw ^ swz_cols<DH>(tt)) << 4) + (i & 1u) * 8u;
  union { s16x4 h[2]; bf16x8 v; } u;
  u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
  u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 8u * ROWB));
  return u.v;
}

// A [64 rows][DH] tile laid out for BOTH kinds of fragment (the backward kernels read Q, dO and
// K along the rows and down the rows): rows as loaded, chunk c of row r at position c ^ both(r),
//   256-byte rows: both(r) = ((r & 3) << 2) | ((r >> 2) & 3)    128-byte rows: (((r >> 1) & 1) << 2) | ((r >> 2) & 3)
// The high part is the column-fragment swizzle above (the four rows of a transpose read land in
// four 64-byte quarters); the low part makes the map a bijection over 16 consecutive rows, so the
// 16 rows of one row-fragment read phase cover every bank once.
template <int DH> __device__ __forceinline__ constexpr unsigned swz_both(unsigned r) {
  return swz_cols<DH>(r) | ((r >> 2) & 3u);
}
// (request i of the DH/32 a wave issues for a tile: rows past the end read the last row, so a tile
// index past the end is harmless too)
template <int DH>
__device__ __forceinline__ void dma_req_both(int i, unsigned lds_byte, const char *src_col0, unsigned ldb, int row0,
                                             int nrows, int wave, int lane) {
  constexpr int NREQ = DH / 32, RPR = 1024 / (DH * 2), CPR = DH / 8;
  const int q = wave * NREQ + i, r = RPR * q + lane / CPR;
  const int rg = min(row0 + r, nrows - 1);
  const unsigned chunk = (unsigned)(lane % CPR) ^ swz_both<DH>((unsigned)r);
  dma16(lds_byte + (unsigned)q * 1024u, (unsigned)rg * ldb + chunk * 16u, src_col0);
}
template <int DH>
__device__ __forceinline__ void dma_tile_both(unsigned lds_byte, const char *src_col0, unsigned ldb, int row0, int nrows,
                                              int wave, int lane) {
#pragma unroll
  for (int i = 0; i < DH / 32; ++i) dma_req_both<DH>(i, lds_byte, src_col0, ldb, row0, nrows, wave, lane);
}
// max / sum of a value over the two halves of the wave (lanes l and l ^ 32), in every lane: the swap
// leaves lanes 0..31 of x beside lanes 32..63 of x in both registers, in the one or the other order
// A wave's 32 x DH result (lane l holds row l % 32; accumulator element e of block d is column
// 32 d + 8 (e / 4) + 4 (l / 32) + e % 4) goes out as whole rows: a store from the accumulators would
// touch 32 rows with 16 bytes each, so the tile is turned through `ew`, 64 DH bytes of LDS that only
// this wave uses (16-byte chunk c of row r at position c ^ (r % chunks a row)), and leaves as
// 16 bytes a lane, DH / 8 lanes a row.  `mul` is the lane's (its row's) factor; rows >= nrows stay unwritten.
template <int DH>
__device__ __forceinline__ void store_rows_via_lds(unsigned char *ew, const f32x16 (&acc)[DH / 32], float mul, bf16 *dst,
                                                   long ld, int nrows, int lane) {
  constexpr int ND = DH / 32, CPR = DH / 8, RPI = 64 / CPR;
  const int row = lane & 31, hh = lane >> 5;
#pragma unroll
  for (int d = 0; d < ND; ++d)
#pragma unroll
    for (int e4 = 0; e4 < 4; ++e4) {
      bf16x4 v;
#pragma unroll
      for (int t = 0; t < 4; ++t) v[t] = (bf16)(acc[d][e4 * 4 + t] * mul);
      const int pos = (d * 4 + e4) ^ (row & (CPR - 1));
      *reinterpret_cast<bf16x4 *>(ew + row * (DH * 2) + pos * 16 + hh * 8) = v;
    }
#pragma unroll
  for (int i = 0; i < 32 / RPI; ++i) {
    const int r = i * RPI + lane / CPR, c = lane % CPR;
    const uint4 q = *reinterpret_cast<const uint4 *>(ew + r * (DH * 2) + ((c ^ (r & (CPR - 1))) * 16));
    if (r < nrows) *reinterpret_cast<uint4 *>(dst + (long)r * ld + c * 8) = q;
  }
}
__device__ __forceinline__ float halves_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
// The fragment addresses of such a tile, as LDS byte addresses a lane keeps in registers: the
// swizzle of a row depends on its low four bits only, so every fragment of the tile is one of
// these DH/16 (along the rows) + 2 * DH/32 (down the rows) addresses plus a compile-time offset
// (a multiple of 16 rows, another tile of the stage), which the read instruction carries.  The
// two stages lie a power of two apart: flip() moves every address to the other stage.
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
typedef __attribute__((address_space(3))) unsigned char lds_u8;
template <int DH>
struct BothAddr {
  static constexpr unsigned ROWB = DH * 2;
  unsigned row[DH / 16], col[2][DH / 32];
  __device__ __forceinline__ void init(int lane) {
    const unsigned r = (unsigned)(lane & 31), hh = (unsigned)(lane >> 5);
#pragma unroll
    for (int kd = 0; kd < DH / 16; ++kd) row[kd] = r * ROWB + (((2u * kd + hh) ^ swz_both<DH>(r)) << 4);
    const unsigned i = (unsigned)(lane & 15), tt = i >> 2, rc = 4u * hh + tt;
    const unsigned cl = 2u * (unsigned)((lane >> 4) & 1) + ((i & 3u) >> 1);
#pragma unroll
    for (int d = 0; d < DH / 32; ++d) {
      col[0][d] = rc * ROWB + (((4u * d + cl) ^ swz_both<DH>(rc)) << 4) + (i & 1u) * 8u;
      col[1][d] = (rc + 8u) * ROWB + (((4u * d + cl) ^ swz_both<DH>(rc + 8u)) << 4) + (i & 1u) * 8u;
    }
  }
  __device__ __forceinline__ void flip_rows(unsigned stage_bytes) {
#pragma unroll
    for (int kd = 0; kd < DH / 16; ++kd) row[kd] ^= stage_bytes;
  }
  __device__ __forceinline__ void flip_cols(unsigned stage_bytes) {
#pragma unroll
    for (int d = 0; d < DH / 32; ++d) { col[0][d] ^= stage_bytes; col[1][d] ^= stage_bytes; }
  }
  __device__ __forceinline__ void flip(unsigned stage_bytes) { flip_rows(stage_bytes); flip_cols(stage_bytes); }
  // 32 rows from row0 (a multiple of 16) of the tile at byte `tile_off` of the stage, contraction elements 16 kd ..
  // (tile_off, row0, r0, kd, d: constants once the callers' loops are unrolled)
  __device__ __forceinline__ bf16x8 rows(unsigned tile_off, int row0, int kd) const {
    return *(const lds_bf16x8 *)(uintptr_t)(row[kd] + tile_off + (unsigned)row0 * ROWB);
  }
  // column 32 d + lane % 32 for the rows r0 + 4 * (lane / 32) + {0,1,2,3} and those 8 further; r0 a multiple of 16
  __device__ __forceinline__ bf16x8 cols(unsigned tile_off, int r0, int d) const {
    union { s16x4 h[2]; bf16x8 v; } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(uintptr_t)(col[0][d] + tile_off + (unsigned)r0 * ROWB));
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(uintptr_t)(col[1][d] + tile_off + (unsigned)r0 * ROWB));
    return u.v;
  }
};

// ------------------------------------------------------------------ forward
// DROP: the probabilities are masked after the softmax (the row sums and the log-sum-exp are
// those of the plain softmax); the scale 1/(1-p) goes into the final normalisation.
template <int DH, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma_kernel(AttnView av, bf16 *__restrict__ o,
                                                               float *__restrict__ lse, int nh, float scale,
                                                               DropArgs da) {
  constexpr int ND = DH / 32, NK = DH / 16;
  // LDS, in bytes: [K even][K odd][V even][V odd], every tile in the dual-use layout; tile t of K
  // (of V) lives in the buffer of t's parity
  constexpr unsigned TILE = BKV * DH * 2, VOFF = 2 * TILE;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_b[];

  const int Sq = av.Sq, S = av.Sk;   // S: the key count, which bounds every key-side loop below
  const int nqt = (Sq + BROWS - 1) / BROWS;
  const int wid = xcd_contiguous(blockIdx.x, gridDim.x);
  const int qt = nqt - 1 - wid % nqt;   // heavy (late) causal tiles first
  const int h = (wid / nqt) % nh, b = wid / (nqt * nh);
  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int H = nh * DH;
  const long ldq = av.ldq, ld = av.ldkv;
  const bf16 *qb = (const bf16 *)av.q + (long)b * Sq * ldq + (long)h * DH;
  const char *kb = uniform_ptr((const char *)((const bf16 *)av.k + (long)b * S * ld + (long)h * DH));
  const char *vb = uniform_ptr((const char *)((const bf16 *)av.v + (long)b * S * ld + (long)h * DH));
  const unsigned ldb = (unsigned)ld * 2u;
  const int q0 = qt * BROWS, iw0 = q0 + wave * 32, qi = iw0 + (lane & 31);
  const float c = scale * kLog2e;
  const DropKeys keys = DROP ? drop_keys(da.base, (uint32_t)(b * nh + h)) : DropKeys{0u, 0u};
  const uint32_t qidx = (uint32_t)qi * (uint32_t)S;   // index of (query qi, key 0) in the head's Sq x Sk matrix

  int nkv = (S + BKV - 1) / BKV;
  if (CAUSAL) nkv = min(nkv, (min(q0 + BROWS, Sq) - 1) / BKV + 1);

  // The K stream runs one tile ahead of the V stream (the logits of tile t+1 are taken while the
  // softmax of tile t is worked out): K tiles 0 and 1 and V tile 0 are on their way while the
  // queries are fetched.
  auto fetch_k = [&](int t) { dma_tile_both<DH>((unsigned)(t & 1) * TILE, kb, ldb, t * BKV, S, wave, lane); };
  auto fetch_v = [&](int t) { dma_tile_both<DH>(VOFF + (unsigned)(t & 1) * TILE, vb, ldb, t * BKV, S, wave, lane); };
  if (nkv > 0) { fetch_k(0); fetch_v(0); }
  if (nkv > 1) fetch_k(1);

  bf16x8 qf[NK];
#pragma unroll
  for (int kd = 0; kd < NK; ++kd)   // (unguarded: a query past the end reads the last row, and nothing of it is stored)
    qf[kd] = as_frag(ld16(qb + (long)min(qi, Sq - 1) * ldq + kd * 16 + 8 * hh));

  f32x16 acc[ND];
#pragma unroll
  for (int d = 0; d < ND; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[d][e] = 0.f;
  float m = -1e30f, l = 0.f;   // m: running maximum of the scaled logits (log2 domain)

  BothAddr<DH> at;
  at.init(lane);
  wait_dma();
  // (a use of the query fragments the compiler can see, here: otherwise it places its own wait for
  // them before their first MFMA inside the tile loop, where it also waits for the tiles in flight)
#pragma unroll
  for (int kd = 0; kd < NK; ++kd) asm volatile("" ::"v"(qf[kd]));
  __syncthreads();

  // A wave runs a software pipeline of four stages a tile, so that the softmax arithmetic issues
  // beside the MFMAs instead of between them, a quarter of it in every stage (A, B: the two 32-key
  // sub-tiles of tile t; halves: 16 keys each):
  //   1: S of tile t+1, first half of the contraction (A and B: two independent chains)
  //        beside  P of the first half of A = exp2(logits - reference point m), row sums
  //   2: S of tile t+1, second half       beside  P of the second half of A
  //   3: O += P_A V_A                      beside  P of the first half of B, maximum over S_A of tile t+1
  //   4: O += P_B V_B                      beside  P of the second half of B (within the first half
  //                                                of the stage), maximum over S_B of tile t+1
  // and the reference point for tile t+1 (with the rescaling of the accumulators if it has to follow
  // the maximum) at the head of the next tile.  Every step reads the operand fragments of the step after it;
  // scheduling fences keep the steps in this order; the code of a tile has no branch inside a
  // stage (MORE = a next tile exists).  (A wave whose queries see no key of the block's last tile
  // runs it all the same, every logit masked: it would wait for the other waves at the tile
  // barrier anyway.)
  bf16x8 fx[2];                  // fragment double buffer
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
  auto ld_k = [&](int slot, int sub, int kd) { fx[slot] = at.rows(0u, sub * 32, kd); };
  auto ld_v = [&](int slot, int sub, int j) { fx[slot] = at.cols(VOFF, sub * 32 + (j / ND) * 16, j % ND); };
  auto zero = [](f32x16 &v) {
#pragma unroll
    for (int e = 0; e < 16; ++e) v[e] = 0.f;
  };
  // keys past the end and keys the causal mask hides, on the tiles that have any: -inf, P = 0
  auto mask = [&](f32x16 (&sv)[2], int j0) {
    if (j0 + BKV > S || (CAUSAL && j0 + BKV - 1 > iw0)) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int lim = (CAUSAL ? min(S, qi + 1) : S) - j0 - 32 * sub - 4 * hh;   // the lane's first hidden row
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (8 * (e >> 2) + (e & 3) >= lim) sv[sub][e] = -INFINITY;
      }
    }
  };
  f32x16 cur[2], nxt[2];   // raw logits of tile t, of tile t+1
  float mx = -INFINITY;    // maximum over the raw logits of the tile about to be worked on (this lane's keys)

  auto tile = [&](int t, auto more_tag) {
    constexpr bool MORE = decltype(more_tag)::value;
    const int j0 = t * BKV;
    mx = halves_max(mx);
    const float m_new = fmaxf(m, mx * c);   // (the scale c > 0 is folded into the exponent below)
    // The reference point m of the exponents need not be the maximum itself: O and the row sum
    // carry the same factor exp2(-m), which cancels in O / l and in the log-sum-exp.  It follows the
    // maximum only once that has moved by more than kLag for some query of the wave (P <= 2^kLag
    // until then: no loss in fp32 sums or in bf16's relative rounding), so that the rescaling of
    // the accumulators, which a maximum creeping upwards would ask for in most tiles, is rare.
    constexpr float kLag = 8.f;
    if (__builtin_amdgcn_ballot_w64(m_new > m + kLag) != 0) {
      const float alpha = fast_exp2(m - m_new);
      l *= alpha;
#pragma unroll
      for (int d = 0; d < ND; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[d][e] *= alpha;
      m = m_new;
    }
    mx = -INFINITY;
    float ps = 0.f;
    // elements e0 .. e0+n-1 of a sub-tile: logits -> P (masked by dropout after the row sum)
    auto soft = [&](f32x16 &sv, int sub, int e0, int n) {
#pragma unroll
      for (int u = 0; u < n; ++u) {
        const int e = e0 + u;
        const float pr = fast_exp2(__builtin_fmaf(sv[e], c, -m));
        ps += pr;
        sv[e] = (DROP && drop_bits(qidx + (uint32_t)(j0 + sub * 32 + acc_row(e, lane)), keys.k0, keys.k1) < da.thr)
                    ? 0.f : pr;
      }
    };
    auto vmax = [&](const f32x16 &sv, int e0, int n) {
#pragma unroll
      for (int u = 0; u < n; ++u) mx = fmaxf(mx, sv[e0 + u]);
    };
    // stages 1 and 2: NK steps of two MFMAs, 16 / NK elements of P_A a step
    if (MORE) { zero(nxt[0]); zero(nxt[1]); ld_k(0, 0, 0); ld_k(1, 1, 0); }
#pragma unroll
    for (int kd = 0; kd < NK; ++kd) {
      if (MORE) {
        // one request a step for the tiles on their way: K of tile t+2, then V of tile t+1 (every
        // wave left the buffers they go to at the barrier that ended the last tile); a burst of
        // them at the head of the tile would hold the wave at the issue of each
        if (kd < NK / 2) dma_req_both<DH>(kd, (unsigned)(t & 1) * TILE, kb, ldb, (t + 2) * BKV, S, wave, lane);
        else dma_req_both<DH>(kd - NK / 2, VOFF + (unsigned)((t + 1) & 1) * TILE, vb, ldb, (t + 1) * BKV, S, wave, lane);
        const bf16x8 ka = fx[0], kb2 = fx[1];
        if (kd + 1 < NK) { ld_k(0, 0, kd + 1); ld_k(1, 1, kd + 1); }
        nxt[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[kd], nxt[0], 0, 0, 0);
        nxt[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb2, qf[kd], nxt[1], 0, 0, 0);
      }
      if (kd + 1 == NK) ld_v(0, 0, 0);   // the first fragment of stage 3
      soft(cur[0], 0, kd * (16 / NK), 16 / NK);
      fence();
    }
    if (MORE) mask(nxt, j0 + BKV);
    bf16x8 pf[2];
    pf[0] = pack8(cur[0], 0); pf[1] = pack8(cur[0], 8);
    // stage 3: NK steps of one MFMA; 8 / NK elements of P_B and 16 / NK of the next maximum a step
#pragma unroll
    for (int j = 0; j < NK; ++j) {
      if (j + 1 < NK) ld_v((j + 1) & 1, 0, j + 1); else ld_v((j + 1) & 1, 1, 0);
      acc[j % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[j & 1], pf[j / ND], acc[j % ND], 0, 0, 0);
      if ((j * 8) % NK == 0) soft(cur[1], 1, j * 8 / NK, 8 / NK >= 1 ? 8 / NK : 1);
      if (MORE) vmax(nxt[0], j * (16 / NK), 16 / NK);
      fence();
    }
    pf[0] = pack8(cur[1], 0);
    // stage 4: the second half of P_B within the first half of the stage, then the rest of the maximum
#pragma unroll
    for (int j = 0; j < NK; ++j) {
      if (j + 1 < NK) ld_v((j + 1) & 1, 1, j + 1);
      if (j == ND) pf[1] = pack8(cur[1], 8);
      acc[j % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[j & 1], pf[j / ND], acc[j % ND], 0, 0, 0);
      if (j < ND) soft(cur[1], 1, 8 + j * (8 / ND), 8 / ND);
      else if (MORE) vmax(nxt[1], (j - ND) * (16 / ND), 16 / ND);
      fence();
    }
    l += ps;
    if (MORE) { cur[0] = nxt[0]; cur[1] = nxt[1]; }
    at.flip(TILE);
    wait_dma();        // this wave's parts of the tiles on their way are in
    __syncthreads();   // everyone's are, and everyone is done with this tile's
  };

  if (nkv > 0) {   // the logits of tile 0 and their maximum
    zero(cur[0]); zero(cur[1]);
#pragma unroll
    for (int kd = 0; kd < NK; ++kd) {
      cur[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at.rows(0u, 0, kd), qf[kd], cur[0], 0, 0, 0);
      cur[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at.rows(0u, 32, kd), qf[kd], cur[1], 0, 0, 0);
    }
    mask(cur, 0);
#pragma unroll
    for (int e = 0; e < 16; ++e) mx = fmaxf(mx, fmaxf(cur[0][e], cur[1][e]));
    at.flip_rows(TILE);   // the K fragments run one tile ahead of the V fragments
  }
  for (int t = 0; t + 1 < nkv; ++t) tile(t, std::true_type{});
  if (nkv > 0) tile(nkv - 1, std::false_type{});

  l += __shfl_xor(l, 32, 64);
  if (lse != nullptr && hh == 0 && qi < Sq) lse[((long)b * nh + h) * Sq + qi] = (m + __log2f(l)) * kLn2;
  if (o == nullptr) return;
  // (every wave is behind the last tile's barrier: nobody reads the tile buffers any more)
  const float inv = (DROP ? da.scale : 1.0f) / l;
  store_rows_via_lds<DH>(smem_b + wave * (64 * DH), acc, inv, o + ((long)b * Sq + iw0) * H + (long)h * DH, H, Sq - iw0, lane);
}

template <typename K>
hipError_t set_smem(K kern, size_t smem) {
  return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)smem);
}

template <int DH>
hipError_t fwd_launch(int B, int nh, int causal, const AttnView &av, void *o, float *lse, const DropArgs *drop,
                      hipStream_t s) {
  constexpr size_t smem = 2 * 2 * (size_t)BKV * DH * sizeof(bf16);   // two stages of a K and a V tile
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = set_smem(attn_fwd_mfma_kernel<DH, true, false>, smem);
    if (e == hipSuccess) e = set_smem(attn_fwd_mfma_kernel<DH, false, false>, smem);
    if (e == hipSuccess) e = set_smem(attn_fwd_mfma_kernel<DH, true, true>, smem);
    if (e == hipSuccess) e = set_smem(attn_fwd_mfma_kernel<DH, false, true>, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const dim3 grid(((av.Sq + BROWS - 1) / BROWS) * nh * B), block(256);
  const float scale = 1.0f / sqrtf((float)DH);
  const bool dropping = drop != nullptr && drop->thr != 0;
  const DropArgs da = dropping ? *drop : DropArgs{0u, 0u, 1.f};
#define DP_FWD(KERN) hipLaunchKernelGGL(KERN, grid, block, smem, s, av, (bf16 *)o, lse, nh, scale, da)
  if (dropping) { if (causal) DP_FWD((attn_fwd_mfma_kernel<DH, true, true>)); else DP_FWD((attn_fwd_mfma_kernel<DH, false, true>)); }
  else { if (causal) DP_FWD((attn_fwd_mfma_kernel<DH, true, false>)); else DP_FWD((attn_fwd_mfma_kernel<DH, false, false>)); }
#undef DP_FWD
  return hipGetLastError();
}

// ------------------------------------------------------------------ backward
// dK, dV: the block owns 128 keys (32 per wave) and streams 64-query tiles of Q and dO.
// (head dimension 128: both accumulators and both key-side fragments need more than the 256
// registers two blocks a CU leave each wave, and spills on this path cost more than the
// lost occupancy)
template <int DH, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(256, DH == 128 ? 1 : 2) void attn_bwd_dkv_kernel(AttnView av,
                                                              const float *__restrict__ lse,
                                                              const bf16 *__restrict__ d_o,
                                                              const float *__restrict__ drow,
                                                              int nh, float scale, DropArgs da) {
  constexpr int ND = DH / 32, NK = DH / 16;
  // stage s: Q tile, dO tile (both in the dual-use layout), then 64 log-sum-exp and 64 row-dot floats
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_b[];
  // LDS, in bytes: [stage 0: Q, dO][stage 1: Q, dO][stage 0: lse, row dots][stage 1: lse, row dots]
  constexpr unsigned TILE = BKV * DH * 2, STAGE = 2 * TILE, FBASE = 2 * STAGE, FSTAGE = 8 * BKV;

  const int Sq = av.Sq, Sk = av.Sk;
  const int nkt = (Sk + BROWS - 1) / BROWS;
  const int wid = xcd_contiguous(blockIdx.x, gridDim.x);
  const int kt = wid % nkt, h = (wid / nkt) % nh, b = wid / (nkt * nh);
  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int H = nh * DH;
  const long ldq = av.ldq, ld = av.ldkv;
  const bf16 *qb = (const bf16 *)av.q + (long)b * Sq * ldq + (long)h * DH;
  const bf16 *kb = (const bf16 *)av.k + (long)b * Sk * ld + (long)h * DH;
  const bf16 *vb = (const bf16 *)av.v + (long)b * Sk * ld + (long)h * DH;
  const bf16 *dob = d_o + (long)b * Sq * H + (long)h * DH;
  const float *lrow = lse + ((long)b * nh + h) * Sq, *drw = drow + ((long)b * nh + h) * Sq;
  const int j0 = kt * BROWS, jw0 = j0 + wave * 32, kj = jw0 + (lane & 31);
  const float c = scale * kLog2e;
  // DROP: the forward multiplied V by P' = mask * P / (1-p): dV takes P', and dP is masked and
  // scaled the same way before the softmax derivative (which is that of the plain P).
  const DropKeys keys = DROP ? drop_keys(da.base, (uint32_t)(b * nh + h)) : DropKeys{0u, 0u};

  bf16x8 kf[NK], vf[NK];
#pragma unroll
  for (int kd = 0; kd < NK; ++kd) {   // (unguarded: a key past the end reads the last row; a lane's key is a column of the
    const long kc = min(kj, Sk - 1);  //  products nobody else sees, and its dK, dV rows are not stored)
    kf[kd] = as_frag(ld16(kb + kc * ld + kd * 16 + 8 * hh));
    vf[kd] = as_frag(ld16(vb + kc * ld + kd * 16 + 8 * hh));
  }
  f32x16 dk[ND], dv[ND];
#pragma unroll
  for (int d = 0; d < ND; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dk[d][e] = 0.f; dv[d][e] = 0.f; }

  const char *qsrc = uniform_ptr((const char *)qb), *osrc = uniform_ptr((const char *)dob);
  const unsigned ldqb = (unsigned)ldq * 2u, ldob = (unsigned)H * 2u;
  // The Q and dO tiles of query tile t go straight to LDS; the two scalars per query go through a
  // register: even waves carry the 64 log-sum-exps, odd waves the 64 row dots (waves 2 and 3 store
  // what waves 0 and 1 store, to the same words, so that no wave branches here).
  // The scalar is asked for with the tile and first touched when it is stored, a tile later: a use any
  // earlier would make the wave wait there for every load in flight, the tile's own among them.
  const float *fsrc = (wave & 1) ? drw : lrow;
  const float fmul = (wave & 1) ? 1.f : kLog2e;
  const float fpad = (wave & 1) ? 0.f : INFINITY;   // +inf: P = 0 for padding rows
  float sl = 0.f;
  auto fetch = [&](int t, unsigned buf) {
    const int i0 = t * BKV;
    dma_tile_both<DH>(buf, qsrc, ldqb, i0, Sq, wave, lane);
    dma_tile_both<DH>(buf + TILE, osrc, ldob, i0, Sq, wave, lane);
    sl = fsrc[min(i0 + lane, Sq - 1)];
  };
  auto stash = [&](int t, unsigned stage) {   // [0,64): lse, [64,128): row dots
    reinterpret_cast<float *>(smem_b + FBASE + stage * FSTAGE)[tid & 127] = t * BKV + lane < Sq ? sl * fmul : fpad;
  };
  const int nq = (Sq + BKV - 1) / BKV;
  const int t0 = CAUSAL ? j0 / BKV : 0;   // query tiles before the block's first key see none of its keys
  if (t0 < nq) { fetch(t0, 0u); stash(t0, 0u); }
  BothAddr<DH> at;
  at.init(lane);
  wait_dma();
  __syncthreads();

  // One 64-query tile is two 32-query sub-tiles, A and B.  The wave runs a software pipeline of
  // four stages a tile, each NK steps of two MFMAs, so that the softmax arithmetic of one
  // sub-tile issues beside the MFMAs of the other instead of between them:
  //   1: S, dP of B              beside  P, dS of A (from the S, dP of A, taken one stage ahead)
  //   2: dV, dK += A's P, dS     beside  P, dS of B
  //   3: dV, dK += B's P, dS
  //   4: (behind the tile barrier) S, dP of A of the next tile
  // Every step reads the operand fragments of the step after it; the scheduling fences keep the
  // steps in this order.  (The sums keep their order: sub-tile A before B, contraction ascending.)
  // A tile's code has no branch: the accumulators are carried through the loop in the registers
  // the MFMAs leave them in.  Whether the causal mask can apply (MASK: the two tiles the block's
  // 128 keys share with the diagonal) and whether a tile follows (MORE) are compile-time tags; a
  // wave whose keys see no query of a diagonal tile adds zeros (it would wait at the barrier anyway).
  constexpr int EPS = 16 / NK;                       // softmax elements a step
  bf16x8 fx[2], fy[2];                               // fragment double buffer
  auto ld_rows = [&](int slot, int sub, int kd) {    // Q and dO along the rows: operands of S and dP
    fx[slot] = at.rows(0u, sub * 32, kd);
    fy[slot] = at.rows(TILE, sub * 32, kd);
  };
  auto ld_cols = [&](int slot, int sub, int j) {     // dO and Q down the rows: operands of dV and dK
    fx[slot] = at.cols(TILE, sub * 32 + (j / ND) * 16, j % ND);
    fy[slot] = at.cols(0u, sub * 32 + (j / ND) * 16, j % ND);
  };
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
  // The two scalars of the queries a softmax step works on come from LDS one step ahead as well:
  // softmax step q of a tile (q < NK: sub-tile A, else B) finds them in slot q % 2.
  const float *lds_f = reinterpret_cast<const float *>(smem_b + FBASE);   // the current tile's scalars
  float lsc[2][EPS], dsc[2][EPS];
  auto ld_soft = [&](int q) {
    const int e0 = (q % NK) * EPS, r0 = (q / NK) * 32 + 8 * (e0 >> 2) + 4 * hh + (e0 & 3);
    if constexpr (EPS == 4) {
      const float4 l4 = *reinterpret_cast<const float4 *>(lds_f + r0), d4 = *reinterpret_cast<const float4 *>(lds_f + BKV + r0);
      lsc[q & 1][0] = l4.x; lsc[q & 1][1] = l4.y; lsc[q & 1][2] = l4.z; lsc[q & 1][3] = l4.w;
      dsc[q & 1][0] = d4.x; dsc[q & 1][1] = d4.y; dsc[q & 1][2] = d4.z; dsc[q & 1][3] = d4.w;
    } else {
      const float2 l2 = *reinterpret_cast<const float2 *>(lds_f + r0), d2 = *reinterpret_cast<const float2 *>(lds_f + BKV + r0);
      lsc[q & 1][0] = l2.x; lsc[q & 1][1] = l2.y; dsc[q & 1][0] = d2.x; dsc[q & 1][1] = d2.y;
    }
  };
  f32x16 sA, dpA;
  auto logits_of_a = [&] {   // stage 4 (and the prologue); leaves the first fragments and scalars of stage 1 in flight
    ld_rows(0, 0, 0);
    ld_soft(0);
#pragma unroll
    for (int e = 0; e < 16; ++e) { sA[e] = 0.f; dpA[e] = 0.f; }
#pragma unroll
    for (int kd = 0; kd < NK; ++kd) {
      if (kd + 1 < NK) ld_rows((kd + 1) & 1, 0, kd + 1); else ld_rows((kd + 1) & 1, 1, 0);
      sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[kd & 1], kf[kd], sA, 0, 0, 0);
      dpA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[kd & 1], vf[kd], dpA, 0, 0, 0);
      fence();
    }
  };

  auto tile = [&](int t, auto mask_tag, auto more_tag) {
    constexpr bool MASK = decltype(mask_tag)::value, MORE = decltype(more_tag)::value;
    const unsigned cur = (unsigned)((t - t0) & 1), nxt = cur ^ 1u;   // stages
    const int i0 = t * BKV;
    if (MORE) fetch(t + 1, nxt * STAGE);   // (every wave left that stage at the barrier below)
    // softmax step q, elements e0 .. e0+EPS-1 of a sub-tile: logits -> P (or P' under dropout), dP -> dS
    auto soft = [&](f32x16 &sv, f32x16 &dpv, int q) {
      const int sub = q / NK, e0 = (q % NK) * EPS;
      const int r0 = sub * 32 + 8 * (e0 >> 2) + 4 * hh + (e0 & 3);
#pragma unroll
      for (int u = 0; u < EPS; ++u) {
        const int e = e0 + u, i = i0 + r0 + u;
        const float l = lsc[q & 1][u], dd = dsc[q & 1][u];
        const float pr = fast_exp2(sv[e] * c - l);   // (rows past the end carry lse = +inf: p = 0 by itself)
        if (DROP) {
          const bool keep = drop_bits((uint32_t)i * (uint32_t)Sk + (uint32_t)kj, keys.k0, keys.k1) >= da.thr;
          sv[e] = keep ? pr * da.scale : 0.f;
          dpv[e] = pr * ((keep ? dpv[e] * da.scale : 0.f) - dd);
        } else {
          sv[e] = pr;
          dpv[e] = pr * (dpv[e] - dd);
        }
      }
    };
    // the causal mask: a masked logit becomes -inf, its P zero
    auto mask = [&](f32x16 &sv, int sub) {
      if (MASK) {
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (kj > i0 + sub * 32 + acc_row(e, lane)) sv[e] = -INFINITY;
      }
    };
    f32x16 sB, dpB;
#pragma unroll
    for (int e = 0; e < 16; ++e) { sB[e] = 0.f; dpB[e] = 0.f; }
    mask(sA, 0);
#pragma unroll
    for (int kd = 0; kd < NK; ++kd) {   // stage 1
      if (kd + 1 < NK) ld_rows((kd + 1) & 1, 1, kd + 1); else ld_cols((kd + 1) & 1, 0, 0);
      ld_soft(kd + 1);
      sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[kd & 1], kf[kd], sB, 0, 0, 0);
      dpB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[kd & 1], vf[kd], dpB, 0, 0, 0);
      soft(sA, dpA, kd);
      fence();
    }
    bf16x8 pf[2], dsf[2];
    pf[0] = pack8(sA, 0); pf[1] = pack8(sA, 8); dsf[0] = pack8(dpA, 0); dsf[1] = pack8(dpA, 8);
    mask(sB, 1);
#pragma unroll
    for (int j = 0; j < NK; ++j) {      // stage 2
      if (j + 1 < NK) ld_cols((j + 1) & 1, 0, j + 1); else ld_cols((j + 1) & 1, 1, 0);
      if (j + 1 < NK) ld_soft(NK + j + 1);
      dv[j % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[j & 1], pf[j / ND], dv[j % ND], 0, 0, 0);
      dk[j % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[j & 1], dsf[j / ND], dk[j % ND], 0, 0, 0);
      soft(sB, dpB, NK + j);
      fence();
    }
    pf[0] = pack8(sB, 0); pf[1] = pack8(sB, 8); dsf[0] = pack8(dpB, 0); dsf[1] = pack8(dpB, 8);
#pragma unroll
    for (int j = 0; j < NK; ++j) {      // stage 3
      if (j + 1 < NK) ld_cols((j + 1) & 1, 1, j + 1);
      dv[j % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[j & 1], pf[j / ND], dv[j % ND], 0, 0, 0);
      dk[j % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[j & 1], dsf[j / ND], dk[j % ND], 0, 0, 0);
      fence();
    }
    if (MORE) stash(t + 1, nxt);
    at.flip(STAGE);
    lds_f = reinterpret_cast<const float *>(smem_b + FBASE + nxt * FSTAGE);
    wait_dma();
    __syncthreads();
    if (MORE) logits_of_a();   // stage 4
  };
  if (t0 < nq) {
    logits_of_a();
    int t = t0;
    if (CAUSAL) {   // the tiles that hold the diagonal for some of the block's keys
      for (; t < t0 + BROWS / BKV && t + 1 < nq; ++t) tile(t, std::true_type{}, std::true_type{});
      if (t < t0 + BROWS / BKV) { tile(t, std::true_type{}, std::false_type{}); ++t; }
    }
    for (; t + 1 < nq; ++t) tile(t, std::false_type{}, std::true_type{});
    if (t < nq) tile(t, std::false_type{}, std::false_type{});
  }

  // (every wave is behind the last tile's barrier, or there was no tile: nobody reads the tile buffers any more)
  const long out0 = ((long)b * Sk + jw0) * ld + (long)h * DH;
  store_rows_via_lds<DH>(smem_b + wave * (128 * DH), dk, scale, (bf16 *)av.dk + out0, ld, Sk - jw0, lane);
  store_rows_via_lds<DH>(smem_b + wave * (128 * DH) + 64 * DH, dv, 1.f, (bf16 *)av.dv + out0, ld, Sk - jw0, lane);
}

// dQ: the block owns 128 queries (32 per wave) and streams 64-key tiles of K and V.  It also takes
// D_i = <dO_i, O_i> over the head's columns for its queries (a lane holds half of dO_i as MFMA
// operand already) and leaves it in drow[b, h, i] for the dK/dV kernel, which is launched after it.
template <int DH, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_kernel(AttnView av,
                                                             const float *__restrict__ lse,
                                                             const bf16 *__restrict__ o,
                                                             const bf16 *__restrict__ d_o,
                                                             float *__restrict__ drow,
                                                             int nh, float scale, DropArgs da) {
  constexpr int ND = DH / 32, NK = DH / 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_b[];
  // LDS, in bytes: [stage 0: K, V][stage 1: K, V], every tile in the dual-use layout
  constexpr unsigned TILE = BKV * DH * 2, STAGE = 2 * TILE;

  const int Sq = av.Sq, S = av.Sk;   // S: the key count
  const int nqt = (Sq + BROWS - 1) / BROWS;
  const int wid = xcd_contiguous(blockIdx.x, gridDim.x);
  const int qt = nqt - 1 - wid % nqt;
  const int h = (wid / nqt) % nh, b = wid / (nqt * nh);
  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int H = nh * DH;
  const long ldq = av.ldq, ld = av.ldkv;
  const bf16 *qb = (const bf16 *)av.q + (long)b * Sq * ldq + (long)h * DH;
  const bf16 *kb = (const bf16 *)av.k + (long)b * S * ld + (long)h * DH;
  const bf16 *vb = (const bf16 *)av.v + (long)b * S * ld + (long)h * DH;
  const bf16 *dob = d_o + (long)b * Sq * H + (long)h * DH;
  const int q0 = qt * BROWS, iw0 = q0 + wave * 32, qi = iw0 + (lane & 31);
  const float c = scale * kLog2e;

  int nkv = (S + BKV - 1) / BKV;
  if (CAUSAL) nkv = min(nkv, (min(q0 + BROWS, Sq) - 1) / BKV + 1);
  const char *ksrc = uniform_ptr((const char *)kb), *vsrc = uniform_ptr((const char *)vb);
  const unsigned ldb = (unsigned)ld * 2u;
  auto fetch = [&](int t, unsigned buf) {
    dma_tile_both<DH>(buf, ksrc, ldb, t * BKV, S, wave, lane);
    dma_tile_both<DH>(buf + TILE, vsrc, ldb, t * BKV, S, wave, lane);
  };
  // the first K and V tiles are on their way while the queries' operands are fetched (and the row
  // dots, which need them, are taken)
  if (nkv > 0) fetch(0, 0u);

  // (no guards around these loads: the compiler would wait for each on its own; a query past the end
  // reads the last row, and its lse = +inf makes every P of it zero)
  const bf16 *ob = o + (long)b * Sq * H + (long)h * DH;
  const long qc = min(qi, Sq - 1);
  bf16x8 qf[NK], gf[NK], of[NK];
#pragma unroll
  for (int kd = 0; kd < NK; ++kd) {
    qf[kd] = as_frag(ld16(qb + qc * ldq + kd * 16 + 8 * hh));
    gf[kd] = as_frag(ld16(dob + qc * H + kd * 16 + 8 * hh));
    of[kd] = as_frag(ld16(ob + qc * H + kd * 16 + 8 * hh));
  }
  float dsum = 0.f;
#pragma unroll
  for (int kd = 0; kd < NK; ++kd)
#pragma unroll
    for (int i = 0; i < 8; ++i) dsum += (float)of[kd][i] * (float)gf[kd][i];
  const float dq_i = dsum + __shfl_xor(dsum, 32, 64);   // the two halves of the row
  if (qi < Sq && hh == 0) drow[((long)b * nh + h) * Sq + qi] = dq_i;
  const DropKeys keys = DROP ? drop_keys(da.base, (uint32_t)(b * nh + h)) : DropKeys{0u, 0u};
  const uint32_t qidx = (uint32_t)qi * (uint32_t)S;
  const float lq = qi < Sq ? lse[((long)b * nh + h) * Sq + qi] * kLog2e : INFINITY;

  f32x16 dq[ND];
#pragma unroll
  for (int d = 0; d < ND; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[d][e] = 0.f;

  BothAddr<DH> at;
  at.init(lane);
  wait_dma();
  __syncthreads();

  // The same four-stage pipeline as the dK/dV kernel, over the two 32-key sub-tiles A and B of a
  // 64-key tile:  1: S, dP of B beside dS of A;  2: dQ += dS_A K beside dS of B;  3: dQ += dS_B K;
  // 4: (behind the tile barrier) S, dP of A of the next tile.  Stages 2 and 3 have one MFMA a step.
  constexpr int EPS = 16 / NK;
  bf16x8 fx[2], fy[2];
  auto ld_rows = [&](int slot, int sub, int kd) {   // K and V along the rows: operands of S and dP
    fx[slot] = at.rows(0u, sub * 32, kd);
    fy[slot] = at.rows(TILE, sub * 32, kd);
  };
  auto ld_cols = [&](int slot, int sub, int j) {    // K down the rows: operand of dQ
    fx[slot] = at.cols(0u, sub * 32 + (j / ND) * 16, j % ND);
  };
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
  // (A wave whose queries see no key of the block's last tile runs it all the same, every logit
  // masked: it would wait for the other waves at the tile barrier anyway.)
  f32x16 sA, dpA;
  auto logits_of_a = [&] {
    ld_rows(0, 0, 0);
#pragma unroll
    for (int e = 0; e < 16; ++e) { sA[e] = 0.f; dpA[e] = 0.f; }
#pragma unroll
    for (int kd = 0; kd < NK; ++kd) {
      if (kd + 1 < NK) ld_rows((kd + 1) & 1, 0, kd + 1); else ld_rows((kd + 1) & 1, 1, 0);
      sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[kd & 1], qf[kd], sA, 0, 0, 0);
      dpA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[kd & 1], gf[kd], dpA, 0, 0, 0);
      fence();
    }
  };
  if (nkv > 0) logits_of_a();

  for (int t = 0; t < nkv; ++t) {
    const int j0 = t * BKV;
    if (t + 1 < nkv) fetch(t + 1, (unsigned)((t & 1) ^ 1) * STAGE);   // (every wave left that stage at the barrier below)
    {
      // keys past the end and keys the causal mask hides, on the sub-tiles that have any: the
      // logit becomes -inf, its P zero
      auto mask = [&](f32x16 &sv, int sub) {
        const int jb = j0 + 32 * sub;
        if (jb + 32 > S || (CAUSAL && jb + 31 > iw0)) {
          const int lim = (CAUSAL ? min(S, qi + 1) : S) - jb - 4 * hh;   // the lane's first hidden row of the sub-tile
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (8 * (e >> 2) + (e & 3) >= lim) sv[e] = -INFINITY;
        }
      };
      // elements e0 .. e0+EPS-1 of a sub-tile: logits -> P, dP -> dS
      auto soft = [&](f32x16 &sv, f32x16 &dpv, int sub, int e0) {
#pragma unroll
        for (int u = 0; u < EPS; ++u) {
          const int e = e0 + u;
          const float pr = fast_exp2(sv[e] * c - lq);   // (queries past the end carry lse = +inf: p = 0)
          if (DROP) {
            const bool keep =
                drop_bits(qidx + (uint32_t)(j0 + sub * 32 + acc_row(e, lane)), keys.k0, keys.k1) >= da.thr;
            dpv[e] = pr * ((keep ? dpv[e] * da.scale : 0.f) - dq_i);
          } else {
            dpv[e] = pr * (dpv[e] - dq_i);
          }
        }
      };
      f32x16 sB, dpB;
#pragma unroll
      for (int e = 0; e < 16; ++e) { sB[e] = 0.f; dpB[e] = 0.f; }
      mask(sA, 0);
#pragma unroll
      for (int kd = 0; kd < NK; ++kd) {   // stage 1
        if (kd + 1 < NK) ld_rows((kd + 1) & 1, 1, kd + 1); else ld_cols((kd + 1) & 1, 0, 0);
        sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[kd & 1], qf[kd], sB, 0, 0, 0);
        dpB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[kd & 1], gf[kd], dpB, 0, 0, 0);
        soft(sA, dpA, 0, kd * EPS);
        fence();
      }
      bf16x8 dsf[2];
      dsf[0] = pack8(dpA, 0); dsf[1] = pack8(dpA, 8);
      mask(sB, 1);
#pragma unroll
      for (int j = 0; j < NK; ++j) {      // stage 2
        if (j + 1 < NK) ld_cols((j + 1) & 1, 0, j + 1); else ld_cols((j + 1) & 1, 1, 0);
        dq[j % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[j & 1], dsf[j / ND], dq[j % ND], 0, 0, 0);
        soft(sB, dpB, 1, j * EPS);
        fence();
      }
      dsf[0] = pack8(dpB, 0); dsf[1] = pack8(dpB, 8);
#pragma unroll
      for (int j = 0; j < NK; ++j) {      // stage 3
        if (j + 1 < NK) ld_cols((j + 1) & 1, 1, j + 1);
        dq[j % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[j & 1], dsf[j / ND], dq[j % ND], 0, 0, 0);
        fence();
      }
    }
    at.flip(STAGE);
    wait_dma();
    __syncthreads();
    if (t + 1 < nkv) logits_of_a();   // stage 4
  }

  // (every wave is behind the last tile's barrier: nobody reads the tile buffers any more)
  store_rows_via_lds<DH>(smem_b + wave * (64 * DH), dq, scale, (bf16 *)av.dq + ((long)b * Sq + iw0) * ldq + (long)h * DH,
                         ldq, Sq - iw0, lane);
}

template <int DH>
hipError_t bwd_launch(int B, int nh, int causal, const AttnView &av, const void *o, const float *lse,
                      const void *d_o, float *ws, const DropArgs *drop, hipStream_t s) {
  constexpr size_t smem_kv = 2 * (2 * (size_t)BKV * DH * sizeof(bf16) + 2 * BKV * sizeof(float));   // Q, dO; lse, row dots
  constexpr size_t smem_q = 2 * 2 * (size_t)BKV * DH * sizeof(bf16);                                 // K, V
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = set_smem(attn_bwd_dkv_kernel<DH, true, false>, smem_kv);
    if (e == hipSuccess) e = set_smem(attn_bwd_dkv_kernel<DH, false, false>, smem_kv);
    if (e == hipSuccess) e = set_smem(attn_bwd_dkv_kernel<DH, true, true>, smem_kv);
    if (e == hipSuccess) e = set_smem(attn_bwd_dkv_kernel<DH, false, true>, smem_kv);
    if (e == hipSuccess) e = set_smem(attn_bwd_dq_kernel<DH, true, false>, smem_q);
    if (e == hipSuccess) e = set_smem(attn_bwd_dq_kernel<DH, false, false>, smem_q);
    if (e == hipSuccess) e = set_smem(attn_bwd_dq_kernel<DH, true, true>, smem_q);
    if (e == hipSuccess) e = set_smem(attn_bwd_dq_kernel<DH, false, true>, smem_q);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipError_t e = hipSuccess;
  const dim3 grid_q(((av.Sq + BROWS - 1) / BROWS) * nh * B), grid_k(((av.Sk + BROWS - 1) / BROWS) * nh * B), block(256);
  const float scale = 1.0f / sqrtf((float)DH);
  const bool dropping = drop != nullptr && drop->thr != 0;
  const DropArgs da = dropping ? *drop : DropArgs{0u, 0u, 1.f};
#define DP_BWD(KERN, GRID, SMEM, ...)                                                                   \
  hipLaunchKernelGGL(KERN, GRID, block, SMEM, s, av, lse, __VA_ARGS__ (const bf16 *)d_o, ws, nh, scale, da)
#define DP_BWD4(NAME, GRID, SMEM, ...)                                                                  \
  if (dropping) { if (causal) DP_BWD((NAME<DH, true, true>), GRID, SMEM, __VA_ARGS__); else DP_BWD((NAME<DH, false, true>), GRID, SMEM, __VA_ARGS__); } \
  else { if (causal) DP_BWD((NAME<DH, true, false>), GRID, SMEM, __VA_ARGS__); else DP_BWD((NAME<DH, false, false>), GRID, SMEM, __VA_ARGS__); }
  // dQ first: it leaves the row dots <dO_i, O_i> in `ws`, which the dK/dV kernel reads
  if (av.Sq > 0 && av.Sk > 0) { DP_BWD4(attn_bwd_dq_kernel, grid_q, smem_q, (const bf16 *)o,) }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (av.Sk > 0) { DP_BWD4(attn_bwd_dkv_kernel, grid_k, smem_kv, ) }   // (no queries: dK = dV = 0 is still written)
#undef DP_BWD4
#undef DP_BWD
  return hipGetLastError();
}

}  // namespace

bool attn_mfma_supported(int S, int dh) { return S >= 1 && (dh == 64 || dh == 128); }

// The tile loads take 16 bytes a lane at 32-bit byte offsets from a head's first row.
static bool view_ok(const AttnView &v) {
  const uintptr_t ptrs = (uintptr_t)v.q | (uintptr_t)v.k | (uintptr_t)v.v;
  if ((ptrs & 15) != 0 || v.ldq % 8 != 0 || v.ldkv % 8 != 0) return false;
  const uint64_t lim = 0xffffffffull - 4096;
  return (uint64_t)v.Sk * (uint64_t)v.ldkv * 2 < lim && (uint64_t)v.Sq * (uint64_t)v.ldq * 2 < lim;
}

hipError_t launch_attn_fwd_mfma_view(int B, int nh, int dh, int causal, const AttnView &v, void *o, float *lse,
                                     hipStream_t s, const DropArgs *drop) {
  if ((causal && v.Sq != v.Sk) || !view_ok(v) || ((uintptr_t)o & 15) != 0) return hipErrorInvalidValue;
  if ((long)B * v.Sq * nh == 0) return hipSuccess;   // (no keys: the caller's case, there is no softmax to take)
  return dh == 64 ? fwd_launch<64>(B, nh, causal, v, o, lse, drop, s) : fwd_launch<128>(B, nh, causal, v, o, lse, drop, s);
}

hipError_t launch_attn_bwd_mfma_view(int B, int nh, int dh, int causal, const AttnView &v, const void *o,
                                     const float *lse, const void *d_o, float *ws, hipStream_t s,
                                     const DropArgs *drop) {
  const uintptr_t outs = (uintptr_t)v.dq | (uintptr_t)v.dk | (uintptr_t)v.dv;   // (rows leave as 16 bytes a lane)
  if ((causal && v.Sq != v.Sk) || !view_ok(v) || (((uintptr_t)d_o | outs) & 15) != 0) return hipErrorInvalidValue;
  if ((long)B * nh == 0 || (v.Sq == 0 && v.Sk == 0)) return hipSuccess;
  return dh == 64 ? bwd_launch<64>(B, nh, causal, v, o, lse, d_o, ws, drop, s)
                  : bwd_launch<128>(B, nh, causal, v, o, lse, d_o, ws, drop, s);
}

hipError_t launch_attn_fwd_mfma(int B, int S, int nh, int dh, int causal, const void *qkv, void *o, float *lse,
                                hipStream_t s, const DropArgs *drop) {
  return launch_attn_fwd_mfma_view(B, nh, dh, causal, attn_self_view(qkv, nullptr, S, nh * dh, sizeof(bf16)), o, lse, s,
                                   drop);
}

hipError_t launch_attn_bwd_mfma(int B, int S, int nh, int dh, int causal, const void *qkv, const void *o,
                                const float *lse, const void *d_o, void *dqkv, float *ws, hipStream_t s,
                                const DropArgs *drop) {
  return launch_attn_bwd_mfma_view(B, nh, dh, causal, attn_self_view(qkv, dqkv, S, nh * dh, sizeof(bf16)), o, lse, d_o,
                                   ws, s, drop);
}

}  // namespace dp
