// HBM-bound kernels of the stage step: LayerNorm forward/backward, GELU
// forward/backward, column sums (bias gradients), transposes, fills.
//
// LayerNorm works one wavefront per row: a lane owns the same 8-element column
// groups in every row, so the row statistics are wave reductions and the
// dgamma/dbeta column sums accumulate in registers over the rows a block
// visits.  Cross-row reductions are two-pass and ordered (no float atomics), so
// results do not depend on scheduling.
#include "common.h"
#include "kernels.h"

#include <mutex>

#include <type_traits>

namespace dp {

// ------------------------------------------------------------------ LayerNorm
template <typename T, int NC>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T *__restrict__ x, const T *__restrict__ gamma,
                                                     const T *__restrict__ beta, T *__restrict__ y,
                                                     float *__restrict__ stats, int rows, int cols, float eps,
                                                     int rms) {
  // rms: no mean is subtracted (y = gamma * x / sqrt(mean(x^2) + eps) + beta); the statistics then
  // hold 0 where the mean would be, which is all the backward needs to know about it
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T *xr = x + (size_t)row * cols;
  float v[NC][8];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int col = (c * 64 + lane) * 8;
    if (col < cols) {
      load8(xr + col, v[c]);
#pragma unroll
      for (int i = 0; i < 8; ++i) sum += v[c][i];
    }
  }
  const float inv_n = 1.0f / (float)cols;
  const float mean = rms ? 0.f : wave_sum(sum) * inv_n;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int col = (c * 64 + lane) * 8;
    if (col < cols) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float d = v[c][i] - mean;
        sq += d * d;
      }
    }
  }
  const float var = wave_sum(sq) * inv_n;
  const float rstd = 1.0f / sqrtf(var + eps);
  if (stats != nullptr && lane == 0) {
    stats[2 * (size_t)row] = mean;
    stats[2 * (size_t)row + 1] = rstd;
  }
  if (y == nullptr) return;
  T *yr = y + (size_t)row * cols;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int col = (c * 64 + lane) * 8;
    if (col < cols) {
      float g[8], b[8], o[8];
      load8(gamma + col, g);
      load8(beta + col, b);
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = g[i] * ((v[c][i] - mean) * rstd) + b[i];
      store8(yr + col, o);
    }
  }
}

// Pass 1 of LayerNorm backward.  Block b handles rows [b*rpb, (b+1)*rpb), one
// wave per row; writes dx and the block's partial row (dgamma | dbeta [| colsum(dx)])
// into part[b][NV*cols], NV = 3 with SUMDX (the column sums of the stored dx are the
// bias gradient of the linear layer that produced LayerNorm's input).
// AHEAD: a wave asks for its next row while it works on the current one (pays when a wave has
// several rows; with two rows a wave the registers it takes cost more than it returns).
template <typename T, int NC, bool SUMDX, bool AHEAD>
__global__ __launch_bounds__(256) void ln_bwd_kernel(const T *dy /* may alias dx */, const T *__restrict__ x,
                                                     const float *__restrict__ stats, const T *__restrict__ gamma,
                                                     const T *__restrict__ dres, T *dx,
                                                     float *__restrict__ part, int rows, int cols, int rpb, int rms) {
  // rms: the forward subtracted no mean (its statistics say mean = 0), so the term that carries the
  // derivative of the mean, mean(g), drops out: dx = rstd (g - xhat mean(g xhat))
  constexpr int NV = SUMDX ? 3 : 2;
  __shared__ float red[4][NV][512];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row_end = min(rows, (int)(blockIdx.x + 1) * rpb);
  float dg[NC][8], db[NC][8], ds[SUMDX ? NC : 1][8];
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int i = 0; i < 8; ++i) { dg[c][i] = 0.f; db[c][i] = 0.f; if (SUMDX) ds[c][i] = 0.f; }
  const float inv_n = 1.0f / (float)cols;
  // Up to 2048 columns the row stays in registers between the row reductions and the output;
  // wider rows are read twice (the second time out of the caches): there the column
  // accumulators alone take 16..24 registers per 512 columns, and occupancy is what hides
  // the latency (measured: 4096 columns 1.6 instead of 2.0 ms for the 8 launches of a step;
  // 1024 and 1600 columns the other way round).  Same arithmetic, same order, either way.
  if constexpr (NC <= 4 && AHEAD) {
    // Everything a row needs from memory (x, dy, its statistics, the residual gradient) is asked
    // for while the row before it is being worked on and waits in registers as loaded, so a row
    // costs the wave one trip to memory that overlaps the previous row's work, instead of two in
    // a row (inputs, then the residual gradient).  gamma stays in registers for all rows.
    Raw8<T> xr[NC], dr[NC], rr[NC], gr[NC];
    float mean_n = 0.f, rstd_n = 0.f;
    auto fetch = [&](int row) {
      if (row >= row_end) return;
      const size_t base = (size_t)row * cols;
      mean_n = stats[2 * (size_t)row];
      rstd_n = stats[2 * (size_t)row + 1];
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int col = (c * 64 + lane) * 8;
        if (col < cols) {
          xr[c].load(x + base + col);
          dr[c].load(dy + base + col);
        }
      }
    };
    auto fetch_res = [&](int row) {   // (after the row before it has used its own: one buffer does)
      if (dres == nullptr || row >= row_end) return;
      const size_t base = (size_t)row * cols;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int col = (c * 64 + lane) * 8;
        if (col < cols) rr[c].load(dres + base + col);
      }
    };
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int col = (c * 64 + lane) * 8;
      if (col < cols) gr[c].load(gamma + col);
    }
    fetch(blockIdx.x * rpb + wave);
    fetch_res(blockIdx.x * rpb + wave);
    for (int row = blockIdx.x * rpb + wave; row < row_end; row += 4) {
      const float mean = mean_n, rstd = rstd_n;
      const size_t base = (size_t)row * cols;
      float xh[NC][8], g[NC][8];
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int col = (c * 64 + lane) * 8;
        if (col < cols) {
          float d[8], gm[8];
          xr[c].unpack(xh[c]);
          dr[c].unpack(d);
          gr[c].unpack(gm);
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            xh[c][i] = (xh[c][i] - mean) * rstd;
            dg[c][i] += d[i] * xh[c][i];
            db[c][i] += d[i];
            g[c][i] = d[i] * gm[i];
            s1 += g[c][i];
            s2 += g[c][i] * xh[c][i];
          }
        }
      }
      fetch(row + 4);   // the wave's next row (another row of dy: the store below cannot touch it)
      const float m1 = rms ? 0.f : wave_sum(s1) * inv_n, m2 = wave_sum(s2) * inv_n;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int col = (c * 64 + lane) * 8;
        if (col < cols) {
          float o[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) o[i] = rstd * (g[c][i] - m1 - xh[c][i] * m2);
          if (dres != nullptr) {
            float r[8];
            rr[c].unpack(r);
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] += r[i];
          }
          store8(dx + base + col, o);
          if (SUMDX) {
#pragma unroll
            for (int i = 0; i < 8; ++i) ds[c][i] += (float)(T)o[i];   // the value as stored
          }
        }
      }
      fetch_res(row + 4);
    }
  } else if constexpr (NC <= 4) {
    for (int row = blockIdx.x * rpb + wave; row < row_end; row += 4) {
      const float mean = stats[2 * (size_t)row], rstd = stats[2 * (size_t)row + 1];
      const size_t base = (size_t)row * cols;
      float xh[NC][8], g[NC][8];
      float s1 = 0.f, s2 = 0.f;
  #pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int col = (c * 64 + lane) * 8;
        if (col < cols) {
          float d[8], gm[8];
          load8(x + base + col, xh[c]);
          load8(dy + base + col, d);
          load8(gamma + col, gm);
  #pragma unroll
          for (int i = 0; i < 8; ++i) {
            xh[c][i] = (xh[c][i] - mean) * rstd;
            dg[c][i] += d[i] * xh[c][i];
            db[c][i] += d[i];
            g[c][i] = d[i] * gm[i];
            s1 += g[c][i];
            s2 += g[c][i] * xh[c][i];
          }
        }
      }
      const float m1 = rms ? 0.f : wave_sum(s1) * inv_n, m2 = wave_sum(s2) * inv_n;
  #pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int col = (c * 64 + lane) * 8;
        if (col < cols) {
          float o[8];
  #pragma unroll
          for (int i = 0; i < 8; ++i) o[i] = rstd * (g[c][i] - m1 - xh[c][i] * m2);
          if (dres != nullptr) {
            float r[8];
            load8(dres + base + col, r);
  #pragma unroll
            for (int i = 0; i < 8; ++i) o[i] += r[i];
          }
          store8(dx + base + col, o);
          if (SUMDX) {
  #pragma unroll
            for (int i = 0; i < 8; ++i) ds[c][i] += (float)(T)o[i];   // the value as stored
          }
        }
      }
    }
  } else {
    for (int row = blockIdx.x * rpb + wave; row < row_end; row += 4) {
      const float mean = stats[2 * (size_t)row], rstd = stats[2 * (size_t)row + 1];
      const size_t base = (size_t)row * cols;
        float s1 = 0.f, s2 = 0.f;
  #pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int col = (c * 64 + lane) * 8;
        if (col < cols) {
          float xh[8], d[8], gm[8];
          load8(x + base + col, xh);
          load8(dy + base + col, d);
          load8(gamma + col, gm);
  #pragma unroll
          for (int i = 0; i < 8; ++i) {
            xh[i] = (xh[i] - mean) * rstd;
            dg[c][i] += d[i] * xh[i];
            db[c][i] += d[i];
            const float g = d[i] * gm[i];
            s1 += g;
            s2 += g * xh[i];
          }
        }
      }
      const float m1 = rms ? 0.f : wave_sum(s1) * inv_n, m2 = wave_sum(s2) * inv_n;
  #pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int col = (c * 64 + lane) * 8;
        if (col < cols) {
          float xh[8], d[8], gm[8], o[8];
          load8(x + base + col, xh);
          load8(dy + base + col, d);
          load8(gamma + col, gm);
  #pragma unroll
          for (int i = 0; i < 8; ++i) {
            xh[i] = (xh[i] - mean) * rstd;
            o[i] = rstd * (d[i] * gm[i] - m1 - xh[i] * m2);
          }
          if (dres != nullptr) {
            float r[8];
            load8(dres + base + col, r);
  #pragma unroll
            for (int i = 0; i < 8; ++i) o[i] += r[i];
          }
          store8(dx + base + col, o);
          if (SUMDX) {
  #pragma unroll
            for (int i = 0; i < 8; ++i) ds[c][i] += (float)(T)o[i];   // the value as stored
          }
        }
      }
    }
  }
  // ordered block reduction of the four waves' column partials, 512 columns at a time
  float *prow = part + (size_t)blockIdx.x * NV * cols;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    if (c * 512 >= cols) break;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      red[wave][0][lane * 8 + i] = dg[c][i];
      red[wave][1][lane * 8 + i] = db[c][i];
      if (SUMDX) red[wave][NV - 1][lane * 8 + i] = ds[c][i];
    }
    __syncthreads();
    for (int j = threadIdx.x; j < NV * 512; j += 256) {
      const int which = j >> 9, k = j & 511;
      const int col = c * 512 + k;
      if (col < cols) {
        const float t = ((red[0][which][k] + red[1][which][k]) + red[2][which][k]) + red[3][which][k];
        prow[(size_t)which * cols + col] = t;
      }
    }
  }
}

// LayerNorm backward for wide rows (more than 2048 columns): a block per row, the columns
// dealt out over its 256 threads (thread t owns the 8-column groups t, t + 256, ...), rows of
// the block's range one after the other.  A thread's column accumulators are then complete sums
// over the block's rows (no reduction across waves at the end), gamma stays in registers, and a
// thread holds 16..32 elements of a row instead of 64..128: several blocks fit a CU where the
// wave-per-row form fits one or two waves a SIMD.  The two row sums cross the waves through LDS
// (one barrier a row; two alternating slots); the next row's loads are issued before that.
// FULL: the row is exactly NP * 2048 columns wide, every block has a multiple of four rows and RES
// says whether there is a residual gradient, so the row loop has no branch in it.  (With branches around the loads the compiler
// can no longer count which of the loads in flight a use needs and waits for all of them, which
// leaves one row in flight instead of PF.)  Rows past the block's range are then fetched as
// copies of its last row and never used.
template <typename T, int NP, bool SUMDX, bool FULL, bool RES>
__global__ __launch_bounds__(256) void ln_bwd_wide_kernel(const T *dy /* may alias dx */, const T *__restrict__ x,
                                                          const float *__restrict__ stats,
                                                          const T *__restrict__ gamma, const T *__restrict__ dres,
                                                          T *dx, float *__restrict__ part, int rows, int cols,
                                                          int rpb, int rms) {
  constexpr int NV = SUMDX ? 3 : 2;
  __shared__ float red[2][2][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row0 = blockIdx.x * rpb, row_end = min(rows, row0 + rpb);
  float gm[NP][8], dg[NP][8], db[NP][8], ds[SUMDX ? NP : 1][8];
#pragma unroll
  for (int c = 0; c < NP; ++c) {
    const int col = (c * 256 + tid) * 8;
    if (FULL || col < cols) load8(gamma + col, gm[c]);
#pragma unroll
    for (int i = 0; i < 8; ++i) { dg[c][i] = 0.f; db[c][i] = 0.f; if (SUMDX) ds[c][i] = 0.f; }
  }
  const float inv_n = 1.0f / (float)cols;
  // PF rows are in flight per block (a block is one wave per SIMD and only a few blocks share a
  // CU, so the loads of several rows ahead are what keeps the memory system busy).  They wait in
  // registers as loaded (8 bf16 in 4 registers) and are widened when their row is worked on; the
  // row's two statistics travel with them, and the residual gradient of a row is asked for one
  // row ahead, so that no load is issued and awaited inside a row's own work.
  constexpr int PF = FULL ? 2 : 4;
  Raw8<T> xn[PF][NP], dn[PF][NP], rn[2][NP];
  float mean_n[PF], rstd_n[PF];
  auto fetch = [&](int row, auto buf_tag) {
    constexpr int BUF = decltype(buf_tag)::value;
    if (FULL) row = min(row, row_end - 1); else if (row >= row_end) return;
    const size_t base = (size_t)row * cols;
    mean_n[BUF] = stats[2 * (size_t)row];
    rstd_n[BUF] = stats[2 * (size_t)row + 1];
#pragma unroll
    for (int c = 0; c < NP; ++c) {
      const int col = (c * 256 + tid) * 8;
      if (FULL || col < cols) { xn[BUF][c].load(x + base + col); dn[BUF][c].load(dy + base + col); }
    }
  };
  auto fetch_res = [&](int row, auto par_tag) {
    constexpr int PAR = decltype(par_tag)::value;
    if (FULL) { if (!RES) return; row = min(row, row_end - 1); }
    else if (dres == nullptr || row >= row_end) return;
    const size_t base = (size_t)row * cols;
#pragma unroll
    for (int c = 0; c < NP; ++c) {
      const int col = (c * 256 + tid) * 8;
      if (FULL || col < cols) rn[PAR][c].load(dres + base + col);
    }
  };
  auto process = [&](int row, auto buf_tag, auto par_tag) {
    constexpr int BUF = decltype(buf_tag)::value;
    constexpr int PAR = decltype(par_tag)::value;
    const float mean = mean_n[BUF], rstd = rstd_n[BUF];
    const size_t base = (size_t)row * cols;
    fetch_res(row + 1, std::integral_constant<int, 1 - PAR>{});
    float xh[NP][8], g[NP][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NP; ++c) {
      const int col = (c * 256 + tid) * 8;
      if (FULL || col < cols) {
        float xv[8], dv[8];
        xn[BUF][c].unpack(xv);
        dn[BUF][c].unpack(dv);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          xh[c][i] = (xv[i] - mean) * rstd;
          dg[c][i] += dv[i] * xh[c][i];
          db[c][i] += dv[i];
          g[c][i] = dv[i] * gm[c][i];
          s1 += g[c][i];
          s2 += g[c][i] * xh[c][i];
        }
      }
    }
    fetch(row + PF, buf_tag);   // this buffer's next row
    s1 = wave_sum(s1); s2 = wave_sum(s2);
    const int slot = (row - row0) & 1;
    if (lane == 0) { red[slot][0][wave] = s1; red[slot][1][wave] = s2; }
    __syncthreads();
    const float m1 = rms ? 0.f : (((red[slot][0][0] + red[slot][0][1]) + red[slot][0][2]) + red[slot][0][3]) * inv_n;
    const float m2 = (((red[slot][1][0] + red[slot][1][1]) + red[slot][1][2]) + red[slot][1][3]) * inv_n;
#pragma unroll
    for (int c = 0; c < NP; ++c) {
      const int col = (c * 256 + tid) * 8;
      if (FULL || col < cols) {
        float o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = rstd * (g[c][i] - m1 - xh[c][i] * m2);
        if (FULL ? RES : dres != nullptr) {
          float r[8];
          rn[PAR][c].unpack(r);
#pragma unroll
          for (int i = 0; i < 8; ++i) o[i] += r[i];
        }
        store8(dx + base + col, o);
        if (SUMDX) {
#pragma unroll
          for (int i = 0; i < 8; ++i) ds[c][i] += (float)(T)o[i];   // the value as stored
        }
      }
    }
  };
  using I0 = std::integral_constant<int, 0>; using I1 = std::integral_constant<int, 1>;
  fetch(row0, I0{});
  fetch(row0 + 1, I1{});
  if (!FULL) {
    fetch(row0 + 2, std::integral_constant<int, FULL ? 0 : 2>{});
    fetch(row0 + 3, std::integral_constant<int, FULL ? 1 : 3>{});
  }
  fetch_res(row0, I0{});
  // (the trip count of the loop is the same for every thread of the block: the barriers inside match;
  //  rows alternate between the two residual buffers)
  if (FULL) {   // (the launcher gives every block a multiple of four rows)
    for (int row = row0; row < row_end; row += 4) {
      // (fences: the rows' instruction streams stay apart, or their temporaries add up)
      process(row, I0{}, I0{});
      __builtin_amdgcn_sched_barrier(0);
      process(row + 1, I1{}, I1{});
      __builtin_amdgcn_sched_barrier(0);
      process(row + 2, I0{}, I0{});
      __builtin_amdgcn_sched_barrier(0);
      process(row + 3, I1{}, I1{});
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
    for (int row = row0; row < row_end; row += 4) {
      process(row, I0{}, I0{});
      if (row + 1 < row_end) process(row + 1, I1{}, I1{});
      if (row + 2 < row_end) process(row + 2, std::integral_constant<int, FULL ? 0 : 2>{}, I0{});
      if (row + 3 < row_end) process(row + 3, std::integral_constant<int, FULL ? 1 : 3>{}, I1{});
    }
  }
  float *prow = part + (size_t)blockIdx.x * NV * cols;
#pragma unroll
  for (int c = 0; c < NP; ++c) {
    const int col = (c * 256 + tid) * 8;
    if (FULL || col < cols) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        prow[col + i] = dg[c][i];
        prow[(size_t)cols + col + i] = db[c][i];
        if (SUMDX) prow[2 * (size_t)cols + col + i] = ds[c][i];
      }
    }
  }
}

// Pass 2: out[j] = sum_{b<nb} part[b][j], summed in a fixed order; column j of the
// `width`-wide partial rows goes to out[j / seg][j % seg].  Block = 64 columns x 16 row groups.
template <typename T>
__global__ __launch_bounds__(1024) void reduce_partials_kernel(const float *__restrict__ part, int nb, int width,
                                                               T *__restrict__ out0, T *__restrict__ out1,
                                                               T *__restrict__ out2, int seg) {
  __shared__ float red[16][64];
  const int cx = threadIdx.x & 63, g = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + cx;
  float s = 0.f;
  if (col < width) {
    // batches of 8 independent loads: the kernel is latency-bound, not bandwidth-bound
    int b = g;
    for (; b + 7 * 16 < nb; b += 8 * 16) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = part[(size_t)(b + u * 16) * width + col];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; b < nb; b += 16) s += part[(size_t)b * width + col];
  }
  red[g][cx] = s;
  __syncthreads();
  if (g == 0 && col < width) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += red[i][cx];
    const int which = col / seg, k = col - which * seg;
    stf((which == 0 ? out0 : which == 1 ? out1 : out2) + k, t);
  }
}

// The same pass for up to kMaxReduceJobs reductions in one launch: block b belongs to the job
// whose block range contains it and does exactly what reduce_partials_kernel does for it.
struct ReduceJobTable {
  ReduceJob job[kMaxReduceJobs];
  int first_block[kMaxReduceJobs + 1];
  int n;
};
template <typename T>
__global__ __launch_bounds__(1024) void reduce_jobs_kernel(ReduceJobTable t) {
  __shared__ float red[16][64];
  int j = 0;
  while (j + 1 < t.n && (int)blockIdx.x >= t.first_block[j + 1]) ++j;
  const ReduceJob &job = t.job[j];
  const float *__restrict__ part = job.part;
  const int nb = job.nb, width = job.width;
  const int cx = threadIdx.x & 63, g = threadIdx.x >> 6;
  const int col = ((int)blockIdx.x - t.first_block[j]) * 64 + cx;
  float s = 0.f;
  if (col < width) {
    int b = g;
    for (; b + 7 * 16 < nb; b += 8 * 16) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = part[(size_t)(b + u * 16) * width + col];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; b < nb; b += 16) s += part[(size_t)b * width + col];
  }
  red[g][cx] = s;
  __syncthreads();
  if (g == 0 && col < width) {
    float tsum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) tsum += red[i][cx];
    const int which = col / job.seg, k = col - which * job.seg;
    T *dst = (T *)(which == 0 ? job.out0 : which == 1 ? job.out1 : job.out2) + k;
    stf(dst, job.accumulate ? tsum + ldf(dst) : tsum);
  }
}

// Column sums of x [rows, cols]: block (cx, rb) covers 512 columns and rows
// [rb*rpb, (rb+1)*rpb); partial row rb of part[nrb][cols].
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T *__restrict__ x, float *__restrict__ part, int rows,
                                                     int cols, int rpb) {
  __shared__ float red[4][512];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = (blockIdx.x * 64 + lane) * 8;
  const int row_end = min(rows, (int)(blockIdx.y + 1) * rpb);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (col < cols) {
    for (int row = blockIdx.y * rpb + wave; row < row_end; row += 4) {
      float v[8];
      load8(x + (size_t)row * cols + col, v);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += v[i];
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) red[wave][lane * 8 + i] = acc[i];
  __syncthreads();
  for (int k = threadIdx.x; k < 512; k += 256) {
    const int c = blockIdx.x * 512 + k;
    if (c < cols) part[(size_t)blockIdx.y * cols + c] = ((red[0][k] + red[1][k]) + red[2][k]) + red[3][k];
  }
}

// ------------------------------------------------------------------ dropout of a hidden state
// y = (res ? res : 0) + keep * scale * x over n elements (8 a thread); element i's decision is
// drop_bits(i, keys of unit 0).  Forward: x is a linear layer's output, res the residual
// branch.  Backward: x is the gradient of y, no res.
template <typename T>
__global__ __launch_bounds__(256) void dropout_kernel(const T *x /* may alias y */, const T *res /* may alias y */,
                                                      T *y, size_t n8, DropArgs a) {
  const DropKeys k = drop_keys(a.base, 0u);
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
    float v[8], r[8];
    load8(x + i * 8, v);
    if (res != nullptr) load8(res + i * 8, r);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const bool keep = drop_bits((uint32_t)(i * 8 + q), k.k0, k.k1) >= a.thr;
      const float d = keep ? v[q] * a.scale : 0.f;
      v[q] = res != nullptr ? r[q] + d : d;
    }
    store8(y + i * 8, v);
  }
}

// ------------------------------------------------------------------ GELU
template <typename T>
__global__ __launch_bounds__(256) void gelu_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, size_t n8,
                                                       int kind) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
    float v[8];
    load8(x + i * 8, v);
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = gelu_f(v[k], kind);
    store8(y + i * 8, v);
  }
}

// dx = dy * gelu'(x) over [rows, cols] plus the column sums of the stored dx (the bias
// gradient of the linear layer in front of the GELU): block (cx, rb) covers 512 columns
// and rows [rb*rpb, (rb+1)*rpb); its partial sums go to part[rb][cols].
template <typename T>
__global__ __launch_bounds__(256) void gelu_bwd_colsum_kernel(const T *dy /* may alias dx */,
                                                              const T *__restrict__ x, T *dx,
                                                              float *__restrict__ part, int rows, int cols, int rpb,
                                                              int kind) {
  __shared__ float red[4][512];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = (blockIdx.x * 64 + lane) * 8;
  const int row_end = min(rows, (int)(blockIdx.y + 1) * rpb);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (col < cols) {
    for (int row = blockIdx.y * rpb + wave; row < row_end; row += 4) {
      const size_t at = (size_t)row * cols + col;
      float v[8], d[8];
      load8(x + at, v);
      load8(dy + at, d);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        v[i] = d[i] * gelu_df(v[i], kind);
        acc[i] += (float)(T)v[i];
      }
      store8(dx + at, v);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) red[wave][lane * 8 + i] = acc[i];
  __syncthreads();
  for (int k = threadIdx.x; k < 512; k += 256) {
    const int c = blockIdx.x * 512 + k;
    if (c < cols) part[(size_t)blockIdx.y * cols + c] = ((red[0][k] + red[1][k]) + red[2][k]) + red[3][k];
  }
}

// ------------------------------------------------------------------ misc
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T *__restrict__ src, T *__restrict__ dst, int rows,
                                                        int cols) {
  __shared__ T tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  for (int i = ty; i < 32; i += 8)
    if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = src[(size_t)(r0 + i) * cols + c0 + tx];
  __syncthreads();
  for (int i = ty; i < 32; i += 8)
    if (c0 + i < cols && r0 + tx < rows) dst[(size_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t *p, size_t n, uint32_t pattern) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = pattern;
}

// ------------------------------------------------------------------ launchers
bool ln_supported(int dtype, int cols) {
  (void)dtype;
  return cols > 0 && cols % 8 == 0 && cols <= 8192;
}

static int ln_chunks(int cols) {
  const int c = (cols + 511) / 512;
  return c <= 1 ? 1 : c <= 2 ? 2 : c <= 4 ? 4 : c <= 8 ? 8 : 16;
}

template <typename T>
static hipError_t ln_fwd_t(int rows, int cols, float eps, const void *x, const void *gamma, const void *beta,
                           void *y, float *stats, hipStream_t s, int rms) {
  const dim3 grid((rows + 3) / 4), block(256);
#define DP_LN_FWD(NC)                                                                                       \
  hipLaunchKernelGGL((ln_fwd_kernel<T, NC>), grid, block, 0, s, (const T *)x, (const T *)gamma,             \
                     (const T *)beta, (T *)y, stats, rows, cols, eps, rms)
  switch (ln_chunks(cols)) {
    case 1: DP_LN_FWD(1); break;
    case 2: DP_LN_FWD(2); break;
    case 4: DP_LN_FWD(4); break;
    case 8: DP_LN_FWD(8); break;
    default: DP_LN_FWD(16); break;
  }
#undef DP_LN_FWD
  return hipGetLastError();
}

hipError_t launch_ln_fwd(int dtype, int rows, int cols, float eps, const void *x, const void *gamma,
                         const void *beta, void *y, float *stats, hipStream_t s, bool rms) {
  if (rows <= 0) return hipSuccess;
  return dtype == kBF16 ? ln_fwd_t<bf16>(rows, cols, eps, x, gamma, beta, y, stats, s, rms ? 1 : 0)
                        : ln_fwd_t<float>(rows, cols, eps, x, gamma, beta, y, stats, s, rms ? 1 : 0);
}

// second pass now, or left to the caller as a job
template <typename T>
static hipError_t reduce_or_defer(const float *part, int nb, int width, int seg, void *o0, void *o1, void *o2,
                                  hipStream_t s, ReduceJob *job) {
  if (job != nullptr) { *job = ReduceJob{part, nb, width, seg, o0, o1, o2, 0}; return hipSuccess; }
  hipLaunchKernelGGL((reduce_partials_kernel<T>), dim3((width + 63) / 64), dim3(1024), 0, s, part, nb, width, (T *)o0,
                     (T *)o1, (T *)o2, seg);
  return hipGetLastError();
}

template <typename T, bool SUMDX>
static hipError_t ln_bwd_t(int rows, int cols, const void *dy, const void *x, const float *stats,
                           const void *gamma, const void *dres, void *dx, void *dgamma, void *dbeta, void *dxsum,
                           void *ws, hipStream_t s, ReduceJob *job, int rms) {
  int rpb;
  const int nb = row_blocks(rows, 8, &rpb);
  const int nv = SUMDX ? 3 : 2;
  float *part = (float *)ws;
#define DP_LN_BWD_AS(NC, AHEAD)                                                                                    \
  hipLaunchKernelGGL((ln_bwd_kernel<T, NC, SUMDX, AHEAD>), dim3(nb), dim3(256), 0, s, (const T *)dy, (const T *)x, \
                     stats, (const T *)gamma, (const T *)dres, (T *)dx, part, rows, cols, rpb, rms)
#define DP_LN_BWD(NC)                                                               \
  do {                                                                              \
    if (NC <= 2 || rpb >= 16) DP_LN_BWD_AS(NC, true); else DP_LN_BWD_AS(NC, false);               \
  } while (0)
#define DP_LN_BWD_WIDE_AS(NP, FULL, RES)                                                                      \
  hipLaunchKernelGGL((ln_bwd_wide_kernel<T, NP, SUMDX, FULL, RES>), dim3(nb), dim3(256), 0, s, (const T *)dy, \
                     (const T *)x, stats, (const T *)gamma, (const T *)dres, (T *)dx, part, rows, cols, rpb, rms)
#define DP_LN_BWD_WIDE(NP)                                                    \
  do {                                                                        \
    if (cols != NP * 2048 || rows % 4 != 0 || rpb % 4 != 0) DP_LN_BWD_WIDE_AS(NP, false, false); \
    else if (dres != nullptr) DP_LN_BWD_WIDE_AS(NP, true, true);              \
    else DP_LN_BWD_WIDE_AS(NP, true, false);                                  \
  } while (0)
  switch (ln_chunks(cols)) {
    case 1: DP_LN_BWD(1); break;
    case 2: DP_LN_BWD(2); break;
    case 4: DP_LN_BWD(4); break;
    case 8: DP_LN_BWD_WIDE(2); break;     // 2049..4096 columns
    default: DP_LN_BWD_WIDE(4); break;    // up to 8192
  }
#undef DP_LN_BWD_WIDE
#undef DP_LN_BWD_WIDE_AS
#undef DP_LN_BWD
#undef DP_LN_BWD_AS
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return reduce_or_defer<T>(part, nb, nv * cols, cols, dgamma, dbeta, dxsum, s, job);
}

// A sum over no rows is zero: the vectors an empty input leaves behind.
static hipError_t zero_vec(int dtype, void *p, int n, hipStream_t s) {
  if (p == nullptr || n <= 0) return hipSuccess;
  return launch_fill_u32(p, (size_t)n * dtype_size(dtype) / 4, 0u, s);
}

hipError_t launch_ln_bwd(int dtype, int rows, int cols, const void *dy, const void *x, const float *stats,
                         const void *gamma, const void *dres, void *dx, void *dgamma, void *dbeta, void *dxsum,
                         void *ws, hipStream_t s, ReduceJob *job, bool rms) {
  const int r = rms ? 1 : 0;
  if (job != nullptr) job->nb = 0;
  if (rows <= 0) {
    hipError_t e = zero_vec(dtype, dgamma, cols, s);
    if (e == hipSuccess) e = zero_vec(dtype, dbeta, cols, s);
    if (e == hipSuccess) e = zero_vec(dtype, dxsum, cols, s);
    return e;
  }
  if (dxsum != nullptr)
    return dtype == kBF16
               ? ln_bwd_t<bf16, true>(rows, cols, dy, x, stats, gamma, dres, dx, dgamma, dbeta, dxsum, ws, s, job, r)
               : ln_bwd_t<float, true>(rows, cols, dy, x, stats, gamma, dres, dx, dgamma, dbeta, dxsum, ws, s, job, r);
  return dtype == kBF16
             ? ln_bwd_t<bf16, false>(rows, cols, dy, x, stats, gamma, dres, dx, dgamma, dbeta, nullptr, ws, s, job, r)
             : ln_bwd_t<float, false>(rows, cols, dy, x, stats, gamma, dres, dx, dgamma, dbeta, nullptr, ws, s, job, r);
}

template <typename T>
static hipError_t gelu_bwd_colsum_t(int kind, int rows, int cols, const void *dy, const void *x, void *dx,
                                    void *dbias, void *ws, hipStream_t s, ReduceJob *job) {
  int rpb;
  const int nb = row_blocks(rows, 16, &rpb);
  float *part = (float *)ws;
  hipLaunchKernelGGL((gelu_bwd_colsum_kernel<T>), dim3((cols + 511) / 512, nb), dim3(256), 0, s, (const T *)dy,
                     (const T *)x, (T *)dx, part, rows, cols, rpb, kind);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return reduce_or_defer<T>(part, nb, cols, cols, dbias, dbias, dbias, s, job);
}

hipError_t launch_gelu_bwd_colsum(int dtype, int kind, int rows, int cols, const void *dy, const void *x, void *dx,
                                  void *dbias, void *ws, hipStream_t s, ReduceJob *job) {
  if (job != nullptr) job->nb = 0;
  if (rows <= 0) return zero_vec(dtype, dbias, cols, s);
  return dtype == kBF16 ? gelu_bwd_colsum_t<bf16>(kind, rows, cols, dy, x, dx, dbias, ws, s, job)
                        : gelu_bwd_colsum_t<float>(kind, rows, cols, dy, x, dx, dbias, ws, s, job);
}

static int ew_grid(size_t n8) {
  size_t g = (n8 + 255) / 256;
  if (g > 256 * 16) g = 256 * 16;
  return g < 1 ? 1 : (int)g;
}

hipError_t launch_gelu_fwd(int dtype, int kind, size_t n, const void *x, void *y, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const size_t n8 = n / 8;
  if (dtype == kBF16)
    hipLaunchKernelGGL((gelu_fwd_kernel<bf16>), dim3(ew_grid(n8)), dim3(256), 0, s, (const bf16 *)x, (bf16 *)y, n8,
                       kind);
  else
    hipLaunchKernelGGL((gelu_fwd_kernel<float>), dim3(ew_grid(n8)), dim3(256), 0, s, (const float *)x, (float *)y,
                       n8, kind);
  return hipGetLastError();
}

hipError_t launch_dropout(int dtype, size_t n, const void *x, const void *res, void *y, const DropArgs &a,
                          hipStream_t s) {
  if (n == 0) return hipSuccess;
  const size_t n8 = n / 8;
  if (dtype == kBF16)
    hipLaunchKernelGGL((dropout_kernel<bf16>), dim3(ew_grid(n8)), dim3(256), 0, s, (const bf16 *)x, (const bf16 *)res,
                       (bf16 *)y, n8, a);
  else
    hipLaunchKernelGGL((dropout_kernel<float>), dim3(ew_grid(n8)), dim3(256), 0, s, (const float *)x,
                       (const float *)res, (float *)y, n8, a);
  return hipGetLastError();
}

template <typename T>
static hipError_t colsum_t(int rows, int cols, const void *x, void *out, void *ws, hipStream_t s, ReduceJob *job) {
  int rpb;
  const int nb = row_blocks(rows, 16, &rpb);
  float *part = (float *)ws;
  hipLaunchKernelGGL((colsum_kernel<T>), dim3((cols + 511) / 512, nb), dim3(256), 0, s, (const T *)x, part, rows,
                     cols, rpb);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return reduce_or_defer<T>(part, nb, cols, cols, out, out, out, s, job);
}

hipError_t launch_colsum(int dtype, int rows, int cols, const void *x, void *out, void *ws, hipStream_t s,
                         ReduceJob *job) {
  if (job != nullptr) job->nb = 0;
  if (rows <= 0) return zero_vec(dtype, out, cols, s);
  return dtype == kBF16 ? colsum_t<bf16>(rows, cols, x, out, ws, s, job) : colsum_t<float>(rows, cols, x, out, ws, s, job);
}

// ---- column sums without a workspace argument and without any allocation -----------------
// The partial sums of the two-pass reduction go to a file-scope device array instead of a
// caller's workspace.  Every GPU the library runs on holds its own copy of the array at its
// own address until the process ends; the host looks that address up once per device.  All
// calls on a GPU share the array: calls that overlap on one GPU race.
constexpr size_t kStaticScratchBytes = 8u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

size_t colsum_static_max_bytes() { return kStaticScratchBytes; }

size_t colsum_static_needed_bytes(int rows, int cols) {
  if (rows <= 0) return 0;   // (no rows: no partial sums)
  int rpb;
  return (size_t)row_blocks(rows, 16, &rpb) * (size_t)cols * sizeof(float);
}

// The array's device address on the current device (host code must never use the array's name
// where its memory is meant: the name is a host-side stand-in, not a device address).
static hipError_t scratch_address(void **out) {
  constexpr int kMaxDevices = 64;
  static void *ptr[kMaxDevices] = {};
  static std::mutex lock;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> guard(lock);
  if (ptr[dev] == nullptr) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return hipSuccess;
}

// launch_colsum with the partial sums in the library's own array.  The caller has checked that
// colsum_static_needed_bytes(rows, cols) fits.  Nothing has to start at zero: the first pass
// writes every partial the second pass reads.
hipError_t launch_colsum_static(int dtype, int rows, int cols, const void *x, void *out, hipStream_t s) {
  if (rows <= 0) return zero_vec(dtype, out, cols, s);
  void *ws = nullptr;
  const hipError_t e = scratch_address(&ws);
  if (e != hipSuccess) return e;
  return dtype == kBF16 ? colsum_t<bf16>(rows, cols, x, out, ws, s, nullptr) : colsum_t<float>(rows, cols, x, out, ws, s, nullptr);
}

hipError_t launch_reduce_jobs(int dtype, const ReduceJob *jobs, int n, hipStream_t s) {
  ReduceJobTable t;
  t.n = 0;
  int blocks = 0;
  for (int i = 0; i < n && t.n < kMaxReduceJobs; ++i) {
    if (jobs[i].nb <= 0 || jobs[i].width <= 0) continue;
    t.job[t.n] = jobs[i];
    t.first_block[t.n] = blocks;
    blocks += (jobs[i].width + 63) / 64;
    ++t.n;
  }
  t.first_block[t.n] = blocks;
  if (t.n == 0) return hipSuccess;
  if (dtype == kBF16) hipLaunchKernelGGL((reduce_jobs_kernel<bf16>), dim3(blocks), dim3(1024), 0, s, t);
  else hipLaunchKernelGGL((reduce_jobs_kernel<float>), dim3(blocks), dim3(1024), 0, s, t);
  return hipGetLastError();
}

hipError_t launch_transpose(int dtype, int rows, int cols, const void *src, void *dst, hipStream_t s) {
  const dim3 grid((cols + 31) / 32, (rows + 31) / 32), block(256);
  if (dtype == kBF16)
    hipLaunchKernelGGL((transpose_kernel<bf16>), grid, block, 0, s, (const bf16 *)src, (bf16 *)dst, rows, cols);
  else
    hipLaunchKernelGGL((transpose_kernel<float>), grid, block, 0, s, (const float *)src, (float *)dst, rows, cols);
  return hipGetLastError();
}

hipError_t launch_fill_u32(void *p, size_t n_words, uint32_t pattern, hipStream_t s) {
  if (n_words == 0) return hipSuccess;
  size_t g = (n_words + 255) / 256;
  if (g > 4096) g = 4096;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((int)g), dim3(256), 0, s, (uint32_t *)p, n_words, pattern);
  return hipGetLastError();
}

}  // namespace dp
