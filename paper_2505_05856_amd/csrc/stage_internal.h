// What the translation units of libdpstage share: error text, the parsed stage shape, the
// forward op tables, the static memory walk (validate) and its timed form (walk_cost), and the
// planner's entry points.  Internal: nothing here is part of the C ABI.
#pragma once
#include "../../include/dpstage.h"
#include "kernels.h"

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <vector>

namespace dpi {

// Sets the calling thread's error text (dp_last_error) and returns `code`.
dp_status fail(dp_status code, const char *fmt, ...);

// ------------------------------------------------------------------ shapes
struct Cfg {
  int L, H, nh, dh, F, S, B;
  long T;
  bool pre, causal;
  int gelu, dtype;
  float eps;
  size_t esz;
  float p_attn, p_hidden;          // dropout rates
  bool drop_attn, drop_hidden;     // rate > 0
  int Sm = 0;                      // length of the encoder memory; 0: no cross-attention block
  long Tm = 0;                     // micro_batch * Sm
  bool cross = false;
  int nslots = DP_SLOTS_PER_LAYER; // slots (and plan bytes) per layer
  bool rms = false;                // the normalisations are RMSNorm
};

dp_status parse_cfg(const dp_stage_config *c, Cfg *o);

// ------------------------------------------------------------------ op tables
// N_OPS: nodes of a plain layer (the cost model's node arrays have that many entries); the five
// that follow are the cross-attention block of a decoder layer.
enum Op { OP_LN1, OP_QKV, OP_ATTN, OP_PROJ, OP_LN2, OP_FC1, OP_GELU, OP_FC2, N_OPS,
          OP_LNC = N_OPS, OP_QC, OP_KVC, OP_ATTNC, OP_PROJC, N_OPS_CROSS };
constexpr int kMaxSlots = DP_SLOTS_PER_LAYER_CROSS;
// A slot reference relative to a layer: dl = 1 means "X_IN of the next layer".
struct Ref { int dl, slot; };
struct OpDef { Op op; int n_in; Ref in[2]; int n_out; Ref out[2]; };
extern const OpDef kPreOps[N_OPS], kPostOps[N_OPS], kPreCrossOps[N_OPS_CROSS];
inline const OpDef *op_table(const Cfg &c) { return c.cross ? kPreCrossOps : c.pre ? kPreOps : kPostOps; }
inline int op_count(const Cfg &c) { return c.cross ? (int)N_OPS_CROSS : (int)N_OPS; }
size_t slot_bytes(const Cfg &c, int slot);
// Saved tensors a backward node reads, in the node order of each style (FreeTime needs the first
// backward reader of every candidate; the swap-ins of a layer are issued in that order).
struct BwdReads { int n; int slot[3]; };
extern const BwdReads kPreBwd[N_OPS], kPostBwd[N_OPS], kPreCrossBwd[N_OPS_CROSS];
inline const BwdReads *bwd_table(const Cfg &c) { return c.cross ? kPreCrossBwd : c.pre ? kPreBwd : kPostBwd; }

// Forward GELU as its own kernel (false) or in the FC1 GEMM epilogue (true).  A second output
// doubles the epilogue's stores (8 bytes a lane) and adds the activation's arithmetic to the
// tail of every tile: measured, the separate kernel with its 16-byte accesses is the faster of
// the two, so it is the default.
constexpr bool kFuseGeluDefault = false;

// DPSTAGE_KERNELS=simple switches the matrix-core kernels off (debugging aid).
bool env_mfma_enabled();

// ------------------------------------------------------------------ the walk, dry
dp_status check_plan(const Cfg &c, const uint8_t *plan, size_t plan_len, dp_plan_report *rep);
// How the executor spends memory a budget leaves over on the swaps of a plan (Appendix C.2 only
// says that the copies are issued "at the appropriate points"):
//   hold_ticks  launch sites for which a swapped-out block stays out of the free list, so that the
//               forward does not wait for the link before it may reuse the block;
//   ahead       layers of backward by which the swap-ins run ahead of their first use (1: the
//               swap-ins of layer l-1 are issued when the backward of layer l starts).
//   through_backward  blocks still held when the forward ends stay held through the backward (the
//               copy-outs of the top layers are still on their way then, and the first blocks
//               the backward allocates would wait for them).
// The tightest policy {0, 1, false} gives a plan's smallest peak.
struct SwapPolicy { long hold_ticks = 0; int ahead = 1; bool through_backward = false; bool defer_top = false; };
// The static memory walk: fills `rep`, picks the first policy, from the most generous down, with
// which inflight * peak fits `budget` (0 = no budget: the tightest) and returns it in *policy_out.
dp_status validate(const Cfg &c, const uint8_t *plan, size_t plan_len, uint64_t budget, uint32_t inflight,
                   dp_plan_report *rep, bool mfma_enabled, bool fuse_gelu_enabled, SwapPolicy *policy_out = nullptr);
struct CostOut { int64_t step_ns; uint64_t slot_peak, arena_peak, d2h, h2d; int replayed; };
// Plays the step under `plan` on the three clocks of the cost model.  exact = false: the
// planner's model (saved tensors only, no waits for handed-on arena blocks); exact = true:
// the executor's own arena and swap policy.
CostOut walk_cost(const Cfg &c, const dp_cost_model &cm, const uint8_t *plan, bool exact, const SwapPolicy &policy);

// Time of node i of a layer in the cost model (decoder layers have thirteen nodes: 8..12 are
// in the arrays that follow the plain layer's eight).
inline int64_t node_fwd_ns(const dp_cost_model &cm, int i) { return i < 8 ? cm.fwd_ns[i] : cm.fwd_more_ns[i - 8]; }
inline int64_t node_bwd_ns(const dp_cost_model &cm, int i) { return i < 8 ? cm.bwd_ns[i] : cm.bwd_more_ns[i - 8]; }

// Nanoseconds a copy of `bytes` takes at `bytes_per_us`, rounded up.
inline int64_t copy_ns(uint64_t bytes, uint64_t bytes_per_us) {
  return (int64_t)(((unsigned __int128)bytes * 1000u + bytes_per_us - 1) / bytes_per_us);
}

// ------------------------------------------------------------------ planner (planner.cpp)
dp_status check_cost_model(const dp_cost_model *cm);
dp_cost_model for_inflight(const dp_cost_model &cm, uint32_t inflight);
bool memopt(const Cfg &c, const dp_cost_model &cm, uint64_t budget, uint32_t inflight, uint64_t fixed_bytes,
            std::vector<uint8_t> &plan, dp_memopt_report *rep);
dp_status memopt_validated(const Cfg &c, const dp_cost_model &cm, uint64_t budget_bytes, uint32_t inflight,
                           std::vector<uint8_t> &plan, dp_memopt_report *r);

}  // namespace dpi

#define HIP_TRY(expr, code)                                                                     \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess) return dpi::fail(code, "%s failed: %s", #expr, hipGetErrorString(e_));     \
  } while (0)
