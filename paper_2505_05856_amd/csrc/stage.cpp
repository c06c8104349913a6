// Step executor, static memory walk and the stage part of dpstage's C ABI (the planners are in
// planner.cpp, the standalone operators in ops.cpp).
//
// One routine, Walk, plays a step's schedule: forward ops, plan actions at each
// saved tensor's last forward use, swap-in prefetch, on-demand replay and the
// backward ops, allocating every buffer from one offset allocator.  Run "dry"
// it launches nothing and yields the memory report (dp_plan_validate); run
// "live" the same walk, hence the same offsets and the same peak, enqueues the
// kernels and copies (dp_stage_step).
#include "stage_internal.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <array>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <vector>

namespace dpi {

thread_local char g_err[512] = "";
dp_status fail(dp_status code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

// ------------------------------------------------------------------ shapes

dp_status parse_cfg(const dp_stage_config *c, Cfg *o) {
  if (c == nullptr) return fail(DP_E_INVAL, "config is null");
  if (c->n_layers <= 0 || c->hidden <= 0 || c->n_heads <= 0 || c->ffn <= 0 || c->seq <= 0 || c->micro_batch <= 0)
    return fail(DP_E_INVAL, "config extents must be positive");
  if (c->norm_style != DP_POST_LN && c->norm_style != DP_PRE_LN) return fail(DP_E_INVAL, "bad norm_style");
  if (c->gelu_kind != DP_GELU_ERF && c->gelu_kind != DP_GELU_TANH && c->gelu_kind != DP_ACT_RELU)
    return fail(DP_E_INVAL, "bad gelu_kind");
  if (c->dtype != DP_F32 && c->dtype != DP_BF16) return fail(DP_E_INVAL, "bad dtype");
  if (c->hidden % c->n_heads != 0) return fail(DP_E_INVAL, "hidden must be a multiple of n_heads");
  if (!(c->ln_eps > 0.f)) return fail(DP_E_INVAL, "ln_eps must be positive");
  o->L = c->n_layers; o->H = c->hidden; o->nh = c->n_heads; o->dh = c->hidden / c->n_heads;
  o->F = c->ffn; o->S = c->seq; o->B = c->micro_batch; o->T = (long)c->micro_batch * c->seq;
  o->pre = c->norm_style == DP_PRE_LN; o->causal = c->causal != 0; o->gelu = c->gelu_kind;
  o->dtype = c->dtype; o->eps = c->ln_eps; o->esz = dp::dtype_size(c->dtype);
  if (!(c->p_attn >= 0.f && c->p_attn < 1.f) || !(c->p_hidden >= 0.f && c->p_hidden < 1.f))
    return fail(DP_E_INVAL, "dropout rates must be in [0, 1)");
  o->p_attn = c->p_attn; o->p_hidden = c->p_hidden;
  o->drop_attn = c->p_attn > 0.f; o->drop_hidden = c->p_hidden > 0.f;
  // a mask position is a 32-bit index into the tensor it belongs to
  if (o->drop_attn && (long)c->seq * c->seq >= (1L << 32))
    return fail(DP_E_UNSUPPORTED, "attention dropout needs seq*seq < 2^32");
  if (o->drop_hidden && (long)c->micro_batch * c->seq * c->hidden >= (1L << 32))
    return fail(DP_E_UNSUPPORTED, "hidden dropout needs tokens*hidden < 2^32");
  if (o->H % 8 || o->F % 8 || o->dh % 8)
    return fail(DP_E_UNSUPPORTED, "hidden, ffn and head_dim must be multiples of 8");
  if (!dp::ln_supported(o->dtype, o->H)) return fail(DP_E_UNSUPPORTED, "hidden > 8192 is not supported");
  if (o->S > 4096 && !(o->dtype == DP_BF16 && dp::attn_mfma_supported(o->S, o->dh)))
    return fail(DP_E_UNSUPPORTED, "seq > 4096 is not supported for this head_dim/dtype");
  if (o->T > (1L << 24) || (long)o->T * std::max(o->F, 3 * o->H) > (1L << 40))
    return fail(DP_E_UNSUPPORTED, "micro_batch*seq too large");
  if (c->norm_kind != DP_NORM_LAYER && c->norm_kind != DP_NORM_RMS) return fail(DP_E_INVAL, "bad norm_kind");
  o->rms = c->norm_kind == DP_NORM_RMS;
  if (c->mem_seq < 0) return fail(DP_E_INVAL, "mem_seq must be >= 0");
  o->Sm = c->mem_seq; o->Tm = (long)c->micro_batch * c->mem_seq; o->cross = c->mem_seq > 0;
  o->nslots = o->cross ? DP_SLOTS_PER_LAYER_CROSS : DP_SLOTS_PER_LAYER;
  if (o->cross) {
    if (!o->pre) return fail(DP_E_UNSUPPORTED, "a stage with a cross-attention block needs norm_style DP_PRE_LN");
    if (o->drop_attn && (long)c->seq * c->mem_seq >= (1L << 32))
      return fail(DP_E_UNSUPPORTED, "attention dropout needs seq*mem_seq < 2^32");
    if (o->Sm > 4096 && !(o->dtype == DP_BF16 && dp::attn_mfma_supported(o->Sm, o->dh)))
      return fail(DP_E_UNSUPPORTED, "mem_seq > 4096 is not supported for this head_dim/dtype");
    if (o->Tm > (1L << 24)) return fail(DP_E_UNSUPPORTED, "micro_batch*mem_seq too large");
  }
  return DP_OK;
}

// ------------------------------------------------------------------ op tables

const OpDef kPreOps[N_OPS] = {
    {OP_LN1, 1, {{0, DP_SLOT_X_IN}}, 2, {{0, DP_SLOT_LN1_OUT}, {0, DP_SLOT_LN1_STATS}}},
    {OP_QKV, 1, {{0, DP_SLOT_LN1_OUT}}, 1, {{0, DP_SLOT_QKV}}},
    {OP_ATTN, 1, {{0, DP_SLOT_QKV}}, 2, {{0, DP_SLOT_ATTN_OUT}, {0, DP_SLOT_ATTN_LSE}}},
    {OP_PROJ, 2, {{0, DP_SLOT_ATTN_OUT}, {0, DP_SLOT_X_IN}}, 1, {{0, DP_SLOT_RES1}}},
    {OP_LN2, 1, {{0, DP_SLOT_RES1}}, 2, {{0, DP_SLOT_LN2_OUT}, {0, DP_SLOT_LN2_STATS}}},
    {OP_FC1, 1, {{0, DP_SLOT_LN2_OUT}}, 1, {{0, DP_SLOT_FC1_OUT}}},
    {OP_GELU, 1, {{0, DP_SLOT_FC1_OUT}}, 1, {{0, DP_SLOT_GELU_OUT}}},
    {OP_FC2, 2, {{0, DP_SLOT_GELU_OUT}, {0, DP_SLOT_RES1}}, 1, {{1, DP_SLOT_X_IN}}},
};
const OpDef kPostOps[N_OPS] = {
    {OP_QKV, 1, {{0, DP_SLOT_X_IN}}, 1, {{0, DP_SLOT_QKV}}},
    {OP_ATTN, 1, {{0, DP_SLOT_QKV}}, 2, {{0, DP_SLOT_ATTN_OUT}, {0, DP_SLOT_ATTN_LSE}}},
    {OP_PROJ, 2, {{0, DP_SLOT_ATTN_OUT}, {0, DP_SLOT_X_IN}}, 1, {{0, DP_SLOT_RES1}}},
    {OP_LN1, 1, {{0, DP_SLOT_RES1}}, 2, {{0, DP_SLOT_LN1_OUT}, {0, DP_SLOT_LN1_STATS}}},
    {OP_FC1, 1, {{0, DP_SLOT_LN1_OUT}}, 1, {{0, DP_SLOT_FC1_OUT}}},
    {OP_GELU, 1, {{0, DP_SLOT_FC1_OUT}}, 1, {{0, DP_SLOT_GELU_OUT}}},
    {OP_FC2, 2, {{0, DP_SLOT_GELU_OUT}, {0, DP_SLOT_LN1_OUT}}, 1, {{0, DP_SLOT_RES2}}},
    {OP_LN2, 1, {{0, DP_SLOT_RES2}}, 2, {{1, DP_SLOT_X_IN}, {0, DP_SLOT_LN2_STATS}}},
};

// a decoder layer: the pre-LN layer with the cross-attention block between PROJ and LN2; the
// key/value projection reads the encoder memory, which is no slot
const OpDef kPreCrossOps[N_OPS_CROSS] = {
    {OP_LN1, 1, {{0, DP_SLOT_X_IN}}, 2, {{0, DP_SLOT_LN1_OUT}, {0, DP_SLOT_LN1_STATS}}},
    {OP_QKV, 1, {{0, DP_SLOT_LN1_OUT}}, 1, {{0, DP_SLOT_QKV}}},
    {OP_ATTN, 1, {{0, DP_SLOT_QKV}}, 2, {{0, DP_SLOT_ATTN_OUT}, {0, DP_SLOT_ATTN_LSE}}},
    {OP_PROJ, 2, {{0, DP_SLOT_ATTN_OUT}, {0, DP_SLOT_X_IN}}, 1, {{0, DP_SLOT_RES1}}},
    {OP_LNC, 1, {{0, DP_SLOT_RES1}}, 2, {{0, DP_SLOT_LNC_OUT}, {0, DP_SLOT_LNC_STATS}}},
    {OP_QC, 1, {{0, DP_SLOT_LNC_OUT}}, 1, {{0, DP_SLOT_Q_C}}},
    {OP_KVC, 0, {}, 1, {{0, DP_SLOT_KV_C}}},
    {OP_ATTNC, 2, {{0, DP_SLOT_Q_C}, {0, DP_SLOT_KV_C}}, 2, {{0, DP_SLOT_ATTN_C_OUT}, {0, DP_SLOT_ATTN_C_LSE}}},
    {OP_PROJC, 2, {{0, DP_SLOT_ATTN_C_OUT}, {0, DP_SLOT_RES1}}, 1, {{0, DP_SLOT_RES_C}}},
    {OP_LN2, 1, {{0, DP_SLOT_RES_C}}, 2, {{0, DP_SLOT_LN2_OUT}, {0, DP_SLOT_LN2_STATS}}},
    {OP_FC1, 1, {{0, DP_SLOT_LN2_OUT}}, 1, {{0, DP_SLOT_FC1_OUT}}},
    {OP_GELU, 1, {{0, DP_SLOT_FC1_OUT}}, 1, {{0, DP_SLOT_GELU_OUT}}},
    {OP_FC2, 2, {{0, DP_SLOT_GELU_OUT}, {0, DP_SLOT_RES_C}}, 1, {{1, DP_SLOT_X_IN}}},
};

inline bool slot_is_alias(const Cfg &c, int slot) {
  return c.pre ? slot == DP_SLOT_RES2 : slot == DP_SLOT_LN2_OUT;
}

size_t slot_bytes(const Cfg &c, int slot) {
  switch (slot) {
    case DP_SLOT_LN1_STATS: case DP_SLOT_LN2_STATS: case DP_SLOT_LNC_STATS: return (size_t)c.T * 2 * sizeof(float);
    case DP_SLOT_ATTN_LSE: case DP_SLOT_ATTN_C_LSE: return (size_t)c.B * c.nh * c.S * sizeof(float);
    case DP_SLOT_KV_C: return (size_t)c.Tm * 2 * c.H * c.esz;
    case DP_SLOT_QKV: return (size_t)c.T * 3 * c.H * c.esz;
    case DP_SLOT_FC1_OUT: case DP_SLOT_GELU_OUT: return (size_t)c.T * c.F * c.esz;
    default: return slot_is_alias(c, slot) ? 0 : (size_t)c.T * c.H * c.esz;
  }
}

double op_flops(const Cfg &c, Op op) {
  const double T = (double)c.T, H = c.H, F = c.F;
  switch (op) {
    case OP_QKV: return 2 * T * H * 3 * H;
    case OP_PROJ: return 2 * T * H * H;
    case OP_FC1: case OP_FC2: return 2 * T * H * F;
    case OP_ATTN: return (c.causal ? 2.0 : 4.0) * T * c.S * H;
    case OP_QC: case OP_PROJC: return 2 * T * H * H;
    case OP_KVC: return 2 * (double)c.Tm * H * 2 * H;
    case OP_ATTNC: return 4.0 * T * c.Sm * H;
    default: return 0;
  }
}

// ------------------------------------------------------------------ allocator
// First-fit offset allocator over an unbounded address space; the high-water
// mark is the arena size a step needs.  Blocks released by a swap-out carry the
// copy's completion event: whoever is handed overlapping memory waits for it.
struct Arena {
  static constexpr uint64_t kAlign = 256;
  struct Free { uint64_t off, size; };
  struct Pending { uint64_t off, size; int event; };
  struct Held { uint64_t off, size; int event; long ready_at; };
  std::vector<Free> free_;   // sorted by offset, coalesced; last entry is the open tail
  std::vector<Pending> pending_;
  // Blocks released by a swap-out are held back for a while before they return to the
  // free list: handing one out at once would make its next user wait for the whole
  // device-to-host copy, which serialises forward compute behind the copy engine.
  std::vector<Held> held_;
  long now = 0;         // advanced by the walk, one tick per kernel launch site
  uint64_t high_water = 0, live = 0, live_peak = 0;

  Arena() { free_.push_back({0, UINT64_MAX}); }
  static uint64_t round(uint64_t n) { return (n + kAlign - 1) / kAlign * kAlign; }

  void tick() {
    ++now;
    for (size_t i = 0; i < held_.size();) {
      if (held_[i].ready_at <= now) {
        insert_free(held_[i].off, held_[i].size);
        pending_.push_back({held_[i].off, held_[i].size, held_[i].event});
        held_.erase(held_.begin() + (long)i);
      } else ++i;
    }
  }

  void release_all_held() {
    for (const Held &h : held_) {
      insert_free(h.off, h.size);
      pending_.push_back({h.off, h.size, h.event});
    }
    held_.clear();
  }

  uint64_t alloc(uint64_t bytes, std::vector<int> *wait_events) {
    const uint64_t n = round(std::max<uint64_t>(bytes, 1));
    for (size_t i = 0; i < free_.size(); ++i) {
      if (free_[i].size < n) continue;
      const uint64_t off = free_[i].off;
      if (free_[i].size == n) free_.erase(free_.begin() + (long)i);
      else { free_[i].off += n; if (free_[i].size != UINT64_MAX) free_[i].size -= n; }
      high_water = std::max(high_water, off + n);
      live += n;
      live_peak = std::max(live_peak, live);
      for (size_t p = 0; p < pending_.size();) {
        if (pending_[p].off < off + n && off < pending_[p].off + pending_[p].size) {
          if (wait_events) wait_events->push_back(pending_[p].event);
          pending_.erase(pending_.begin() + (long)p);
        } else ++p;
      }
      return off;
    }
    return UINT64_MAX;  // unreachable: the tail is unbounded
  }

  // hold_ticks > 0: the block (whose copy-out `pending_event` marks) rejoins the free list
  // only that many ticks from now
  void release(uint64_t off, uint64_t bytes, int pending_event = -1, long hold_ticks = 0) {
    const uint64_t n = round(std::max<uint64_t>(bytes, 1));
    live -= n;
    if (pending_event >= 0 && hold_ticks > 0) { held_.push_back({off, n, pending_event, now + hold_ticks}); return; }
    if (pending_event >= 0) pending_.push_back({off, n, pending_event});
    insert_free(off, n);
  }

  void insert_free(uint64_t off, uint64_t n) {
    size_t i = 0;
    while (i < free_.size() && free_[i].off < off) ++i;
    free_.insert(free_.begin() + (long)i, {off, n});
    // merge with next, then with previous
    if (i + 1 < free_.size() && free_[i].off + free_[i].size == free_[i + 1].off) {
      free_[i].size = free_[i + 1].size == UINT64_MAX ? UINT64_MAX : free_[i].size + free_[i + 1].size;
      free_.erase(free_.begin() + (long)i + 1);
    }
    if (i > 0 && free_[i - 1].off + free_[i - 1].size == free_[i].off) {
      free_[i - 1].size = free_[i].size == UINT64_MAX ? UINT64_MAX : free_[i - 1].size + free_[i].size;
      free_.erase(free_.begin() + (long)i);
    }
  }
};

// ------------------------------------------------------------------ stage
struct LayerW {  // library-owned device copies
  void *ln1_g, *ln1_b, *b_qkv, *b_o, *ln2_g, *ln2_b, *b_fc1, *b_fc2;
  void *w_qkv, *w_o, *w_fc1, *w_fc2;       // as given: [in, out]
  void *wt_qkv, *wt_o, *wt_fc1, *wt_fc2;   // transposed: [out, in]
};

struct CrossW {  // the cross-attention block of one layer: library-owned device copies
  void *ln_g, *ln_b, *b_q, *b_kv, *b_o;
  void *w_q, *w_kv, *w_o;       // as given: [in, out]
  void *wt_q, *wt_kv, *wt_o;    // transposed: [out, in]
};

// One version of the stage's parameters.  A micro-batch in flight keeps the version its forward
// used (Section 1: an asynchronous schedule updates the parameters between a micro-batch's
// forward and its backward, so a stage keeps one version per micro-batch in flight).
struct WeightSet {
  void *slab = nullptr;
  std::vector<LayerW> w;
  void *xslab = nullptr;         // decoder stages: the cross-attention blocks' parameters of this version
  std::vector<CrossW> xw;
  int refs = 0;                  // micro-batch slots holding this version
  hipEvent_t ready = nullptr;    // upload finished
  hipEvent_t last_use = nullptr; // end of the last pass that read it
};

}  // namespace dpi
using namespace dpi;


namespace { struct Walk; }

// One micro-batch between its forward and its backward (dp_stage_forward / dp_stage_backward):
// its own arena, pinned pool and events, and the walk that holds where every saved tensor is.
struct Flight {
  Walk *walk = nullptr;          // non-null from forward to backward
  WeightSet *weights = nullptr;  // the parameter version its forward used
  std::vector<uint8_t> plan;
  void *arena = nullptr;
  uint64_t arena_bytes = 0;
  void *host_pool = nullptr;
  uint64_t host_bytes = 0;
  std::vector<hipEvent_t> events;
  uint64_t arena_peak = 0;
  hipEvent_t done = nullptr;     // end of the slot's last backward
  // what the plan in `plan` validated to (a schedule feeds the same plan again and again)
  uint64_t v_budget = 0; uint32_t v_inflight = 0, v_switches = ~0u;
  dp_plan_report v_report{};
  SwapPolicy v_hold;
};

struct dp_stage {
  Cfg c;
  dp_stage_config pub;
  std::vector<std::unique_ptr<WeightSet>> versions;
  WeightSet *current = nullptr;     // what the next forward uses
  uint64_t weight_bytes = 0;        // of one version
  void *arena = nullptr;
  uint64_t arena_bytes = 0;
  void *host_pool = nullptr;
  uint64_t host_bytes = 0;
  hipStream_t d2h = nullptr, h2d = nullptr;
  hipStream_t d2hx = nullptr;   // second copy-out stream ("express", see Walk::swap_out)
  std::vector<hipEvent_t> events;       // sync events (no timing)
  bool profiling = false;
  std::vector<hipEvent_t> prof_events;  // timing pairs
  std::vector<int> prof_class;
  std::vector<uint32_t> prof_tag;       // node of each bracket: phase << 16 | layer << 4 | node
  size_t prof_used = 0;
  double prof_flops[DP_OPC_COUNT] = {};  // algorithmic FLOP of the bracketed GEMM launches, by class
  std::vector<hipEvent_t> span_events;  // timing events of a step that reports statistics
  uint32_t debug = 0;
  bool use_mfma = true;
  std::vector<std::unique_ptr<Flight>> flights;   // indexed by the caller's micro-batch slot
  uint64_t rng_seed = 0, rng_counter = 0;         // dropout: the seed, and the micro-batch number the next forward takes
  hipEvent_t bwd_end[2] = {nullptr, nullptr};     // ends of the last two dp_stage_backward calls
  uint64_t bwd_issued = 0;
  // decoder stages: the bound memory buffers
  const void *mem = nullptr;
  void *d_mem = nullptr;
  std::vector<dp_cross_grads> dw_cross;
  // result of the last successful plan validation (a training loop repeats one plan)
  std::vector<uint8_t> cached_plan;
  uint64_t cached_budget = 0;
  uint32_t cached_switches = 0;
  dp_plan_report cached_report;
  SwapPolicy cached_hold;
  // The host may run at most kStepsInFlight steps ahead of the device: deeper command
  // backlogs made the runtime's copy path several times slower on plans that swap.
  static constexpr int kStepsInFlight = 2;
  hipEvent_t step_end[kStepsInFlight] = {nullptr, nullptr};
  uint64_t steps_issued = 0;
};

namespace {

enum SlotWhere { ABSENT = 0, RESIDENT = 1, ON_HOST = 2 };
struct SlotState {
  int where = ABSENT;
  uint64_t off = 0;        // arena offset when RESIDENT
  uint64_t host_off = 0;   // pinned-pool offset when ON_HOST (kept after swap-in)
  int ready_event = -1;    // swap-in completion the compute stream has not waited for yet
  int out_event = -1;      // swap-out completion: the host copy is whole only after it
  bool consumed = false;   // its last backward consumer has run
  bool ever_produced = false;
};

struct Buf { uint64_t off = UINT64_MAX, bytes = 0; };


struct Walk {
  const Cfg &c;
  const uint8_t *plan;
  const bool live;
  dp_stage *st;             // live only
  char *arena_base = nullptr;   // live only: where this walk's blocks and swapped copies live
  char *host_base = nullptr;
  std::vector<hipEvent_t> *evs = nullptr;
  const WeightSet *wts = nullptr;   // live only: the parameter version this micro-batch uses
  uint64_t rng_seed = 0, rng_mb = 0; // what this micro-batch's dropout masks are a function of
  bool accumulate = false;      // weight gradients are added to what the caller's buffers hold
  hipStream_t cs = nullptr; // compute stream (caller's)
  hipStream_t d2h = nullptr, h2d = nullptr;
  // The backward needs what the top layers swapped out first, and those copy-outs are the last
  // to be queued: behind the bulk of the lower layers' copies on one first-in-first-out stream
  // they would land long after the backward has asked for them back.  The copy-outs of the top
  // layers therefore go to a stream of their own (both share the link): the layers from
  // `express_from` up, which hold at most a quarter of the bytes the plan swaps (more, and the
  // top layer's copies queue behind too much on that stream as well), but always the topmost
  // layer that swaps anything.
  hipStream_t d2hx = nullptr;
  bool use_express = false;
  int express_from = -1;   // -1: not worked out yet
  bool on_express(int l) { return use_express && d2hx != nullptr && (defer_top ? deferred_layer(l) : top_layer(l)); }
  // With room to keep their blocks until the forward is over (defer_top, the most generous
  // policy), only the bottom layers' copy-outs are queued as their tensors are produced (they keep
  // the link busy during the forward and are needed back last); those of the layers above, at
  // most three quarters of the swapped bytes, are queued when the forward has been issued, on the
  // second stream, in the order the backward will ask for them: topmost layer first, within a
  // layer as the backward nodes first read them.  No tensor the backward needs early then waits on the
  // link behind one it needs late.  (A block whose copy-out is queued late must not be handed on
  // before that: the event its next user would wait for is not recorded yet.  Hence only under
  // a policy that holds such blocks through the forward.)
  bool defer_top = false;
  struct Deferred { int l, slot, produced; };
  std::vector<Deferred> deferred;
  int defer_from = -1;
  bool deferred_layer(int l) {
    if (defer_from < 0) {
      std::vector<uint64_t> per_layer((size_t)c.L, 0);
      uint64_t total = 0;
      for (int k = 0; k < c.L; ++k)
        for (int slot = 0; slot < c.nslots; ++slot)
          if (action(k, slot) == DP_SWAP) { per_layer[(size_t)k] += slot_bytes(c, slot); total += slot_bytes(c, slot); }
      defer_from = c.L;
      uint64_t sum = 0;
      for (int k = c.L - 1; k >= 0; --k) {
        if ((sum + per_layer[(size_t)k]) * 4 > total * 3) break;
        sum += per_layer[(size_t)k];
        defer_from = k;
      }
    }
    return l >= defer_from;
  }
  bool top_layer(int l) {
    if (express_from < 0) {
      std::vector<uint64_t> per_layer((size_t)c.L, 0);
      uint64_t total = 0;
      for (int k = 0; k < c.L; ++k)
        for (int slot = 0; slot < c.nslots; ++slot)
          if (action(k, slot) == DP_SWAP) { per_layer[(size_t)k] += slot_bytes(c, slot); total += slot_bytes(c, slot); }
      express_from = c.L;
      uint64_t sum = 0;
      for (int k = c.L - 1; k >= 0; --k) {
        if (per_layer[(size_t)k] == 0) { if (sum == 0) continue; }
        if (sum > 0 && (sum + per_layer[(size_t)k]) * 4 > total) break;
        sum += per_layer[(size_t)k];
        express_from = k;
      }
    }
    return l >= express_from;
  }
  const void *x_in = nullptr, *dy = nullptr;
  void *y_out = nullptr, *dx_out = nullptr;
  const dp_layer_grads *dw = nullptr;
  const void *mem = nullptr;            // decoder stages: encoder memory, its gradient, the block's gradients
  void *d_mem = nullptr;
  const dp_cross_grads *dwx = nullptr;

  Arena arena;
  std::vector<SlotState> slots;  // (L+1) * DP_SLOTS_PER_LAYER
  uint64_t host_top = 0;
  int next_event = 0;
  hipError_t herr = hipSuccess;
  bool in_backward = false;
  // kernel-selection switches; the dry walk must be given the same values as the live one
  bool mfma_enabled = true, fuse_gelu_enabled = true;
  long swap_hold_ticks = 0;   // how long a swapped-out block stays out of the free list (launch sites)
  int prefetch_ahead = 1;     // layers of backward by which the swap-ins run ahead of their first use
  bool hold_through_backward = false;   // blocks held at the end of the forward stay held
  // report
  uint64_t d2h_bytes = 0, h2d_bytes = 0, kept_bytes = 0;
  // ---- cost simulation (dry walks only; see dp_plan_cost) -------------------------------
  // With a cost model the walk also plays the schedule on three clocks, compute, copy-out
  // and copy-in, under the event rules of the live walk: record() stamps an event with its
  // stream's clock, wait() moves a stream's clock up to an event's stamp, a node adds its
  // modelled time to the compute clock and a copy its size over the link speed to its copy
  // clock.  The dry walk then stands for the streams with the small integers 1, 2, 3.
  const dp_cost_model *cm = nullptr;
  int64_t clk[4] = {0, 0, 0, 0};   // compute, copy-out, copy-in, express copy-out
  std::vector<int64_t> ev_ns;
  bool sim_arena_waits = false;            // also wait where a block is handed on behind a copy-out
  bool no_arena = false;                   // the planner's model: saved tensors only, no offsets (the searches play thousands of plans)
  uint64_t slot_live = 0, slot_peak = 0;   // saved tensors alone: Algorithm 2's walk without transients
  std::vector<std::pair<int64_t, uint64_t>> lingering;   // (copy-out landing time, bytes) of swapped-out tensors
  // a swapped-out tensor's memory counts until its copy-out has landed, seen from the compute clock
  void settle() {
    for (size_t i = 0; i < lingering.size();)
      if (lingering[i].first <= clk[0]) { slot_live -= lingering[i].second; lingering.erase(lingering.begin() + (long)i); }
      else ++i;
  }
  // A step that reports statistics times its copies (on their streams), the waits of the compute
  // stream for a swap-in or for a block handed on behind a copy-out, and its replays.
  enum SpanKind { SPAN_D2H = 0, SPAN_H2D, SPAN_WAIT, SPAN_REPLAY };
  struct Span { int kind, l, slot; size_t ev; uint64_t bytes; };
  std::vector<Span> *spans = nullptr;
  size_t span_used = 0;
  void span_begin(int kind, int l, int slot, hipStream_t s, uint64_t bytes = 0) {
    if (!live || spans == nullptr) return;
    while (st->span_events.size() < span_used + 2) {
      hipEvent_t e;
      check(hipEventCreate(&e));
      if (herr != hipSuccess) return;
      st->span_events.push_back(e);
    }
    spans->push_back(Span{kind, l, slot, span_used, bytes});
    check(hipEventRecord(st->span_events[span_used], s));
  }
  void span_end(hipStream_t s) {
    if (!live || spans == nullptr || herr != hipSuccess) return;
    check(hipEventRecord(st->span_events[span_used + 1], s));
    span_used += 2;
  }
  int n_fallback = 0;                      // launches of a bf16 stage that took a vector-ALU kernel
  uint32_t tag = 0;                        // node the next launches belong to (timing brackets)
  double replay_flops = 0, step_flops = 0;
  int n_replayed = 0, n_swapped = 0, n_launch = 0;

  Walk(const Cfg &cfg, const uint8_t *p, bool is_live, dp_stage *s)
      : c(cfg), plan(p), live(is_live), st(s), slots((size_t)(cfg.L + 1) * (size_t)cfg.nslots) {}

  // ---- helpers ------------------------------------------------------------
  SlotState &S(int l, int slot) { return slots[(size_t)l * (size_t)c.nslots + slot]; }
  const OpDef *ops() const { return op_table(c); }
  int n_ops() const { return op_count(c); }
  bool caller_owned(int l, int slot) const { return slot == DP_SLOT_X_IN && (l == 0 || l == c.L); }
  int action(int l, int slot) const {
    if (l >= c.L || slot_is_alias(c, slot) || caller_owned(l, slot)) return DP_KEEP;
    return plan[(size_t)l * (size_t)c.nslots + slot];
  }
  char *base() const { return live ? arena_base : nullptr; }
  void *ptr(int l, int slot) {
    if (slot == DP_SLOT_X_IN && l == 0) return const_cast<void *>(x_in);
    if (slot == DP_SLOT_X_IN && l == c.L) return y_out;
    return live ? base() + S(l, slot).off : nullptr;
  }
  void *bptr(const Buf &b) const { return live ? base() + b.off : nullptr; }
  void check(hipError_t e) { if (herr == hipSuccess && e != hipSuccess) herr = e; }

  int new_event() {
    const int id = next_event++;
    if (live) {
      while ((int)evs->size() <= id) {
        hipEvent_t e;
        check(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        evs->push_back(e);
      }
    }
    return id;
  }
  static int clock_of(hipStream_t s) { return (int)(intptr_t)s - 1; }
  void record(int ev, hipStream_t s) {
    if (live) check(hipEventRecord((*evs)[(size_t)ev], s));
    else if (cm) { if ((int)ev_ns.size() <= ev) ev_ns.resize((size_t)ev + 1, 0); ev_ns[(size_t)ev] = clk[clock_of(s)]; }
  }
  void wait(hipStream_t s, int ev) {
    if (live) check(hipStreamWaitEvent(s, (*evs)[(size_t)ev], 0));
    else if (cm && ev < (int)ev_ns.size()) clk[clock_of(s)] = std::max(clk[clock_of(s)], ev_ns[(size_t)ev]);
  }
  static int64_t copy_ns(uint64_t bytes, uint64_t bytes_per_us) { return dpi::copy_ns(bytes, bytes_per_us); }
  enum { TAG_FWD = 0, TAG_BWD = 1, TAG_REPLAY = 2 };
  // the launches that follow belong to node `node` of layer l; with a cost model the node's time is charged here
  void begin_node(int phase, int l, int node) {
    tag = ((uint32_t)phase << 16) | ((uint32_t)l << 4) | (uint32_t)node;
    if (cm) clk[0] += phase == TAG_BWD ? node_bwd_ns(*cm, node) : node_fwd_ns(*cm, node);
  }

  uint64_t arena_alloc(uint64_t bytes) {
    if (no_arena) return 0;
    std::vector<int> waits;
    const uint64_t off = arena.alloc(bytes, &waits);
    if (live || sim_arena_waits) {
      if (!waits.empty()) span_begin(SPAN_WAIT, -1, -1, cs);
      for (int ev : waits) wait(cs, ev);
      if (!waits.empty()) span_end(cs);
    }
    return off;
  }
  void arena_release(uint64_t off, uint64_t bytes, int pending_event = -1) {
    if (no_arena) return;
    if (live && (st->debug & 2u)) {
      if (pending_event >= 0) wait(cs, pending_event);
      check(dp::launch_fill_u32(base() + off, Arena::round(bytes) / 4, 0xFFFFFFFFu, cs));
    }
    arena.release(off, bytes, pending_event, pending_event >= 0 ? swap_hold_ticks : 0);
  }
  Buf tmp(uint64_t bytes) { Buf b; b.bytes = bytes; b.off = arena_alloc(bytes); return b; }
  void drop(Buf &b) { if (b.off != UINT64_MAX) arena_release(b.off, b.bytes); b.off = UINT64_MAX; }

  void slot_alloc(int l, int slot) {
    SlotState &s = S(l, slot);
    if (caller_owned(l, slot)) { s.where = RESIDENT; return; }
    s.off = arena_alloc(slot_bytes(c, slot));
    s.where = RESIDENT;
    settle();
    slot_live += slot_bytes(c, slot);
    slot_peak = std::max(slot_peak, slot_live);
  }
  void slot_free(int l, int slot) {
    SlotState &s = S(l, slot);
    if (s.where != RESIDENT) return;
    // a prefetched copy may still be in flight into this block
    if (s.ready_event >= 0) { wait(cs, s.ready_event); s.ready_event = -1; }
    if (!caller_owned(l, slot)) { arena_release(s.off, slot_bytes(c, slot)); slot_live -= slot_bytes(c, slot); }
    s.where = ABSENT;
  }

  // ---- profiling brackets ---------------------------------------------------
  void prof_begin(int cls) {
    ++n_launch;
    if (!no_arena) arena.tick();
    if (!live || !st->profiling) return;
    if (st->prof_used + 2 > st->prof_events.size()) {
      for (int i = 0; i < 2; ++i) { hipEvent_t e; check(hipEventCreate(&e)); st->prof_events.push_back(e); }
    }
    st->prof_class.push_back(cls);
    st->prof_tag.push_back(tag);
    check(hipEventRecord(st->prof_events[st->prof_used], cs));
  }
  void prof_end() {
    if (!live || !st->profiling) return;
    check(hipEventRecord(st->prof_events[st->prof_used + 1], cs));
    st->prof_used += 2;
  }

  // ---- kernels ----------------------------------------------------------------
  // true if a GEMM of this shape runs on the matrix-core kernel (which can also emit GELU(C))
  bool gemm_on_mfma(int mode, long M, long N, long K) const {
    if (c.dtype != DP_BF16 || !mfma_enabled) return false;
    dp::GemmArgs a{mode, (int)M, (int)N, (int)K, (const void *)16, (const void *)16, nullptr, nullptr, nullptr};
    return dp::gemm_mfma_supported(a);
  }
  void gemm(int cls, int mode, long M, long N, long K, const void *A, const void *B, const void *bias,
            const void *res, void *C, void *gelu_out = nullptr) {
    if (c.dtype == DP_BF16 && mfma_enabled && !gemm_on_mfma(mode, M, N, K)) ++n_fallback;
    if (live && st->profiling) st->prof_flops[cls] += 2.0 * (double)M * (double)N * (double)K;
    prof_begin(cls);
    if (live) {
      dp::GemmArgs a{mode, (int)M, (int)N, (int)K, A, B, bias, res, C};
      if (cls == DP_OPC_GEMM_WGRAD && accumulate) a.res = C;   // dW += X^T dY
      a.C2 = gelu_out;
      a.gelu_kind = c.gelu;
      if (c.dtype == DP_BF16 && st->use_mfma && dp::gemm_mfma_supported(a)) check(dp::launch_gemm_mfma(a, cs));
      else check(dp::launch_gemm_simple(c.dtype, a, cs));
    }
    prof_end();
  }
  // The second passes of the backward's column reductions (bias and LayerNorm parameter
  // gradients) only feed the caller's gradient buffers, so they are collected and run as one
  // launch per layer instead of one small launch each; their partial buffers live until then.
  std::vector<dp::ReduceJob> red_jobs;
  std::vector<Buf> red_ws;
  void defer_reduce(dp::ReduceJob j, const Buf &ws) {
    j.accumulate = accumulate ? 1 : 0;
    red_jobs.push_back(j);
    red_ws.push_back(ws);
    if ((int)red_ws.size() == dp::kMaxReduceJobs) flush_reduces();
  }
  void flush_reduces() {
    if (red_ws.empty()) return;
    prof_begin(DP_OPC_REDUCE);
    if (live) check(dp::launch_reduce_jobs(c.dtype, red_jobs.data(), (int)red_jobs.size(), cs));
    prof_end();
    for (Buf &b : red_ws) drop(b);
    red_jobs.clear();
    red_ws.clear();
  }
  void colsum(long rows, long cols, const void *x, void *out) {
    Buf ws = tmp(dp::reduce_ws_bytes((int)rows, (int)cols));
    dp::ReduceJob job{};
    prof_begin(DP_OPC_REDUCE);
    if (live) check(dp::launch_colsum(c.dtype, (int)rows, (int)cols, x, out, bptr(ws), cs, &job));
    prof_end();
    defer_reduce(job, ws);
  }
  // y = (res ? res : 0) + mask * scale * x at one of a layer's two hidden-state dropout sites
  void hidden_dropout(int l, int site, const void *x, const void *res, void *y) {
    prof_begin(DP_OPC_DROPOUT);
    if (live)
      check(dp::launch_dropout(c.dtype, (size_t)c.T * c.H, x, res, y,
                               dp::make_drop_args(rng_seed, rng_mb, l, site, c.p_hidden), cs));
    prof_end();
  }
  // The gradient that enters a linear layer whose output was dropped: dy through the mask, in a
  // block of its own (dy itself goes on along the residual branch), plus its column sums, which
  // are that layer's bias gradient.
  Buf masked_grad(int l, int site, const void *dyp, void *dbias) {
    Buf m = tmp((size_t)c.T * c.H * c.esz);
    hidden_dropout(l, site, dyp, nullptr, bptr(m));
    colsum(c.T, c.H, bptr(m), dbias);
    return m;
  }
  void ln_bwd(const void *dyp, const void *x, const void *stats, const void *gamma, const void *dres, void *dx,
              void *dgamma, void *dbeta, void *dxsum) {
    Buf ws = tmp(dp::reduce_ws_bytes((int)c.T, c.H));
    dp::ReduceJob job{};
    prof_begin(DP_OPC_LN_BWD);
    if (live)
      check(dp::launch_ln_bwd(c.dtype, (int)c.T, c.H, dyp, x, (const float *)stats, gamma, dres, dx, dgamma, dbeta,
                              dxsum, bptr(ws), cs, &job, c.rms));
    prof_end();
    defer_reduce(job, ws);
  }

  // dF = dG * gelu'(FC1_OUT) in place, plus db1 = column sums of dF
  void gelu_bwd(void *dg, const void *fc1_out, void *db1) {
    Buf ws = tmp(dp::reduce_ws_bytes((int)c.T, c.F));
    dp::ReduceJob job{};
    prof_begin(DP_OPC_GELU_BWD);
    if (live)
      check(dp::launch_gelu_bwd_colsum(c.dtype, c.gelu, (int)c.T, c.F, dg, fc1_out, dg, db1, bptr(ws), cs, &job));
    prof_end();
    defer_reduce(job, ws);
  }

  // Runs forward op `d` of layer l; out_ptr[i] is where output i goes (null = not written).
  void run_op(int l, const OpDef &d, void *out0, void *out1) {
    const LayerW *w = live ? &wts->w[(size_t)l] : nullptr;
    const long T = c.T, H = c.H, F = c.F;
    auto in = [&](int i) { return ptr(l + d.in[i].dl, d.in[i].slot); };
    switch (d.op) {
      case OP_LN1: case OP_LN2: {
        prof_begin(DP_OPC_LN_FWD);
        if (live) {
          const void *g = d.op == OP_LN1 ? w->ln1_g : w->ln2_g, *b = d.op == OP_LN1 ? w->ln1_b : w->ln2_b;
          check(dp::launch_ln_fwd(c.dtype, (int)T, (int)H, c.eps, in(0), g, b, out0, (float *)out1, cs, c.rms));
        }
        prof_end();
        break;
      }
      case OP_QKV:
        gemm(DP_OPC_GEMM_FWD, dp::kGemmNT, T, 3 * H, H, in(0), live ? w->wt_qkv : nullptr,
             live ? w->b_qkv : nullptr, nullptr, out0);
        break;
      case OP_ATTN:
        if (c.dtype == DP_BF16 && mfma_enabled && !dp::attn_mfma_supported(c.S, c.dh)) ++n_fallback;
        prof_begin(DP_OPC_ATTN_FWD);
        if (live) {
          const dp::DropArgs da = dp::make_drop_args(rng_seed, rng_mb, l, dp::kSiteAttn, c.p_attn);
          if (c.dtype == DP_BF16 && st->use_mfma && dp::attn_mfma_supported(c.S, c.dh))
            check(dp::launch_attn_fwd_mfma(c.B, c.S, c.nh, c.dh, c.causal, in(0), out0, (float *)out1, cs, &da));
          else
            check(dp::launch_attn_fwd_simple(c.dtype, c.B, c.S, c.nh, c.dh, c.causal, in(0), out0, (float *)out1,
                                             cs, &da));
        }
        prof_end();
        break;
      case OP_PROJ:   // with dropout: the linear layer alone, then residual + dropped output in place
        gemm(DP_OPC_GEMM_FWD, dp::kGemmNT, T, H, H, in(0), live ? w->wt_o : nullptr, live ? w->b_o : nullptr,
             c.drop_hidden ? nullptr : in(1), out0);
        if (c.drop_hidden) hidden_dropout(l, dp::kSiteProj, out0, in(1), out0);
        break;
      case OP_FC1:   // out1: GELU_OUT when the activation rides the epilogue (forward only)
        gemm(DP_OPC_GEMM_FWD, dp::kGemmNT, T, F, H, in(0), live ? w->wt_fc1 : nullptr, live ? w->b_fc1 : nullptr,
             nullptr, out0, out1);
        break;
      case OP_GELU:
        prof_begin(DP_OPC_GELU_FWD);
        if (live) check(dp::launch_gelu_fwd(c.dtype, c.gelu, (size_t)T * F, in(0), out0, cs));
        prof_end();
        break;
      case OP_FC2:
        gemm(DP_OPC_GEMM_FWD, dp::kGemmNT, T, H, F, in(0), live ? w->wt_fc2 : nullptr, live ? w->b_fc2 : nullptr,
             c.drop_hidden ? nullptr : in(1), out0);
        if (c.drop_hidden) hidden_dropout(l, dp::kSiteFc2, out0, in(1), out0);
        break;
      case OP_LNC: {
        prof_begin(DP_OPC_LN_FWD);
        if (live) {
          const CrossW &x = wts->xw[(size_t)l];
          check(dp::launch_ln_fwd(c.dtype, (int)T, (int)H, c.eps, in(0), x.ln_g, x.ln_b, out0, (float *)out1, cs, c.rms));
        }
        prof_end();
        break;
      }
      case OP_QC:
        gemm(DP_OPC_GEMM_FWD, dp::kGemmNT, T, H, H, in(0), live ? wts->xw[(size_t)l].wt_q : nullptr,
             live ? wts->xw[(size_t)l].b_q : nullptr, nullptr, out0);
        break;
      case OP_KVC:   // reads the encoder memory, which is no slot: a replay repeats the projection
        gemm(DP_OPC_GEMM_FWD, dp::kGemmNT, c.Tm, 2 * H, H, mem, live ? wts->xw[(size_t)l].wt_kv : nullptr,
             live ? wts->xw[(size_t)l].b_kv : nullptr, nullptr, out0);
        break;
      case OP_ATTNC:
        if (c.dtype == DP_BF16 && mfma_enabled && !dp::attn_mfma_supported(c.Sm, c.dh)) ++n_fallback;
        prof_begin(DP_OPC_ATTN_FWD);
        if (live) {
          const dp::AttnView v = cross_view(in(0), in(1), nullptr, nullptr);
          const dp::DropArgs da = dp::make_drop_args(rng_seed, rng_mb, l, dp::kSiteCross, c.p_attn);
          if (c.dtype == DP_BF16 && st->use_mfma && dp::attn_mfma_supported(c.Sm, c.dh))
            check(dp::launch_attn_fwd_mfma_view(c.B, c.nh, c.dh, 0, v, out0, (float *)out1, cs, &da));
          else
            check(dp::launch_attn_fwd_simple_view(c.dtype, c.B, c.nh, c.dh, 0, v, out0, (float *)out1, cs, &da));
        }
        prof_end();
        break;
      case OP_PROJC:
        gemm(DP_OPC_GEMM_FWD, dp::kGemmNT, T, H, H, in(0), live ? wts->xw[(size_t)l].wt_o : nullptr,
             live ? wts->xw[(size_t)l].b_o : nullptr, c.drop_hidden ? nullptr : in(1), out0);
        if (c.drop_hidden) hidden_dropout(l, dp::kSiteCrossProj, out0, in(1), out0);
        break;
      default: break;
    }
  }
  // queries [T,H] over the keys and values of kv [Tm,2H] = [K | V]
  dp::AttnView cross_view(const void *q, const void *kv, void *dq, void *dkv) const {
    const size_t hb = (size_t)c.H * c.esz;
    const char *k = (const char *)kv;
    char *dk = (char *)dkv;
    return dp::AttnView{q, k, k + hb, dq, dk, dk ? dk + hb : nullptr, (long)c.H, 2L * c.H, c.S, c.Sm};
  }

  // ---- swap engine --------------------------------------------------------------
  void swap_out(int l, int slot) {
    if (defer_top && deferred_layer(l)) {
      int produced = -1;
      if (live || cm) { produced = new_event(); record(produced, cs); }
      deferred.push_back({l, slot, produced});
      S(l, slot).where = ON_HOST;   // (nothing reads it before the backward; the block stays until copy_out)
      return;
    }
    copy_out(l, slot, -1);
  }
  void flush_deferred() {   // at the end of the forward: in the order the backward first reads them
    int rank[kMaxSlots];
    for (int sl = 0; sl < kMaxSlots; ++sl) rank[sl] = kMaxSlots * 4;
    const BwdReads *bwd = bwd_table(c);
    int pos = 0;
    for (int i = 0; i < n_ops(); ++i)
      for (int k = 0; k < bwd[i].n; ++k, ++pos)
        if (rank[bwd[i].slot[k]] > pos) rank[bwd[i].slot[k]] = pos;
    std::stable_sort(deferred.begin(), deferred.end(), [&](const Deferred &a, const Deferred &b) {
      return a.l != b.l ? a.l > b.l : rank[a.slot] < rank[b.slot];
    });
    for (const Deferred &d : deferred) copy_out(d.l, d.slot, d.produced);
    deferred.clear();
  }
  void copy_out(int l, int slot, int produced) {
    SlotState &s = S(l, slot);
    const uint64_t bytes = slot_bytes(c, slot);
    s.host_off = host_top;
    host_top += Arena::round(bytes);
    const int done = new_event();
    if (live || cm) {
      if (produced < 0) { produced = new_event(); record(produced, cs); }
      hipStream_t out = on_express(l) ? d2hx : d2h;
      wait(out, produced);
      span_begin(SPAN_D2H, l, slot, out, bytes);
      if (live) check(hipMemcpyAsync(host_base + s.host_off, base() + s.off, bytes, hipMemcpyDeviceToHost, out));
      else clk[clock_of(out)] += copy_ns(bytes, cm->d2h_bytes_per_us);
      span_end(out);
      record(done, out);
    }
    d2h_bytes += bytes;
    ++n_swapped;
    if (cm) lingering.push_back({clk[clock_of(on_express(l) ? d2hx : d2h)], bytes}); else slot_live -= bytes;
    arena_release(s.off, bytes, done);
    s.out_event = done;
    s.where = ON_HOST;
  }
  void swap_in(int l, int slot) {
    SlotState &s = S(l, slot);
    if (s.where != ON_HOST) return;
    const uint64_t bytes = slot_bytes(c, slot);
    s.off = arena_alloc(bytes);
    settle();
    slot_live += bytes;
    slot_peak = std::max(slot_peak, slot_live);
    const int done = new_event();
    if (live || cm) {
      const int region_free = new_event();
      record(region_free, cs);
      wait(h2d, region_free);
      wait(h2d, s.out_event);   // the copy-out of this slot must have landed in the host pool
      span_begin(SPAN_H2D, l, slot, h2d, bytes);
      if (live) check(hipMemcpyAsync(base() + s.off, host_base + s.host_off, bytes, hipMemcpyHostToDevice, h2d));
      else clk[2] += copy_ns(bytes, cm->h2d_bytes_per_us);
      span_end(h2d);
      record(done, h2d);
    }
    h2d_bytes += bytes;
    s.ready_event = done;
    s.where = RESIDENT;
  }
  // The swap-ins of layer l, in the order its backward first reads them.
  void prefetch_layer(int l) {
    if (l < 0) return;
    const BwdReads *bwd = bwd_table(c);
    for (int i = 0; i < n_ops(); ++i)
      for (int k = 0; k < bwd[i].n; ++k) swap_in(l, bwd[i].slot[k]);   // (a second call finds the slot resident)
    for (int slot = 0; slot < c.nslots; ++slot) swap_in(l, slot);      // whatever no backward node reads
  }

  // Makes slot (l, slot) readable by the compute stream: waits for its swap-in,
  // or fetches it, or replays its producer (inputs first).
  void ensure(int l, int slot) {
    SlotState &s = S(l, slot);
    if (s.where == ON_HOST) swap_in(l, slot);
    if (s.where == RESIDENT) {
      if (s.ready_event >= 0) {
        span_begin(SPAN_WAIT, l, slot, cs);
        wait(cs, s.ready_event);
        span_end(cs);
        s.ready_event = -1;
      }
      return;
    }
    // ABSENT: replay.  X_IN of layer l is produced by the last op of layer l-1.
    const int pl = slot == DP_SLOT_X_IN ? l - 1 : l;
    const OpDef *d = nullptr;
    for (int i = 0; i < n_ops() && d == nullptr; ++i)
      for (int o = 0; o < ops()[i].n_out; ++o)
        if (pl + ops()[i].out[o].dl == l && ops()[i].out[o].slot == slot) d = &ops()[i];
    for (int i = 0; i < d->n_in; ++i) ensure(pl + d->in[i].dl, d->in[i].slot);
    void *outp[2] = {nullptr, nullptr};
    for (int o = 0; o < d->n_out; ++o) {
      const int ol = pl + d->out[o].dl, os = d->out[o].slot;
      SlotState &t = S(ol, os);
      // a sibling output is written only if it is gone and still has a backward consumer ahead
      if (t.where == ABSENT && !t.consumed) { slot_alloc(ol, os); outp[o] = ptr(ol, os); }
    }
    begin_node(TAG_REPLAY, pl, (int)(d - ops()));
    span_begin(SPAN_REPLAY, pl, (int)(d - ops()), cs);
    run_op(pl, *d, outp[0], outp[1]);
    span_end(cs);
    ++n_replayed;
    replay_flops += op_flops(c, d->op);
  }
  void need(int l, std::initializer_list<int> list) { for (int s : list) ensure(l, s); }
  void done_with(int l, std::initializer_list<int> list) {
    for (int s : list) { slot_free(l, s); S(l, s).consumed = true; }
  }

  // ---- forward -------------------------------------------------------------------
  void forward() {
    S(0, DP_SLOT_X_IN).where = RESIDENT;
    for (int l = 0; l < c.L; ++l) {
      // last forward reader of every slot of this layer (producer if nobody reads it)
      int last[kMaxSlots];
      for (int s = 0; s < kMaxSlots; ++s) last[s] = -1;
      for (int i = 0; i < n_ops(); ++i) {
        const OpDef &d = ops()[i];
        for (int k = 0; k < d.n_in; ++k) if (d.in[k].dl == 0) last[d.in[k].slot] = i;
        for (int k = 0; k < d.n_out; ++k) if (d.out[k].dl == 0) last[d.out[k].slot] = i;
      }
      // In forward the GELU rides the FC1 epilogue when FC1 runs on the matrix cores (both
      // tensors are written by one kernel; the GELU op then only does its bookkeeping).
      const bool fuse_gelu = fuse_gelu_enabled && gemm_on_mfma(dp::kGemmNT, c.T, c.F, c.H);
      for (int i = 0; i < n_ops(); ++i) {
        const OpDef &d = ops()[i];
        void *outp[2] = {nullptr, nullptr};
        const bool produced_already = fuse_gelu && d.op == OP_GELU;
        for (int o = 0; o < d.n_out && !produced_already; ++o) {
          slot_alloc(l + d.out[o].dl, d.out[o].slot);
          outp[o] = ptr(l + d.out[o].dl, d.out[o].slot);
        }
        if (fuse_gelu && d.op == OP_FC1) {
          slot_alloc(l, DP_SLOT_GELU_OUT);
          outp[1] = ptr(l, DP_SLOT_GELU_OUT);
        }
        begin_node(TAG_FWD, l, i);
        if (!produced_already) run_op(l, d, outp[0], outp[1]);
        step_flops += op_flops(c, d.op);
        for (int s = 0; s < c.nslots; ++s) {
          if (last[s] != i || S(l, s).where != RESIDENT) continue;
          const int a = action(l, s);
          if (a == DP_RECOMPUTE) slot_free(l, s);
          else if (a == DP_SWAP) swap_out(l, s);
          else if (!caller_owned(l, s)) kept_bytes += slot_bytes(c, s);
        }
      }
    }
    flush_deferred();
  }

  // ---- backward ------------------------------------------------------------------
  void backward() {
    in_backward = true;
    // forward is over; unless the policy holds them on (their copy-outs may still be on their way, and
    // the first blocks the backward allocates would wait for them), the held blocks rejoin the free list
    if (!hold_through_backward) arena.release_all_held();
    const long T = c.T, H = c.H, F = c.F;
    const size_t th = (size_t)T * H * c.esz, tf = (size_t)T * F * c.esz;
    const void *dcur = dy;   // gradient of the current layer's output
    Buf dcur_buf;            // its arena block, if the library owns it
    // swap-ins run `prefetch_ahead` layers ahead of their first use, top layer first
    int fetched_down_to = c.L;   // layers >= this one have had their swap-ins issued
    auto prefetch_down_to = [&](int lo) {
      for (int k = fetched_down_to - 1; k >= std::max(lo, 0); --k) prefetch_layer(k);
      fetched_down_to = std::min(fetched_down_to, std::max(lo, 0));
    };
    prefetch_down_to(c.L - 1);
    for (int l = c.L - 1; l >= 0; --l) {
      prefetch_down_to(l - prefetch_ahead);
      const LayerW *w = live ? &wts->w[(size_t)l] : nullptr;
      const dp_layer_grads *g = live ? &dw[l] : nullptr;
#define W_(f) (live ? w->f : nullptr)
#define G_(f) (live ? g->f : nullptr)
      const int xo = c.cross ? 5 : 0;   // a decoder layer's five cross-attention nodes run between nodes 3 and 4
      if (c.pre) {
        // FC2: dG = dY W2^T, dW2 = GELU_OUT^T dY, db2 = colsum(dY)
        need(l, {DP_SLOT_GELU_OUT});
        begin_node(TAG_BWD, l, 0);
        Buf dg = tmp(tf);
        if (c.drop_hidden) {
          Buf dym = masked_grad(l, dp::kSiteFc2, dcur, G_(b_fc2));
          gemm(DP_OPC_GEMM_DGRAD, dp::kGemmNT, T, F, H, bptr(dym), W_(w_fc2), nullptr, nullptr, bptr(dg));
          gemm(DP_OPC_GEMM_WGRAD, dp::kGemmTN, F, H, T, ptr(l, DP_SLOT_GELU_OUT), bptr(dym), nullptr, nullptr,
               G_(w_fc2));
          drop(dym);
        } else {
          gemm(DP_OPC_GEMM_DGRAD, dp::kGemmNT, T, F, H, dcur, W_(w_fc2), nullptr, nullptr, bptr(dg));
          gemm(DP_OPC_GEMM_WGRAD, dp::kGemmTN, F, H, T, ptr(l, DP_SLOT_GELU_OUT), dcur, nullptr, nullptr, G_(w_fc2));
          // db2 = column sums of dY: below the top layer they come out of the LayerNorm backward
          // that produced dY (layer l+1's LN1)
          if (l == c.L - 1) colsum(T, H, dcur, G_(b_fc2));
        }
        done_with(l, {DP_SLOT_GELU_OUT});
        // GELU: dF = dG * gelu'(FC1_OUT), in place
        need(l, {DP_SLOT_FC1_OUT});
        begin_node(TAG_BWD, l, 1);
        gelu_bwd(bptr(dg), ptr(l, DP_SLOT_FC1_OUT), G_(b_fc1));
        done_with(l, {DP_SLOT_FC1_OUT});
        // FC1: dC = dF W1^T, dW1 = LN2_OUT^T dF
        need(l, {DP_SLOT_LN2_OUT});
        begin_node(TAG_BWD, l, 2);
        Buf dc = tmp(th);
        gemm(DP_OPC_GEMM_DGRAD, dp::kGemmNT, T, H, F, bptr(dg), W_(w_fc1), nullptr, nullptr, bptr(dc));
        gemm(DP_OPC_GEMM_WGRAD, dp::kGemmTN, H, F, T, ptr(l, DP_SLOT_LN2_OUT), bptr(dg), nullptr, nullptr,
             G_(w_fc1));
        drop(dg);
        done_with(l, {DP_SLOT_LN2_OUT});
        // LN2: dM = dY + LN2'(dC), in place in dC
        const int res_mlp = c.cross ? DP_SLOT_RES_C : DP_SLOT_RES1;   // the residual stream the feed-forward block reads
        need(l, {res_mlp, DP_SLOT_LN2_STATS});
        begin_node(TAG_BWD, l, 3);
        // the column sums of dM are the bias gradient of the projection that wrote that residual stream
        ln_bwd(bptr(dc), ptr(l, res_mlp), ptr(l, DP_SLOT_LN2_STATS), W_(ln2_g), dcur, bptr(dc), G_(ln2_g),
               G_(ln2_b), c.drop_hidden ? nullptr : c.cross ? (live ? dwx[l].b_o : nullptr) : G_(b_o));
        drop(dcur_buf);
        done_with(l, {res_mlp, DP_SLOT_LN2_STATS});
        Buf dm = dc;
        if (c.cross) dm = cross_block_bwd(l, dm, c.drop_hidden ? nullptr : G_(b_o));
        // out-projection: dO = dM Wo^T, dWo = ATTN_OUT^T dM
        need(l, {DP_SLOT_ATTN_OUT});
        begin_node(TAG_BWD, l, 4 + xo);
        Buf dob = tmp(th);
        {
          Buf dmm;
          if (c.drop_hidden) dmm = masked_grad(l, dp::kSiteProj, bptr(dm), G_(b_o));
          const void *dmp = c.drop_hidden ? bptr(dmm) : bptr(dm);
          gemm(DP_OPC_GEMM_DGRAD, dp::kGemmNT, T, H, H, dmp, W_(w_o), nullptr, nullptr, bptr(dob));
          gemm(DP_OPC_GEMM_WGRAD, dp::kGemmTN, H, H, T, ptr(l, DP_SLOT_ATTN_OUT), dmp, nullptr, nullptr, G_(w_o));
          if (c.drop_hidden) drop(dmm);
        }
        Buf dqkv = attention_bwd(l, dob);
        // QKV: dA = dQKV Wqkv^T, dWqkv = LN1_OUT^T dQKV
        need(l, {DP_SLOT_LN1_OUT});
        begin_node(TAG_BWD, l, 6 + xo);
        Buf da = tmp(th);
        gemm(DP_OPC_GEMM_DGRAD, dp::kGemmNT, T, H, 3 * H, bptr(dqkv), W_(w_qkv), nullptr, nullptr, bptr(da));
        gemm(DP_OPC_GEMM_WGRAD, dp::kGemmTN, H, 3 * H, T, ptr(l, DP_SLOT_LN1_OUT), bptr(dqkv), nullptr, nullptr,
             G_(w_qkv));
        drop(dqkv);
        done_with(l, {DP_SLOT_LN1_OUT});
        // LN1: dX = dM + LN1'(dA)
        need(l, {DP_SLOT_X_IN, DP_SLOT_LN1_STATS});
        begin_node(TAG_BWD, l, 7 + xo);
        void *dxp = l == 0 ? dx_out : bptr(da);
        ln_bwd(bptr(da), ptr(l, DP_SLOT_X_IN), ptr(l, DP_SLOT_LN1_STATS), W_(ln1_g), bptr(dm), dxp, G_(ln1_g),
               G_(ln1_b), (live && l > 0 && !c.drop_hidden) ? dw[l - 1].b_fc2 : nullptr);   // = db2 of the layer below
        drop(dm);
        done_with(l, {DP_SLOT_X_IN, DP_SLOT_LN1_STATS});
        if (l == 0) drop(da); else { dcur_buf = da; dcur = bptr(da); }
      } else {
        // LN2: dR2 = LN2'(dY)
        need(l, {DP_SLOT_RES2, DP_SLOT_LN2_STATS});
        begin_node(TAG_BWD, l, 0);
        Buf dr2 = tmp(th);
        ln_bwd(dcur, ptr(l, DP_SLOT_RES2), ptr(l, DP_SLOT_LN2_STATS), W_(ln2_g), nullptr, bptr(dr2), G_(ln2_g),
               G_(ln2_b), c.drop_hidden ? nullptr : G_(b_fc2));   // db2 = column sums of dR2 (masked with dropout)
        drop(dcur_buf);
        done_with(l, {DP_SLOT_RES2, DP_SLOT_LN2_STATS});
        // FC2
        need(l, {DP_SLOT_GELU_OUT});
        begin_node(TAG_BWD, l, 1);
        Buf dg = tmp(tf);
        {
          Buf dr2m;
          if (c.drop_hidden) dr2m = masked_grad(l, dp::kSiteFc2, bptr(dr2), G_(b_fc2));
          const void *dp2 = c.drop_hidden ? bptr(dr2m) : bptr(dr2);
          gemm(DP_OPC_GEMM_DGRAD, dp::kGemmNT, T, F, H, dp2, W_(w_fc2), nullptr, nullptr, bptr(dg));
          gemm(DP_OPC_GEMM_WGRAD, dp::kGemmTN, F, H, T, ptr(l, DP_SLOT_GELU_OUT), dp2, nullptr, nullptr, G_(w_fc2));
          if (c.drop_hidden) drop(dr2m);
        }
        done_with(l, {DP_SLOT_GELU_OUT});
        // GELU
        need(l, {DP_SLOT_FC1_OUT});
        begin_node(TAG_BWD, l, 2);
        gelu_bwd(bptr(dg), ptr(l, DP_SLOT_FC1_OUT), G_(b_fc1));
        done_with(l, {DP_SLOT_FC1_OUT});
        // FC1: dM = dR2 + dF W1^T, dW1 = LN1_OUT^T dF
        need(l, {DP_SLOT_LN1_OUT});
        begin_node(TAG_BWD, l, 3);
        Buf dm = tmp(th);
        gemm(DP_OPC_GEMM_DGRAD, dp::kGemmNT, T, H, F, bptr(dg), W_(w_fc1), nullptr, bptr(dr2), bptr(dm));
        gemm(DP_OPC_GEMM_WGRAD, dp::kGemmTN, H, F, T, ptr(l, DP_SLOT_LN1_OUT), bptr(dg), nullptr, nullptr,
             G_(w_fc1));
        drop(dg);
        drop(dr2);
        done_with(l, {DP_SLOT_LN1_OUT});
        // LN1: dR1 = LN1'(dM), in place
        need(l, {DP_SLOT_RES1, DP_SLOT_LN1_STATS});
        begin_node(TAG_BWD, l, 4);
        ln_bwd(bptr(dm), ptr(l, DP_SLOT_RES1), ptr(l, DP_SLOT_LN1_STATS), W_(ln1_g), nullptr, bptr(dm), G_(ln1_g),
               G_(ln1_b), c.drop_hidden ? nullptr : G_(b_o));   // dbo = column sums of dR1 (masked with dropout)
        done_with(l, {DP_SLOT_RES1, DP_SLOT_LN1_STATS});
        Buf dr1 = dm;
        // out-projection
        need(l, {DP_SLOT_ATTN_OUT});
        begin_node(TAG_BWD, l, 5);
        Buf dob = tmp(th);
        {
          Buf dr1m;
          if (c.drop_hidden) dr1m = masked_grad(l, dp::kSiteProj, bptr(dr1), G_(b_o));
          const void *dp1 = c.drop_hidden ? bptr(dr1m) : bptr(dr1);
          gemm(DP_OPC_GEMM_DGRAD, dp::kGemmNT, T, H, H, dp1, W_(w_o), nullptr, nullptr, bptr(dob));
          gemm(DP_OPC_GEMM_WGRAD, dp::kGemmTN, H, H, T, ptr(l, DP_SLOT_ATTN_OUT), dp1, nullptr, nullptr, G_(w_o));
          if (c.drop_hidden) drop(dr1m);
        }
        Buf dqkv = attention_bwd(l, dob);
        // QKV: dX = dR1 + dQKV Wqkv^T, dWqkv = X_IN^T dQKV
        need(l, {DP_SLOT_X_IN});
        begin_node(TAG_BWD, l, 7);
        Buf dxb;
        void *dxp = dx_out;
        if (l > 0) { dxb = tmp(th); dxp = bptr(dxb); }
        gemm(DP_OPC_GEMM_DGRAD, dp::kGemmNT, T, H, 3 * H, bptr(dqkv), W_(w_qkv), nullptr, bptr(dr1), dxp);
        gemm(DP_OPC_GEMM_WGRAD, dp::kGemmTN, H, 3 * H, T, ptr(l, DP_SLOT_X_IN), bptr(dqkv), nullptr, nullptr,
             G_(w_qkv));
        drop(dqkv);
        drop(dr1);
        done_with(l, {DP_SLOT_X_IN});
        if (l > 0) { dcur_buf = dxb; dcur = dxp; }
      }
#undef W_
#undef G_
      // whatever a replay left behind in this layer goes now
      for (int s = 0; s < c.nslots; ++s) { slot_free(l, s); S(l, s).consumed = true; }
      flush_reduces();
    }
    flush_reduces();
  }

  // Backward of a decoder layer's cross-attention block: takes dRc (the gradient of RES_C), returns
  // dR1 = dRc + the block's share; adds the layer's share to dMem; dbo_self receives the column sums
  // of dR1 (the bias gradient of the self-attention projection, which wrote RES1).
  Buf cross_block_bwd(int l, Buf dm, void *dbo_self) {
    const long T = c.T, H = c.H, Tm = c.Tm;
    const size_t th = (size_t)T * H * c.esz;
    const CrossW *xw = live ? &wts->xw[(size_t)l] : nullptr;
    const dp_cross_grads *xg = live ? &dwx[l] : nullptr;
#define XW_(f) (live ? xw->f : nullptr)
#define XG_(f) (live ? xg->f : nullptr)
    // output projection: dOc = dRc Wo_c^T, dWo_c = ATTN_C_OUT^T dRc
    need(l, {DP_SLOT_ATTN_C_OUT});
    begin_node(TAG_BWD, l, 4);
    Buf doc = tmp(th);
    {
      // with dropout the projection saw its output through the mask: so does its gradient, whose
      // column sums are then the bias gradient (without dropout LN2's backward handed those on)
      Buf dmm;
      if (c.drop_hidden) dmm = masked_grad(l, dp::kSiteCrossProj, bptr(dm), XG_(b_o));
      const void *dmp = c.drop_hidden ? bptr(dmm) : bptr(dm);
      gemm(DP_OPC_GEMM_DGRAD, dp::kGemmNT, T, H, H, dmp, XW_(w_o), nullptr, nullptr, bptr(doc));
      gemm(DP_OPC_GEMM_WGRAD, dp::kGemmTN, H, H, T, ptr(l, DP_SLOT_ATTN_C_OUT), dmp, nullptr, nullptr, XG_(w_o));
      if (c.drop_hidden) drop(dmm);
    }
    // attention: dQc, dKVc
    need(l, {DP_SLOT_Q_C, DP_SLOT_KV_C, DP_SLOT_ATTN_C_LSE});
    begin_node(TAG_BWD, l, 5);
    Buf dqc = tmp(th);
    Buf dkvc = tmp((size_t)Tm * 2 * H * c.esz);
    Buf ws = tmp((size_t)c.B * c.nh * c.S * sizeof(float));
    if (c.dtype == DP_BF16 && mfma_enabled && !dp::attn_mfma_supported(c.Sm, c.dh)) ++n_fallback;
    prof_begin(DP_OPC_ATTN_BWD);
    if (live) {
      const dp::AttnView v = cross_view(ptr(l, DP_SLOT_Q_C), ptr(l, DP_SLOT_KV_C), bptr(dqc), bptr(dkvc));
      const dp::DropArgs da = dp::make_drop_args(rng_seed, rng_mb, l, dp::kSiteCross, c.p_attn);
      if (c.dtype == DP_BF16 && st->use_mfma && dp::attn_mfma_supported(c.Sm, c.dh))
        check(dp::launch_attn_bwd_mfma_view(c.B, c.nh, c.dh, 0, v, ptr(l, DP_SLOT_ATTN_C_OUT),
                                            (const float *)ptr(l, DP_SLOT_ATTN_C_LSE), bptr(doc), (float *)bptr(ws), cs,
                                            &da));
      else
        check(dp::launch_attn_bwd_simple_view(c.dtype, c.B, c.nh, c.dh, 0, v, ptr(l, DP_SLOT_ATTN_C_OUT),
                                              (const float *)ptr(l, DP_SLOT_ATTN_C_LSE), bptr(doc), (float *)bptr(ws),
                                              cs, &da));
    }
    prof_end();
    drop(ws);
    drop(doc);
    done_with(l, {DP_SLOT_Q_C, DP_SLOT_KV_C, DP_SLOT_ATTN_C_OUT, DP_SLOT_ATTN_C_LSE});
    colsum(T, H, bptr(dqc), XG_(b_q));
    colsum(Tm, 2 * H, bptr(dkvc), XG_(b_kv));
    // key/value projection: dMem (+)= dKVc Wkv^T (the top layer writes, the others add), dWkv = mem^T dKVc
    begin_node(TAG_BWD, l, 6);
    gemm(DP_OPC_GEMM_DGRAD, dp::kGemmNT, Tm, H, 2 * H, bptr(dkvc), XW_(w_kv), nullptr, l == c.L - 1 ? nullptr : d_mem,
         d_mem);
    gemm(DP_OPC_GEMM_WGRAD, dp::kGemmTN, H, 2 * H, Tm, mem, bptr(dkvc), nullptr, nullptr, XG_(w_kv));
    drop(dkvc);
    // query projection: dC = dQc Wq^T, dWq = LNC_OUT^T dQc
    need(l, {DP_SLOT_LNC_OUT});
    begin_node(TAG_BWD, l, 7);
    Buf dcx = tmp(th);
    gemm(DP_OPC_GEMM_DGRAD, dp::kGemmNT, T, H, H, bptr(dqc), XW_(w_q), nullptr, nullptr, bptr(dcx));
    gemm(DP_OPC_GEMM_WGRAD, dp::kGemmTN, H, H, T, ptr(l, DP_SLOT_LNC_OUT), bptr(dqc), nullptr, nullptr, XG_(w_q));
    drop(dqc);
    done_with(l, {DP_SLOT_LNC_OUT});
    // LayerNorm of the block: dR1 = dRc + LNc'(dC), in place in dC
    need(l, {DP_SLOT_RES1, DP_SLOT_LNC_STATS});
    begin_node(TAG_BWD, l, 8);
    ln_bwd(bptr(dcx), ptr(l, DP_SLOT_RES1), ptr(l, DP_SLOT_LNC_STATS), XW_(ln_g), bptr(dm), bptr(dcx), XG_(ln_g),
           XG_(ln_b), dbo_self);
    drop(dm);
    done_with(l, {DP_SLOT_RES1, DP_SLOT_LNC_STATS});
#undef XW_
#undef XG_
    return dcx;
  }

  // dQKV from dO; frees dO and the attention slots; also the QKV bias gradient.
  Buf attention_bwd(int l, Buf &dob) {
    const long T = c.T, H = c.H;
    need(l, {DP_SLOT_QKV, DP_SLOT_ATTN_OUT, DP_SLOT_ATTN_LSE});
    begin_node(TAG_BWD, l, c.pre ? (c.cross ? 10 : 5) : 6);
    Buf dqkv = tmp((size_t)T * 3 * H * c.esz);
    Buf ws = tmp((size_t)c.B * c.nh * c.S * sizeof(float));
    if (c.dtype == DP_BF16 && mfma_enabled && !dp::attn_mfma_supported(c.S, c.dh)) ++n_fallback;
    prof_begin(DP_OPC_ATTN_BWD);
    if (live) {
      const dp_layer_grads *g = &dw[l];
      (void)g;
      const dp::DropArgs da = dp::make_drop_args(rng_seed, rng_mb, l, dp::kSiteAttn, c.p_attn);
      if (c.dtype == DP_BF16 && st->use_mfma && dp::attn_mfma_supported(c.S, c.dh))
        check(dp::launch_attn_bwd_mfma(c.B, c.S, c.nh, c.dh, c.causal, ptr(l, DP_SLOT_QKV), ptr(l, DP_SLOT_ATTN_OUT),
                                       (const float *)ptr(l, DP_SLOT_ATTN_LSE), bptr(dob), bptr(dqkv),
                                       (float *)bptr(ws), cs, &da));
      else
        check(dp::launch_attn_bwd_simple(c.dtype, c.B, c.S, c.nh, c.dh, c.causal, ptr(l, DP_SLOT_QKV),
                                         ptr(l, DP_SLOT_ATTN_OUT), (const float *)ptr(l, DP_SLOT_ATTN_LSE),
                                         bptr(dob), bptr(dqkv), (float *)bptr(ws), cs, &da));
    }
    prof_end();
    drop(ws);
    drop(dob);
    done_with(l, {DP_SLOT_QKV, DP_SLOT_ATTN_OUT, DP_SLOT_ATTN_LSE});
    colsum(T, 3 * H, bptr(dqkv), live ? dw[l].b_qkv : nullptr);
    return dqkv;
  }
};

}  // namespace

namespace dpi {

uint64_t weight_elems_per_layer(const Cfg &c, uint64_t *matrix_elems) {
  const uint64_t H = (uint64_t)c.H, F = (uint64_t)c.F;
  const uint64_t mats = H * 3 * H + H * H + 2 * H * F;
  const uint64_t vecs = 2 * H + 3 * H + H + 2 * H + F + H;
  if (matrix_elems) *matrix_elems = mats;
  return mats + vecs;
}

dp_status check_plan(const Cfg &c, const uint8_t *plan, size_t plan_len, dp_plan_report *rep) {
  if (plan == nullptr) return fail(DP_E_INVAL, "plan is null");
  const size_t ns = (size_t)c.nslots;
  if (plan_len != (size_t)c.L * ns)
    return fail(DP_E_INVAL, "plan_len is %zu, expected %zu", plan_len, (size_t)c.L * ns);
  for (size_t i = 0; i < plan_len; ++i)
    if (plan[i] > DP_SWAP) {
      if (rep) { rep->first_bad_layer = (int)(i / ns); rep->first_bad_slot = (int)(i % ns); }
      return fail(DP_E_INVAL, "plan[%zu] = %u is not an action", i, (unsigned)plan[i]);
    }
  if (plan[DP_SLOT_X_IN] == DP_RECOMPUTE) {
    if (rep) { rep->first_bad_layer = 0; rep->first_bad_slot = DP_SLOT_X_IN; }
    return fail(DP_E_PLAN, "X_IN of layer 0 cannot be recomputed: it has no producer inside the stage");
  }
  return DP_OK;
}

static void fill_report(const Cfg &c, const Walk &w, dp_plan_report *r) {
  uint64_t mats;
  const uint64_t per_layer = weight_elems_per_layer(c, &mats);
  r->weight_bytes = (uint64_t)c.L * (per_layer + mats) * c.esz;  // given + transposed matrices
  r->grad_bytes = (uint64_t)c.L * per_layer * c.esz;
  r->fixed_bytes = r->weight_bytes + r->grad_bytes + 4 * (uint64_t)c.T * c.H * c.esz;
  if (c.cross) {   // the block's parameters, and the encoder memory with its gradient
    const uint64_t H = (uint64_t)c.H, xm = 4 * H * H, xv = 6 * H;
    r->weight_bytes += (uint64_t)c.L * (2 * xm + xv) * c.esz;
    r->grad_bytes += (uint64_t)c.L * (xm + xv) * c.esz;
    r->fixed_bytes += (uint64_t)c.L * (3 * xm + 2 * xv) * c.esz + 2 * (uint64_t)c.Tm * H * c.esz;
  }
  r->arena_peak_bytes = w.arena.high_water;
  r->peak_bytes = r->fixed_bytes + w.arena.high_water;
  r->live_peak_bytes = r->fixed_bytes + w.arena.live_peak;
  r->kept_act_bytes = w.kept_bytes;
  r->swap_out_bytes = w.d2h_bytes;
  r->swap_in_bytes = w.h2d_bytes;
  r->host_pinned_bytes = w.host_top;
  r->replay_flops = w.replay_flops;
  r->step_flops = 3.0 * w.step_flops;
  r->n_replayed_ops = w.n_replayed;
  r->n_swapped_slots = w.n_swapped;
  r->n_fallback_launches = w.n_fallback;
}

bool env_mfma_enabled() {
  const char *env = getenv("DPSTAGE_KERNELS");
  return !(env != nullptr && strcmp(env, "simple") == 0);
}

// How long (in launch sites) a swapped-out block stays out of the free list, tried in
// this order until the plan fits the budget: for the rest of forward (forward compute never
// waits for a copy-out; forward memory is not reduced, backward memory is), then ever
// shorter spans (a layer's forward is about ten launch sites), finally not at all (least
// memory; the next user of the block waits for the copy).
constexpr int kNumSwapHolds = 7;
const long kSwapHolds[kNumSwapHolds] = {1L << 40, 96, 48, 24, 12, 6, 0};

dp_status validate(const Cfg &c, const uint8_t *plan, size_t plan_len, uint64_t budget, uint32_t inflight,
                   dp_plan_report *rep, bool mfma_enabled, bool fuse_gelu_enabled, SwapPolicy *policy_out) {
  dp_plan_report local;
  dp_plan_report *r = rep ? rep : &local;
  memset(r, 0, sizeof *r);
  r->first_bad_layer = r->first_bad_slot = -1;
  dp_status s = check_plan(c, plan, plan_len, r);
  if (s != DP_OK) return s;
  if (inflight < 1) return fail(DP_E_INVAL, "inflight must be >= 1");
  // Policies from the most generous down: the swap-ins as far ahead as the stage is deep, then
  // half as far and so on to one layer, each with the hold spans from "until the forward ends"
  // down to none.  Running ahead is given up before holding back: a late swap-in stalls one
  // backward node, a block handed on behind its copy-out stalls the forward at every reuse.
  std::vector<int> aheads;
  for (int a = c.L; a > 1; a /= 2) aheads.push_back(a);
  aheads.push_back(1);
  auto run = [&](int ahead, long hold, bool through, bool defer, int *n_swapped) {
    Walk w(c, plan, false, nullptr);
    w.mfma_enabled = mfma_enabled;
    w.fuse_gelu_enabled = fuse_gelu_enabled;
    w.swap_hold_ticks = hold;
    w.prefetch_ahead = ahead;
    w.hold_through_backward = through;
    w.defer_top = defer;
    w.forward();
    w.backward();
    fill_report(c, w, r);
    if (policy_out) *policy_out = SwapPolicy{hold, ahead, through, defer};
    *n_swapped = w.n_swapped;
  };
  int n_swapped = 0;
  if (budget == 0) {   // no budget: the caller wants the plan's memory saving, i.e. the tightest policy
    run(1, 0, false, false, &n_swapped);
    return DP_OK;
  }
  for (size_t ai = 0; ai < aheads.size(); ++ai)
    for (int attempt = -2; attempt < kNumSwapHolds; ++attempt) {   // -1: held through the backward as well; -2: and the top layers' copy-outs deferred
      run(aheads[ai], kSwapHolds[attempt < 0 ? 0 : attempt], attempt < 0, attempt == -2, &n_swapped);
      if ((long double)inflight * (long double)r->peak_bytes <= (long double)budget) return DP_OK;
      if (n_swapped == 0) goto out;   // nothing is swapped: every policy gives this peak
    }
out:
  return fail(DP_E_BUDGET, "plan needs %u x %llu bytes, budget is %llu", inflight,
              (unsigned long long)r->peak_bytes, (unsigned long long)budget);
}


// Plays the step under `plan` on the three clocks of the cost model.  exact = false: the
// planner's model (saved tensors only, no waits for handed-on arena blocks); exact = true:
// the executor's own arena and hold policy for `budget`.
CostOut walk_cost(const Cfg &c, const dp_cost_model &cm, const uint8_t *plan, bool exact, const SwapPolicy &policy) {
  Walk w(c, plan, false, nullptr);
  w.mfma_enabled = env_mfma_enabled();
  w.fuse_gelu_enabled = kFuseGeluDefault;
  w.swap_hold_ticks = exact ? policy.hold_ticks : 0;
  w.prefetch_ahead = exact ? policy.ahead : 1;
  w.hold_through_backward = exact && policy.through_backward;
  w.defer_top = exact && policy.defer_top;
  w.use_express = exact;
  w.cm = &cm;
  w.sim_arena_waits = exact;
  w.no_arena = !exact;
  w.cs = (hipStream_t)(intptr_t)1; w.d2h = (hipStream_t)(intptr_t)2; w.h2d = (hipStream_t)(intptr_t)3;
  w.d2hx = (hipStream_t)(intptr_t)4;
  w.forward();
  w.backward();
  CostOut o;
  o.step_ns = std::max(std::max(w.clk[0], w.clk[3]), std::max(w.clk[1], w.clk[2]));   // the copy streams are joined at the end
  o.slot_peak = w.slot_peak; o.arena_peak = w.arena.high_water;
  o.d2h = w.d2h_bytes; o.h2d = w.h2d_bytes; o.replayed = w.n_replayed;
  return o;
}




}  // namespace dpi

// ====================================================================== C ABI
extern "C" {

const char *dp_last_error(void) { return g_err; }

size_t dp_plan_len(const dp_stage_config *cfg) {
  Cfg c;
  if (parse_cfg(cfg, &c) != DP_OK) return 0;
  return (size_t)c.L * (size_t)c.nslots;
}

dp_status dp_plan_validate(const dp_stage_config *cfg, const uint8_t *plan, size_t plan_len, uint64_t budget_bytes,
                           uint32_t inflight, dp_plan_report *report) {
  Cfg c;
  dp_status s = parse_cfg(cfg, &c);
  if (s != DP_OK) return s;
  return validate(c, plan, plan_len, budget_bytes, inflight, report, env_mfma_enabled(), kFuseGeluDefault);
}

static uint64_t cross_slab_bytes(const Cfg &c);
static void cross_layout(const Cfg &c, void *slab, std::vector<CrossW> *out);

// Copies the caller's parameters (and the transposed matrices the kernels want) into a version
// of their own, on `stream`; recycles a version nothing refers to any more, else allocates one.
static dp_status upload_weights(dp_stage *st, const dp_layer_weights *layers, hipStream_t stream, WeightSet **out) {
  const Cfg &c = st->c;
  uint64_t mats;
  const uint64_t per_layer = weight_elems_per_layer(c, &mats);
  // every tensor starts on a 256-byte boundary
  const uint64_t slab = ((per_layer + mats) * c.esz + 16 * 256) * (uint64_t)c.L;
  st->weight_bytes = slab;
  WeightSet *ws = nullptr;
  for (auto &v : st->versions)
    if (v->refs == 0) { ws = v.get(); break; }   // also the current one: no micro-batch needs it any more
  if (ws == nullptr) {
    std::unique_ptr<WeightSet> fresh(new WeightSet);
    if (hipMalloc(&fresh->slab, slab) != hipSuccess) {
      (void)hipGetLastError();
      return fail(DP_E_DEVMEM, "cannot allocate %llu bytes for the weights", (unsigned long long)slab);
    }
    st->versions.push_back(std::move(fresh));
    ws = st->versions.back().get();
    HIP_TRY(hipEventCreateWithFlags(&ws->ready, hipEventDisableTiming), DP_E_HIP);
    HIP_TRY(hipEventCreateWithFlags(&ws->last_use, hipEventDisableTiming), DP_E_HIP);
  } else {
    // its last reader may have run on another stream
    HIP_TRY(hipStreamWaitEvent(stream, ws->last_use, 0), DP_E_HIP);
  }
  char *cur = (char *)ws->slab;
  auto take = [&](uint64_t elems) { void *p = cur; cur += (elems * c.esz + 255) / 256 * 256; return p; };
  ws->w.assign((size_t)c.L, LayerW{});
  const uint64_t H = (uint64_t)c.H, F = (uint64_t)c.F;
  hipError_t e = hipSuccess;
  auto copy_vec = [&](void **dst, const void *src, uint64_t n) {
    *dst = take(n);
    if (e == hipSuccess) e = hipMemcpyAsync(*dst, src, n * c.esz, hipMemcpyDeviceToDevice, stream);
  };
  auto copy_mat = [&](void **dst, void **dst_t, const void *src, uint64_t rows, uint64_t cols) {
    copy_vec(dst, src, rows * cols);
    *dst_t = take(rows * cols);
    if (e == hipSuccess) e = dp::launch_transpose(c.dtype, (int)rows, (int)cols, src, *dst_t, stream);
  };
  for (int l = 0; l < c.L; ++l) {
    LayerW &w = ws->w[(size_t)l];
    const dp_layer_weights &s0 = layers[l];
    copy_vec(&w.ln1_g, s0.ln1_g, H); copy_vec(&w.ln1_b, s0.ln1_b, H);
    copy_vec(&w.b_qkv, s0.b_qkv, 3 * H); copy_vec(&w.b_o, s0.b_o, H);
    copy_vec(&w.ln2_g, s0.ln2_g, H); copy_vec(&w.ln2_b, s0.ln2_b, H);
    copy_vec(&w.b_fc1, s0.b_fc1, F); copy_vec(&w.b_fc2, s0.b_fc2, H);
    copy_mat(&w.w_qkv, &w.wt_qkv, s0.w_qkv, H, 3 * H);
    copy_mat(&w.w_o, &w.wt_o, s0.w_o, H, H);
    copy_mat(&w.w_fc1, &w.wt_fc1, s0.w_fc1, H, F);
    copy_mat(&w.w_fc2, &w.wt_fc2, s0.w_fc2, F, H);
  }
  // decoder stages: a new version starts with the cross-attention parameters of the current one
  // (dp_stage_set_cross then replaces them)
  if (e == hipSuccess && c.cross && st->current != nullptr && ws != st->current && !st->current->xw.empty()) {
    if (ws->xslab == nullptr && hipMalloc(&ws->xslab, cross_slab_bytes(c)) != hipSuccess) {
      (void)hipGetLastError();
      ws->xslab = nullptr;
      return fail(DP_E_DEVMEM, "cannot allocate %llu bytes for the cross-attention weights",
                  (unsigned long long)cross_slab_bytes(c));
    }
    e = hipStreamWaitEvent(stream, st->current->ready, 0);
    if (e == hipSuccess)
      e = hipMemcpyAsync(ws->xslab, st->current->xslab, cross_slab_bytes(c), hipMemcpyDeviceToDevice, stream);
    cross_layout(c, ws->xslab, &ws->xw);
  }
  if (e == hipSuccess) e = hipEventRecord(ws->ready, stream);
  if (e == hipSuccess) e = hipEventRecord(ws->last_use, stream);
  if (e != hipSuccess) return fail(DP_E_HIP, "weight upload: %s", hipGetErrorString(e));
  *out = ws;
  return DP_OK;
}

static dp_status check_layer_pointers(const Cfg &c, const dp_layer_weights *layers) {
  if (layers == nullptr) return fail(DP_E_INVAL, "layers is null");
  for (int l = 0; l < c.L; ++l) {
    const void *const *p = reinterpret_cast<const void *const *>(&layers[l]);
    for (int i = 0; i < 12; ++i)
      if (p[i] == nullptr) return fail(DP_E_INVAL, "weight pointer %d of layer %d is null", i, l);
  }
  return DP_OK;
}

dp_status dp_stage_init(const dp_stage_config *cfg, const dp_layer_weights *layers, uint64_t arena_bytes_hint,
                        dp_stage **out) {
  if (out == nullptr) return fail(DP_E_INVAL, "out is null");
  *out = nullptr;
  Cfg c;
  dp_status s = parse_cfg(cfg, &c);
  if (s != DP_OK) return s;
  s = check_layer_pointers(c, layers);
  if (s != DP_OK) return s;
  dp_stage *st = new dp_stage();
  st->c = c;
  st->pub = *cfg;
  st->use_mfma = env_mfma_enabled();
  hipError_t e = hipSuccess;
  {
    WeightSet *ws = nullptr;
    s = upload_weights(st, layers, nullptr, &ws);
    if (s != DP_OK) { dp_stage_destroy(st); return s; }
    st->current = ws;
    e = hipStreamSynchronize(nullptr);
  }
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&st->d2h, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&st->h2d, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&st->d2hx, hipStreamNonBlocking);
  if (e == hipSuccess && arena_bytes_hint > 0) {
    if (hipMalloc(&st->arena, arena_bytes_hint) == hipSuccess) st->arena_bytes = arena_bytes_hint;
    else { dp_stage_destroy(st); return fail(DP_E_DEVMEM, "cannot allocate the arena hint"); }
  }
  if (e != hipSuccess) {
    dp_stage_destroy(st);
    return fail(DP_E_HIP, "stage_init: %s", hipGetErrorString(e));
  }
  *out = st;
  return DP_OK;
}

// Memory a live walk needs; a resize waits for the device first.
static dp_status ensure_memory(void **arena, uint64_t *arena_bytes, void **host_pool, uint64_t *host_bytes,
                               const dp_plan_report &rep) {
  if (rep.arena_peak_bytes > *arena_bytes) {
    HIP_TRY(hipDeviceSynchronize(), DP_E_HIP);
    if (*arena) HIP_TRY(hipFree(*arena), DP_E_HIP);
    *arena = nullptr; *arena_bytes = 0;
    if (hipMalloc(arena, rep.arena_peak_bytes) != hipSuccess) {
      (void)hipGetLastError();
      *arena = nullptr;
      return fail(DP_E_DEVMEM, "cannot allocate a %llu-byte arena", (unsigned long long)rep.arena_peak_bytes);
    }
    *arena_bytes = rep.arena_peak_bytes;
  }
  if (rep.host_pinned_bytes > *host_bytes) {
    HIP_TRY(hipDeviceSynchronize(), DP_E_HIP);
    if (*host_pool) HIP_TRY(hipHostFree(*host_pool), DP_E_HIP);
    *host_pool = nullptr; *host_bytes = 0;
    if (hipHostMalloc(host_pool, rep.host_pinned_bytes, hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      *host_pool = nullptr;
      return fail(DP_E_HOSTMEM, "cannot pin %llu bytes of host memory", (unsigned long long)rep.host_pinned_bytes);
    }
    *host_bytes = rep.host_pinned_bytes;
  }
  return DP_OK;
}

// A decoder stage can run once its block's parameters are uploaded and its memory is bound.
static dp_status cross_ready(const dp_stage *st, bool backward_too) {
  if (st->current->xw.empty()) return fail(DP_E_INVAL, "the stage has a cross-attention block: call dp_stage_set_cross first");
  if (st->mem == nullptr) return fail(DP_E_INVAL, "the stage has a cross-attention block: bind its memory with dp_stage_bind_memory");
  if (backward_too && (st->d_mem == nullptr || st->dw_cross.empty()))
    return fail(DP_E_INVAL, "the backward pass of a decoder stage needs d_mem and dw_cross (dp_stage_bind_memory)");
  return DP_OK;
}

// Bytes of one version's cross-attention parameters (every tensor on a 256-byte boundary).
static uint64_t cross_slab_bytes(const Cfg &c) {
  const uint64_t H = (uint64_t)c.H;
  return ((2 * 4 * H * H + 6 * H) * c.esz + 16 * 256) * (uint64_t)c.L;
}
// Where the tensors of layer l's block sit in a slab (the same places in every version).
static void cross_layout(const Cfg &c, void *slab, std::vector<CrossW> *out) {
  const uint64_t H = (uint64_t)c.H;
  char *cur = (char *)slab;
  auto take = [&](uint64_t elems) { void *p = cur; cur += (elems * c.esz + 255) / 256 * 256; return p; };
  out->assign((size_t)c.L, CrossW{});
  for (CrossW &w : *out) {
    w.ln_g = take(H); w.ln_b = take(H); w.b_q = take(H); w.b_kv = take(2 * H); w.b_o = take(H);
    w.w_q = take(H * H); w.wt_q = take(H * H);
    w.w_kv = take(2 * H * H); w.wt_kv = take(2 * H * H);
    w.w_o = take(H * H); w.wt_o = take(H * H);
  }
}

dp_status dp_stage_set_cross(dp_stage *st, const dp_cross_weights *layers, void *hip_stream) {
  if (st == nullptr || layers == nullptr) return fail(DP_E_INVAL, "null argument");
  const Cfg &c = st->c;
  if (!c.cross) return fail(DP_E_INVAL, "the stage has no cross-attention block (mem_seq is 0)");
  for (int l = 0; l < c.L; ++l) {
    const void *const *p = reinterpret_cast<const void *const *>(&layers[l]);
    for (int i = 0; i < 8; ++i)
      if (p[i] == nullptr) return fail(DP_E_INVAL, "cross-attention weight pointer %d of layer %d is null", i, l);
  }
  WeightSet *ws = st->current;
  if (ws->refs > 0)
    return fail(DP_E_INVAL, "a micro-batch in flight uses the current parameter version: make a new one with "
                            "dp_stage_set_weights first");
  hipStream_t stream = (hipStream_t)hip_stream;
  if (ws->xslab == nullptr) {
    if (hipMalloc(&ws->xslab, cross_slab_bytes(c)) != hipSuccess) {
      (void)hipGetLastError();
      ws->xslab = nullptr;
      return fail(DP_E_DEVMEM, "cannot allocate %llu bytes for the cross-attention weights",
                  (unsigned long long)cross_slab_bytes(c));
    }
  }
  // after the version's own upload and after its last reader, which may have run on other streams
  HIP_TRY(hipStreamWaitEvent(stream, ws->ready, 0), DP_E_HIP);
  HIP_TRY(hipStreamWaitEvent(stream, ws->last_use, 0), DP_E_HIP);
  cross_layout(c, ws->xslab, &ws->xw);
  const uint64_t H = (uint64_t)c.H;
  hipError_t e = hipSuccess;
  auto copy_vec = [&](void *dst, const void *src, uint64_t n) {
    if (e == hipSuccess) e = hipMemcpyAsync(dst, src, n * c.esz, hipMemcpyDeviceToDevice, stream);
  };
  auto copy_mat = [&](void *dst, void *dst_t, const void *src, uint64_t rows, uint64_t cols) {
    copy_vec(dst, src, rows * cols);
    if (e == hipSuccess) e = dp::launch_transpose(c.dtype, (int)rows, (int)cols, src, dst_t, stream);
  };
  for (int l = 0; l < c.L; ++l) {
    const CrossW &w = ws->xw[(size_t)l];
    const dp_cross_weights &s0 = layers[l];
    copy_vec(w.ln_g, s0.ln_g, H); copy_vec(w.ln_b, s0.ln_b, H);
    copy_vec(w.b_q, s0.b_q, H); copy_vec(w.b_kv, s0.b_kv, 2 * H); copy_vec(w.b_o, s0.b_o, H);
    copy_mat(w.w_q, w.wt_q, s0.w_q, H, H);
    copy_mat(w.w_kv, w.wt_kv, s0.w_kv, H, 2 * H);
    copy_mat(w.w_o, w.wt_o, s0.w_o, H, H);
  }
  // the version is ready once this upload is done too (every pass waits for `ready` first)
  if (e == hipSuccess) e = hipEventRecord(ws->ready, stream);
  if (e == hipSuccess) e = hipEventRecord(ws->last_use, stream);
  if (e != hipSuccess) { ws->xw.clear(); return fail(DP_E_HIP, "cross-attention weight upload: %s", hipGetErrorString(e)); }
  return DP_OK;
}

dp_status dp_stage_bind_memory(dp_stage *st, const void *mem, void *d_mem, const dp_cross_grads *dw_cross) {
  if (st == nullptr) return fail(DP_E_INVAL, "stage handle is null");
  const Cfg &c = st->c;
  if (!c.cross) return fail(DP_E_INVAL, "the stage has no cross-attention block (mem_seq is 0)");
  if (mem == nullptr) return fail(DP_E_INVAL, "mem is null");
  if (dw_cross != nullptr)
    for (int l = 0; l < c.L; ++l) {
      void *const *p = reinterpret_cast<void *const *>(&dw_cross[l]);
      for (int i = 0; i < 8; ++i)
        if (p[i] == nullptr) return fail(DP_E_INVAL, "cross-attention gradient pointer %d of layer %d is null", i, l);
    }
  st->mem = mem;
  st->d_mem = d_mem;
  if (dw_cross != nullptr) st->dw_cross.assign(dw_cross, dw_cross + c.L); else st->dw_cross.clear();
  return DP_OK;
}

dp_status dp_stage_step(dp_stage *st, const void *x_in, const void *dy, const uint8_t *plan, size_t plan_len,
                        uint64_t budget_bytes, void *y_out, void *dx_out, const dp_layer_grads *dw, void *hip_stream,
                        dp_step_stats *stats) {
  if (st == nullptr) return fail(DP_E_INVAL, "stage handle is null");
  if (!x_in || !dy || !y_out || !dx_out || !dw) return fail(DP_E_INVAL, "null buffer argument");
  const Cfg &c = st->c;
  for (int l = 0; l < c.L; ++l) {
    void *const *p = reinterpret_cast<void *const *>(&dw[l]);
    for (int i = 0; i < 12; ++i)
      if (p[i] == nullptr) return fail(DP_E_INVAL, "gradient pointer %d of layer %d is null", i, l);
  }
  if (c.cross) {
    const dp_status xs = cross_ready(st, true);
    if (xs != DP_OK) return xs;
  }
  dp_plan_report rep;
  const bool fuse_gelu = ((st->debug & 4u) != 0) != kFuseGeluDefault;   // debug bit 2 flips the default
  SwapPolicy swap_hold;
  const uint32_t switches = (st->use_mfma ? 1u : 0u) | (fuse_gelu ? 2u : 0u);
  if (plan != nullptr && st->cached_plan.size() == plan_len && st->cached_budget == budget_bytes &&
      st->cached_switches == switches && plan_len > 0 && memcmp(st->cached_plan.data(), plan, plan_len) == 0) {
    rep = st->cached_report;
    swap_hold = st->cached_hold;
  } else {
    dp_status s = validate(c, plan, plan_len, budget_bytes, 1, &rep, st->use_mfma, fuse_gelu, &swap_hold);
    if (s != DP_OK) return s;
    st->cached_plan.assign(plan, plan + plan_len);
    st->cached_budget = budget_bytes; st->cached_switches = switches;
    st->cached_report = rep; st->cached_hold = swap_hold;
  }
  {
    const dp_status ms = ensure_memory(&st->arena, &st->arena_bytes, &st->host_pool, &st->host_bytes, rep);
    if (ms != DP_OK) return ms;
  }
  hipStream_t cs = (hipStream_t)hip_stream;
  hipEvent_t &step_end = st->step_end[st->steps_issued % dp_stage::kStepsInFlight];
  if (step_end == nullptr) HIP_TRY(hipEventCreateWithFlags(&step_end, hipEventDisableTiming), DP_E_HIP);
  else HIP_TRY(hipEventSynchronize(step_end), DP_E_HIP);   // the step issued kStepsInFlight calls ago
  // A plan that swaps starts on an idle device: with the previous step still running, the
  // copies and cross-stream waits queued behind it ran markedly slower (measured: 17 ms
  // instead of 12 ms a step for 22 small swaps); the step's own launches still run ahead.
  if (rep.n_swapped_slots > 0)
    for (hipEvent_t e : st->step_end) if (e != nullptr && e != step_end) HIP_TRY(hipEventSynchronize(e), DP_E_HIP);
  Walk w(c, plan, true, st);
  w.arena_base = (char *)st->arena; w.host_base = (char *)st->host_pool; w.evs = &st->events;
  w.wts = st->current;
  w.rng_seed = st->rng_seed; w.rng_mb = st->rng_counter++;
  HIP_TRY(hipStreamWaitEvent(cs, st->current->ready, 0), DP_E_HIP);
  w.mfma_enabled = st->use_mfma;
  w.fuse_gelu_enabled = fuse_gelu;
  w.swap_hold_ticks = swap_hold.hold_ticks;
  w.prefetch_ahead = swap_hold.ahead;
  w.hold_through_backward = swap_hold.through_backward;
  w.defer_top = swap_hold.defer_top;
  w.cs = cs;
  const bool serial = (st->debug & 1u) != 0;
  w.d2h = serial ? cs : st->d2h;
  w.h2d = serial ? cs : st->h2d;
  w.d2hx = serial ? cs : st->d2hx;
  w.use_express = true;
  w.x_in = x_in; w.dy = dy; w.y_out = y_out; w.dx_out = dx_out; w.dw = dw;
  w.mem = st->mem; w.d_mem = st->d_mem; w.dwx = st->dw_cross.data();
  hipEvent_t t0 = nullptr, t1 = nullptr, t2 = nullptr;
  std::vector<Walk::Span> spans;
  if (stats) {
    w.spans = &spans;
    HIP_TRY(hipEventCreate(&t0), DP_E_HIP); HIP_TRY(hipEventCreate(&t1), DP_E_HIP); HIP_TRY(hipEventCreate(&t2), DP_E_HIP);
    HIP_TRY(hipEventRecord(t0, cs), DP_E_HIP);
  }
  w.forward();
  if (stats) HIP_TRY(hipEventRecord(t1, cs), DP_E_HIP);
  w.backward();
  // join the copy streams: every swap-out must have landed before the step is over
  if (!serial) {
    const int j1 = w.new_event(); w.record(j1, st->d2h); w.wait(cs, j1);
    const int j2 = w.new_event(); w.record(j2, st->h2d); w.wait(cs, j2);
    const int j3 = w.new_event(); w.record(j3, st->d2hx); w.wait(cs, j3);
  }
  if (w.herr != hipSuccess) return fail(DP_E_HIP, "stage_step: %s", hipGetErrorString(w.herr));
  HIP_TRY(hipEventRecord(step_end, cs), DP_E_HIP);
  HIP_TRY(hipEventRecord(st->current->last_use, cs), DP_E_HIP);
  ++st->steps_issued;
  if (w.arena.high_water != rep.arena_peak_bytes)
    return fail(DP_E_HIP, "internal: live walk peak %llu differs from the validated %llu",
                (unsigned long long)w.arena.high_water, (unsigned long long)rep.arena_peak_bytes);
  if (stats) {
    HIP_TRY(hipEventRecord(t2, cs), DP_E_HIP);
    HIP_TRY(hipEventSynchronize(t2), DP_E_HIP);
    memset(stats, 0, sizeof *stats);
    HIP_TRY(hipEventElapsedTime(&stats->fwd_ms, t0, t1), DP_E_HIP);
    HIP_TRY(hipEventElapsedTime(&stats->bwd_ms, t1, t2), DP_E_HIP);
    stats->step_ms = stats->fwd_ms + stats->bwd_ms;
    stats->d2h_bytes = w.d2h_bytes; stats->h2d_bytes = w.h2d_bytes;
    stats->arena_high_water = w.arena.high_water; stats->peak_bytes = rep.peak_bytes;
    stats->n_kernel_launches = w.n_launch; stats->n_replayed_ops = w.n_replayed;
    stats->n_fallback_launches = w.n_fallback;
    // the timed spans: copies on their streams, waits and replays on the compute stream
    const bool dump = getenv("DPSTAGE_TIMELINE") != nullptr;
    static const char *const kSpanName[] = {"d2h", "h2d", "wait", "replay"};
    for (const Walk::Span &sp : spans) {
      float a = 0.f, b = 0.f;
      HIP_TRY(hipEventElapsedTime(&a, t0, st->span_events[sp.ev]), DP_E_HIP);
      HIP_TRY(hipEventElapsedTime(&b, t0, st->span_events[sp.ev + 1]), DP_E_HIP);
      const float d = b - a;
      if (sp.kind == Walk::SPAN_D2H) stats->d2h_busy_ms += d;
      else if (sp.kind == Walk::SPAN_H2D) stats->h2d_busy_ms += d;
      else if (sp.kind == Walk::SPAN_WAIT) stats->swap_wait_ms += d;
      else stats->replay_ms += d;
      if (dump)
        fprintf(stderr, "dpstage timeline: %-6s layer %2d slot/node %2d  %9.3f .. %9.3f ms  (%.3f ms, %llu bytes)\n",
                kSpanName[sp.kind], sp.l, sp.slot, a, b, d, (unsigned long long)sp.bytes);
    }
    (void)hipEventDestroy(t0); (void)hipEventDestroy(t1); (void)hipEventDestroy(t2);
  }
  return DP_OK;
}

// ---------------------------------------------------------------- forward and backward as separate calls
namespace { constexpr uint32_t kMaxInflight = 64; }

dp_status dp_stage_forward(dp_stage *st, uint32_t slot, uint32_t inflight, const void *x_in, const uint8_t *plan,
                           size_t plan_len, uint64_t budget_bytes, void *y_out, void *hip_stream) {
  if (st == nullptr) return fail(DP_E_INVAL, "stage handle is null");
  if (!x_in || !y_out) return fail(DP_E_INVAL, "null buffer argument");
  if (inflight < 1 || inflight > kMaxInflight) return fail(DP_E_INVAL, "inflight must be 1..%u", kMaxInflight);
  if (slot >= inflight) return fail(DP_E_INVAL, "slot %u is not below inflight %u", slot, inflight);
  const Cfg &c = st->c;
  if (c.cross) {
    const dp_status xs = cross_ready(st, false);
    if (xs != DP_OK) return xs;
  }
  if (st->flights.size() <= slot) st->flights.resize((size_t)slot + 1);
  if (!st->flights[slot]) st->flights[slot].reset(new Flight);
  Flight &f = *st->flights[slot];
  if (f.walk != nullptr) return fail(DP_E_INVAL, "slot %u still holds a micro-batch whose backward has not been called", slot);
  const bool fuse_gelu = ((st->debug & 4u) != 0) != kFuseGeluDefault;
  const uint32_t switches = (st->use_mfma ? 1u : 0u) | (fuse_gelu ? 2u : 0u);
  dp_plan_report rep;
  SwapPolicy swap_hold;
  dp_status s = DP_OK;
  if (plan != nullptr && plan_len > 0 && f.plan.size() == plan_len && f.v_budget == budget_bytes &&
      f.v_inflight == inflight && f.v_switches == switches && memcmp(f.plan.data(), plan, plan_len) == 0) {
    rep = f.v_report; swap_hold = f.v_hold;
  } else {
    s = validate(c, plan, plan_len, budget_bytes, inflight, &rep, st->use_mfma, fuse_gelu, &swap_hold);
    if (s != DP_OK) return s;
    f.v_switches = ~0u;                    // nothing cached until the plan below is stored
  }
  // The host runs at most two backward passes ahead of the device; with a plan that swaps it
  // waits for the slot's last backward, since copies and cross-stream waits queued far ahead
  // of the device ran markedly slower (measured with budget 0, i.e. the tightest arena policy:
  // 6 GPT-2 1.5B layers, four in flight, every slot swapped: 92 instead of 63 ms a micro-batch;
  // never faster).  Debug bit 3 drops this wait.
  if (hipEvent_t e = st->bwd_end[st->bwd_issued % 2]) HIP_TRY(hipEventSynchronize(e), DP_E_HIP);
  if (rep.n_swapped_slots > 0 && (st->debug & 8u) == 0 && f.done != nullptr)
    HIP_TRY(hipEventSynchronize(f.done), DP_E_HIP);
  s = ensure_memory(&f.arena, &f.arena_bytes, &f.host_pool, &f.host_bytes, rep);
  if (s != DP_OK) return s;
  // the slot's last micro-batch leaves its arena before this one's kernels touch it
  if (f.done != nullptr) HIP_TRY(hipStreamWaitEvent((hipStream_t)hip_stream, f.done, 0), DP_E_HIP);
  if (f.v_switches == ~0u) {
    f.plan.assign(plan, plan + plan_len);
    f.v_budget = budget_bytes; f.v_inflight = inflight; f.v_switches = switches; f.v_report = rep; f.v_hold = swap_hold;
  }
  f.arena_peak = rep.arena_peak_bytes;
  Walk *w = new Walk(c, f.plan.data(), true, st);
  w->arena_base = (char *)f.arena; w->host_base = (char *)f.host_pool; w->evs = &f.events;
  w->wts = st->current;
  w->rng_seed = st->rng_seed; w->rng_mb = st->rng_counter++;
  HIP_TRY(hipStreamWaitEvent((hipStream_t)hip_stream, st->current->ready, 0), DP_E_HIP);
  w->mfma_enabled = st->use_mfma;
  w->fuse_gelu_enabled = fuse_gelu;
  w->swap_hold_ticks = swap_hold.hold_ticks;
  w->prefetch_ahead = swap_hold.ahead;
  w->hold_through_backward = swap_hold.through_backward;
  w->defer_top = swap_hold.defer_top;
  w->cs = (hipStream_t)hip_stream;
  const bool serial = (st->debug & 1u) != 0;
  w->d2h = serial ? w->cs : st->d2h;
  w->h2d = serial ? w->cs : st->h2d;
  w->d2hx = serial ? w->cs : st->d2hx;
  w->use_express = true;
  w->x_in = x_in; w->y_out = y_out;
  w->mem = st->mem;
  w->forward();
  if (w->herr != hipSuccess) {
    const hipError_t e = w->herr;
    delete w;
    return fail(DP_E_HIP, "stage_forward: %s", hipGetErrorString(e));
  }
  f.walk = w;
  f.weights = st->current;       // held until the backward has been issued
  ++f.weights->refs;
  return DP_OK;
}

dp_status dp_stage_backward(dp_stage *st, uint32_t slot, const void *dy, void *dx_out, const dp_layer_grads *dw,
                            uint32_t flags, void *hip_stream) {
  if (st == nullptr) return fail(DP_E_INVAL, "stage handle is null");
  if (!dy || !dx_out || !dw) return fail(DP_E_INVAL, "null buffer argument");
  if ((flags & ~(uint32_t)DP_GRAD_ACCUMULATE) != 0) return fail(DP_E_INVAL, "unknown flag bits 0x%x", flags);
  if (slot >= st->flights.size() || !st->flights[slot] || st->flights[slot]->walk == nullptr)
    return fail(DP_E_INVAL, "slot %u holds no micro-batch (call dp_stage_forward first)", slot);
  const Cfg &c = st->c;
  for (int l = 0; l < c.L; ++l) {
    void *const *p = reinterpret_cast<void *const *>(&dw[l]);
    for (int i = 0; i < 12; ++i)
      if (p[i] == nullptr) return fail(DP_E_INVAL, "gradient pointer %d of layer %d is null", i, l);
  }
  if (c.cross) {
    const dp_status xs = cross_ready(st, true);
    if (xs != DP_OK) return xs;
  }
  Flight &f = *st->flights[slot];
  std::unique_ptr<Walk> w(f.walk);
  f.walk = nullptr;                       // the slot is free again whatever happens below
  WeightSet *wset = f.weights;
  f.weights = nullptr;
  --wset->refs;
  hipStream_t cs = (hipStream_t)hip_stream;
  const bool serial = (st->debug & 1u) != 0;
  if (serial) { w->d2h = cs; w->h2d = cs; w->d2hx = cs; }
  else if (cs != w->cs) {
    // swap-outs and kernels of the forward were ordered on its stream; this one must follow them
    const int j = w->new_event(); w->record(j, w->cs); w->wait(cs, j);
  }
  w->cs = cs;
  w->dy = dy; w->dx_out = dx_out; w->dw = dw;
  w->d_mem = st->d_mem; w->dwx = st->dw_cross.data();   // (the memory itself is the one its forward saw)
  w->accumulate = (flags & DP_GRAD_ACCUMULATE) != 0;
  w->backward();
  if (!serial) {
    const int j1 = w->new_event(); w->record(j1, st->d2h); w->wait(cs, j1);
    const int j2 = w->new_event(); w->record(j2, st->h2d); w->wait(cs, j2);
    const int j3 = w->new_event(); w->record(j3, st->d2hx); w->wait(cs, j3);
  }
  if (w->herr != hipSuccess) return fail(DP_E_HIP, "stage_backward: %s", hipGetErrorString(w->herr));
  if (f.done == nullptr) HIP_TRY(hipEventCreateWithFlags(&f.done, hipEventDisableTiming), DP_E_HIP);
  HIP_TRY(hipEventRecord(f.done, cs), DP_E_HIP);
  HIP_TRY(hipEventRecord(wset->last_use, cs), DP_E_HIP);
  hipEvent_t &ring = st->bwd_end[st->bwd_issued % 2];
  if (ring == nullptr) HIP_TRY(hipEventCreateWithFlags(&ring, hipEventDisableTiming), DP_E_HIP);
  HIP_TRY(hipEventRecord(ring, cs), DP_E_HIP);
  ++st->bwd_issued;
  if (w->arena.high_water != f.arena_peak)
    return fail(DP_E_HIP, "internal: live walk peak %llu differs from the validated %llu",
                (unsigned long long)w->arena.high_water, (unsigned long long)f.arena_peak);
  return DP_OK;
}

dp_status dp_stage_read_saved(dp_stage *st, uint32_t slot, uint32_t layer, uint32_t tensor, void *dst,
                              size_t dst_bytes, void *hip_stream) {
  if (st == nullptr || dst == nullptr) return fail(DP_E_INVAL, "null argument");
  if (slot >= st->flights.size() || !st->flights[slot] || st->flights[slot]->walk == nullptr)
    return fail(DP_E_INVAL, "slot %u holds no micro-batch (call dp_stage_forward first)", slot);
  const Cfg &c = st->c;
  if ((int)layer >= c.L || (int)tensor >= c.nslots) return fail(DP_E_INVAL, "layer %u / tensor %u out of range", layer, tensor);
  Walk *w = st->flights[slot]->walk;
  if (slot_is_alias(c, (int)tensor) || slot_bytes(c, (int)tensor) == 0 || w->caller_owned((int)layer, (int)tensor))
    return fail(DP_E_INVAL, "tensor %u of layer %u has no storage of its own in the stage", tensor, layer);
  if (dst_bytes != slot_bytes(c, (int)tensor))
    return fail(DP_E_INVAL, "tensor %u is %zu bytes, dst_bytes is %zu", tensor, slot_bytes(c, (int)tensor), dst_bytes);
  if (w->S((int)layer, (int)tensor).where != RESIDENT)
    return fail(DP_E_PLAN, "tensor %u of layer %u is not on the device under this plan", tensor, layer);
  hipStream_t cs = (hipStream_t)hip_stream;
  if (cs != w->cs) { const int j = w->new_event(); w->record(j, w->cs); w->wait(cs, j); }
  HIP_TRY(hipMemcpyAsync(dst, w->ptr((int)layer, (int)tensor), dst_bytes, hipMemcpyDeviceToDevice, cs), DP_E_HIP);
  return DP_OK;
}

dp_status dp_stage_set_weights(dp_stage *st, const dp_layer_weights *layers, void *hip_stream) {
  if (st == nullptr) return fail(DP_E_INVAL, "stage handle is null");
  dp_status s = check_layer_pointers(st->c, layers);
  if (s != DP_OK) return s;
  WeightSet *ws = nullptr;
  s = upload_weights(st, layers, (hipStream_t)hip_stream, &ws);
  if (s != DP_OK) return s;
  st->current = ws;
  return DP_OK;
}

dp_status dp_stage_set_rng(dp_stage *st, uint64_t seed, uint64_t counter) {
  if (st == nullptr) return fail(DP_E_INVAL, "stage handle is null");
  st->rng_seed = seed;
  st->rng_counter = counter;
  return DP_OK;
}

int32_t dp_stage_weight_versions(const dp_stage *st) {
  if (st == nullptr) return 0;
  int32_t n = 0;
  for (const auto &v : st->versions) n += (v->refs > 0 || v.get() == st->current) ? 1 : 0;
  return n;
}

dp_status dp_stage_set_profiling(dp_stage *st, int32_t enabled) {
  if (st == nullptr) return fail(DP_E_INVAL, "stage handle is null");
  st->profiling = enabled != 0;
  return DP_OK;
}

dp_status dp_stage_op_flops(dp_stage *st, double *flops_by_class) {
  if (st == nullptr || flops_by_class == nullptr) return fail(DP_E_INVAL, "null argument");
  for (int i = 0; i < DP_OPC_COUNT; ++i) { flops_by_class[i] = st->prof_flops[i]; st->prof_flops[i] = 0.0; }
  return DP_OK;
}

dp_status dp_stage_op_times(dp_stage *st, float *ms_by_class, uint64_t *launches_by_class) {
  if (st == nullptr || ms_by_class == nullptr || launches_by_class == nullptr)
    return fail(DP_E_INVAL, "null argument");
  HIP_TRY(hipDeviceSynchronize(), DP_E_HIP);
  for (int i = 0; i < DP_OPC_COUNT; ++i) { ms_by_class[i] = 0.f; launches_by_class[i] = 0; }
  for (size_t i = 0; i + 1 < st->prof_used; i += 2) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, st->prof_events[i], st->prof_events[i + 1]), DP_E_HIP);
    const int cls = st->prof_class[i / 2];
    ms_by_class[cls] += ms;
    launches_by_class[cls] += 1;
  }
  st->prof_used = 0;
  st->prof_class.clear();
  st->prof_tag.clear();
  return DP_OK;
}

dp_status dp_stage_measure_cost_model(dp_stage *st, const void *x_in, const void *dy, void *y_out, void *dx_out,
                                      const dp_layer_grads *dw, void *hip_stream, int32_t steps, dp_cost_model *out) {
  if (st == nullptr || out == nullptr) return fail(DP_E_INVAL, "null argument");
  if (steps < 1) return fail(DP_E_INVAL, "steps must be >= 1");
  const Cfg &c = st->c;
  memset(out, 0, sizeof *out);
  // node times: keep-all steps with every launch bracketed, averaged over layers and steps
  std::vector<uint8_t> plan((size_t)c.L * (size_t)c.nslots, DP_KEEP);
  dp_status s = dp_stage_step(st, x_in, dy, plan.data(), plan.size(), 0, y_out, dx_out, dw, hip_stream, nullptr);   // warm-up
  if (s != DP_OK) return s;
  HIP_TRY(hipDeviceSynchronize(), DP_E_HIP);
  const bool was_profiling = st->profiling;
  st->profiling = true;
  st->prof_used = 0; st->prof_class.clear(); st->prof_tag.clear();
  for (int i = 0; i < steps && s == DP_OK; ++i)
    s = dp_stage_step(st, x_in, dy, plan.data(), plan.size(), 0, y_out, dx_out, dw, hip_stream, nullptr);
  st->profiling = was_profiling;
  if (s != DP_OK) return s;
  HIP_TRY(hipDeviceSynchronize(), DP_E_HIP);
  double fwd_ms[N_OPS_CROSS] = {0}, bwd_ms[N_OPS_CROSS] = {0};
  for (size_t i = 0; i + 1 < st->prof_used; i += 2) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, st->prof_events[i], st->prof_events[i + 1]), DP_E_HIP);
    const uint32_t tag = st->prof_tag[i / 2];
    const int phase = (int)(tag >> 16), node = (int)(tag & 15u);
    if (phase == Walk::TAG_BWD) bwd_ms[node] += ms; else fwd_ms[node] += ms;
  }
  st->prof_used = 0; st->prof_class.clear(); st->prof_tag.clear();
  const double per = 1e6 / ((double)steps * c.L);
  for (int i = 0; i < op_count(c); ++i) {
    const int64_t f = (int64_t)(fwd_ms[i] * per + 0.5), b = (int64_t)(bwd_ms[i] * per + 0.5);
    if (i < N_OPS) { out->fwd_ns[i] = f; out->bwd_ns[i] = b; } else { out->fwd_more_ns[i - N_OPS] = f; out->bwd_more_ns[i - N_OPS] = b; }
  }
  // link speed: a saved-tensor-sized block each way through pinned memory on the copy streams
  const size_t bytes = std::max<size_t>(slot_bytes(c, DP_SLOT_FC1_OUT), (size_t)16 << 20);
  void *dev = nullptr, *host = nullptr;
  if (hipMalloc(&dev, bytes) != hipSuccess) { (void)hipGetLastError(); return fail(DP_E_DEVMEM, "cannot allocate the %zu-byte probe block", bytes); }
  if (hipHostMalloc(&host, bytes, hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError(); (void)hipFree(dev);
    return fail(DP_E_HOSTMEM, "cannot pin the %zu-byte probe block", bytes);
  }
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  float ms_out = 0.f, ms_in = 0.f;
  constexpr int kReps = 4;
  if (e == hipSuccess) e = hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, st->d2h);   // warm-up
  if (e == hipSuccess) e = hipEventRecord(e0, st->d2h);
  for (int i = 0; i < kReps && e == hipSuccess; ++i) e = hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, st->d2h);
  if (e == hipSuccess) e = hipEventRecord(e1, st->d2h);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  if (e == hipSuccess) e = hipEventElapsedTime(&ms_out, e0, e1);
  if (e == hipSuccess) e = hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, st->h2d);
  if (e == hipSuccess) e = hipEventRecord(e0, st->h2d);
  for (int i = 0; i < kReps && e == hipSuccess; ++i) e = hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, st->h2d);
  if (e == hipSuccess) e = hipEventRecord(e1, st->h2d);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  if (e == hipSuccess) e = hipEventElapsedTime(&ms_in, e0, e1);
  // both directions at once: a second pair of blocks goes in while the first goes out
  float ms_out2 = 0.f, ms_in2 = 0.f;
  void *dev2 = nullptr, *host2 = nullptr;
  hipEvent_t f0 = nullptr, f1 = nullptr;
  if (e == hipSuccess && hipMalloc(&dev2, bytes) == hipSuccess && hipHostMalloc(&host2, bytes, hipHostMallocDefault) == hipSuccess) {
    e = hipEventCreate(&f0);
    if (e == hipSuccess) e = hipEventCreate(&f1);
    if (e == hipSuccess) e = hipEventRecord(e0, st->d2h);
    if (e == hipSuccess) e = hipEventRecord(f0, st->h2d);
    for (int i = 0; i < kReps && e == hipSuccess; ++i) {
      e = hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, st->d2h);
      if (e == hipSuccess) e = hipMemcpyAsync(dev2, host2, bytes, hipMemcpyHostToDevice, st->h2d);
    }
    if (e == hipSuccess) e = hipEventRecord(e1, st->d2h);
    if (e == hipSuccess) e = hipEventRecord(f1, st->h2d);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventSynchronize(f1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms_out2, e0, e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms_in2, f0, f1);
  } else if (e == hipSuccess) {
    (void)hipGetLastError();   // no room for the second pair: the two-way figures stay unknown
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (f0) (void)hipEventDestroy(f0);
  if (f1) (void)hipEventDestroy(f1);
  (void)hipHostFree(host);
  (void)hipFree(dev);
  if (host2) (void)hipHostFree(host2);
  if (dev2) (void)hipFree(dev2);
  if (e != hipSuccess) return fail(DP_E_HIP, "link probe failed: %s", hipGetErrorString(e));
  if (ms_out <= 0.f || ms_in <= 0.f) return fail(DP_E_HIP, "link probe measured no time");
  out->d2h_bytes_per_us = (uint64_t)((double)bytes * kReps / ((double)ms_out * 1e3));
  out->h2d_bytes_per_us = (uint64_t)((double)bytes * kReps / ((double)ms_in * 1e3));
  if (ms_out2 > 0.f && ms_in2 > 0.f) {
    out->d2h_duplex_bytes_per_us = std::min(out->d2h_bytes_per_us, (uint64_t)((double)bytes * kReps / ((double)ms_out2 * 1e3)));
    out->h2d_duplex_bytes_per_us = std::min(out->h2d_bytes_per_us, (uint64_t)((double)bytes * kReps / ((double)ms_in2 * 1e3)));
  }
  return DP_OK;
}

dp_status dp_stage_set_debug(dp_stage *st, uint32_t flags) {
  if (st == nullptr) return fail(DP_E_INVAL, "stage handle is null");
  st->debug = flags;
  return DP_OK;
}

void dp_stage_destroy(dp_stage *st) {
  if (st == nullptr) return;
  (void)hipDeviceSynchronize();
  for (hipEvent_t e : st->events) (void)hipEventDestroy(e);
  for (hipEvent_t e : st->prof_events) (void)hipEventDestroy(e);
  for (hipEvent_t e : st->step_end) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : st->bwd_end) if (e) (void)hipEventDestroy(e);
  if (st->d2h) (void)hipStreamDestroy(st->d2h);
  if (st->h2d) (void)hipStreamDestroy(st->h2d);
  if (st->d2hx) (void)hipStreamDestroy(st->d2hx);
  for (hipEvent_t e : st->span_events) (void)hipEventDestroy(e);
  if (st->arena) (void)hipFree(st->arena);
  if (st->host_pool) (void)hipHostFree(st->host_pool);
  for (auto &f : st->flights) {
    if (!f) continue;
    delete f->walk;
    for (hipEvent_t e : f->events) (void)hipEventDestroy(e);
    if (f->done) (void)hipEventDestroy(f->done);
    if (f->arena) (void)hipFree(f->arena);
    if (f->host_pool) (void)hipHostFree(f->host_pool);
  }
  for (auto &v : st->versions) {
    if (v->ready) (void)hipEventDestroy(v->ready);
    if (v->last_use) (void)hipEventDestroy(v->last_use);
    if (v->slab) (void)hipFree(v->slab);
    if (v->xslab) (void)hipFree(v->xslab);
  }
  delete st;
}

}  // extern "C"
