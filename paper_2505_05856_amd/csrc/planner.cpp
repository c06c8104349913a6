// The planners of dpstage: the cost model of a plan and the memory-optimisation step of
// Section 4.3 (dp_plan_cost, dp_plan_generate), and the pipeline partition search of
// Section 4.2 / Appendix B.1 over a chain of layers (dp_partition).  Host only: everything
// here runs the step's walk dry.
#include "stage_internal.h"

#include <algorithm>
#include <array>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <thread>
#include <vector>

namespace dpi {

dp_status check_cost_model(const dp_cost_model *cm) {
  if (cm == nullptr) return fail(DP_E_INVAL, "cost model is null");
  for (int i = 0; i < N_OPS_CROSS; ++i)
    if (node_fwd_ns(*cm, i) < 0 || node_bwd_ns(*cm, i) < 0) return fail(DP_E_INVAL, "negative node time in the cost model");
  if (cm->d2h_bytes_per_us == 0 || cm->h2d_bytes_per_us == 0) return fail(DP_E_INVAL, "link speed is zero");
  return DP_OK;
}

extern const BwdReads kPreBwd[N_OPS] = {
    {1, {DP_SLOT_GELU_OUT}}, {1, {DP_SLOT_FC1_OUT}}, {1, {DP_SLOT_LN2_OUT}}, {2, {DP_SLOT_RES1, DP_SLOT_LN2_STATS}},
    {1, {DP_SLOT_ATTN_OUT}}, {3, {DP_SLOT_QKV, DP_SLOT_ATTN_OUT, DP_SLOT_ATTN_LSE}}, {1, {DP_SLOT_LN1_OUT}},
    {2, {DP_SLOT_X_IN, DP_SLOT_LN1_STATS}}};
extern const BwdReads kPostBwd[N_OPS] = {
    {2, {DP_SLOT_RES2, DP_SLOT_LN2_STATS}}, {1, {DP_SLOT_GELU_OUT}}, {1, {DP_SLOT_FC1_OUT}}, {1, {DP_SLOT_LN1_OUT}},
    {2, {DP_SLOT_RES1, DP_SLOT_LN1_STATS}}, {1, {DP_SLOT_ATTN_OUT}},
    {3, {DP_SLOT_QKV, DP_SLOT_ATTN_OUT, DP_SLOT_ATTN_LSE}}, {1, {DP_SLOT_X_IN}}};

extern const BwdReads kPreCrossBwd[N_OPS_CROSS] = {
    {1, {DP_SLOT_GELU_OUT}}, {1, {DP_SLOT_FC1_OUT}}, {1, {DP_SLOT_LN2_OUT}}, {2, {DP_SLOT_RES_C, DP_SLOT_LN2_STATS}},
    {1, {DP_SLOT_ATTN_C_OUT}}, {3, {DP_SLOT_Q_C, DP_SLOT_KV_C, DP_SLOT_ATTN_C_LSE}}, {0, {}}, {1, {DP_SLOT_LNC_OUT}},
    {2, {DP_SLOT_RES1, DP_SLOT_LNC_STATS}},
    {1, {DP_SLOT_ATTN_OUT}}, {3, {DP_SLOT_QKV, DP_SLOT_ATTN_OUT, DP_SLOT_ATTN_LSE}}, {1, {DP_SLOT_LN1_OUT}},
    {2, {DP_SLOT_X_IN, DP_SLOT_LN1_STATS}}};

struct Cand { int l, slot; int64_t free_ns; };

// fn(i) for i in [0, n) on up to 16 host threads (DPSTAGE_PLANNER_THREADS overrides; 1 = inline).  The
// planner's trial plans are independent walks; their results are read back in index order, so the
// outcome does not depend on how many threads ran them.
template <typename F>
void parallel_for(size_t n, F fn) {
  unsigned want = std::min(16u, std::max(1u, std::thread::hardware_concurrency()));
  if (const char *env = getenv("DPSTAGE_PLANNER_THREADS")) want = (unsigned)std::max(1, atoi(env));
  const size_t nt = std::min<size_t>(want, n);
  if (nt <= 1) { for (size_t i = 0; i < n; ++i) fn(i); return; }
  std::atomic<size_t> next{0};
  auto work = [&] { for (size_t i = next++; i < n; i = next++) fn(i); };
  std::vector<std::thread> pool;
  for (size_t t = 1; t < nt; ++t) pool.emplace_back(work);
  work();
  for (std::thread &t : pool) t.join();
}

// The planner proper (Section 4.3): swaps by decreasing FreeTime while they stay hidden, then
// the action with the most memory saved per second of overhead, until inflight * peak fits.
// Peak = fixed_bytes + running peak of the saved tensors.  Returns false if it cannot fit.
// The model a planner uses for a stage with `inflight` micro-batches between forward and
// backward: from two on, copy-outs of one micro-batch and copy-ins of another run side by side
// all the time, so the two-way link speed applies where it is known.
dp_cost_model for_inflight(const dp_cost_model &cm, uint32_t inflight) {
  dp_cost_model e = cm;
  if (inflight >= 2) {
    if (cm.d2h_duplex_bytes_per_us) e.d2h_bytes_per_us = cm.d2h_duplex_bytes_per_us;
    if (cm.h2d_duplex_bytes_per_us) e.h2d_bytes_per_us = cm.h2d_duplex_bytes_per_us;
  }
  return e;
}

bool memopt(const Cfg &c, const dp_cost_model &cm_given, uint64_t budget, uint32_t inflight, uint64_t fixed_bytes,
            std::vector<uint8_t> &plan, dp_memopt_report *rep) {
  const dp_cost_model cm = for_inflight(cm_given, inflight);
  const OpDef *ops = op_table(c);
  const BwdReads *bwd = bwd_table(c);
  const int n_ops = op_count(c), ns = c.nslots;
  plan.assign((size_t)c.L * (size_t)ns, DP_KEEP);
  auto cost = [&](const std::vector<uint8_t> &p, int64_t *t, uint64_t *peak) {
    const CostOut o = walk_cost(c, cm, p.data(), false, SwapPolicy{});
    *t = o.step_ns; *peak = fixed_bytes + o.slot_peak;
  };
  auto fits = [&](uint64_t peak) { return budget == 0 || (unsigned __int128)inflight * peak <= budget; };
  int64_t T; uint64_t P;
  cost(plan, &T, &P);
  const int64_t base = T;
  // FreeTime on the timeline of the unoptimised step
  int64_t fsum = 0, bsum = 0, fend[N_OPS_CROSS], bstart[N_OPS_CROSS];
  for (int i = 0; i < n_ops; ++i) { fsum += node_fwd_ns(cm, i); fend[i] = fsum; }
  for (int i = 0; i < n_ops; ++i) { bstart[i] = bsum; bsum += node_bwd_ns(cm, i); }
  std::vector<Cand> cands;
  for (int l = 0; l < c.L; ++l)
    for (int s = 0; s < ns; ++s) {
      if (slot_bytes(c, s) == 0 || (l == 0 && s == DP_SLOT_X_IN)) continue;
      int last = -1, first = -1;
      for (int i = 0; i < n_ops; ++i) {
        for (int k = 0; k < ops[i].n_in; ++k) if (ops[i].in[k].dl == 0 && ops[i].in[k].slot == s) last = i;
        for (int k = 0; k < ops[i].n_out; ++k) if (ops[i].out[k].dl == 0 && ops[i].out[k].slot == s) last = i;
      }
      for (int i = n_ops - 1; i >= 0; --i)
        for (int k = 0; k < bwd[i].n; ++k) if (bwd[i].slot[k] == s) first = i;
      const int64_t last_end = (int64_t)l * fsum + fend[last];
      const int64_t first_start = (int64_t)c.L * fsum + (int64_t)(c.L - 1 - l) * bsum + bstart[first];
      const uint64_t b = slot_bytes(c, s);
      cands.push_back({l, s, (first_start - copy_ns(b, cm.h2d_bytes_per_us)) -
                                 (last_end + copy_ns(b, cm.d2h_bytes_per_us))});
    }
  std::stable_sort(cands.begin(), cands.end(), [](const Cand &a, const Cand &b) { return a.free_ns > b.free_ns; });
  auto idx = [ns](const Cand &k) { return (size_t)k.l * (size_t)ns + k.slot; };
  int n_free = 0, n_paid = 0, n_rec = 0;
  // phase 1
  for (const Cand &k : cands) {
    if (fits(P)) break;
    std::vector<uint8_t> trial = plan;
    trial[idx(k)] = DP_SWAP;
    int64_t T1; uint64_t P1;
    cost(trial, &T1, &P1);
    if (T1 > T) break;
    plan.swap(trial); T = T1; P = P1; ++n_free;
  }
  // phase 2
  std::vector<Cand> rest;
  for (const Cand &k : cands) if (plan[idx(k)] == DP_KEEP) rest.push_back(k);
  bool ok = true;
  while (!fits(P)) {
    int best = -1, best_a = 0; int64_t best_dt = 0, best_T = 0; uint64_t best_saved = 0, best_P = 0;
    // every remaining candidate under both actions: independent walks, played side by side
    const int actions[2] = {(int)DP_SWAP, (int)DP_RECOMPUTE};
    std::vector<std::pair<int64_t, uint64_t>> played(rest.size() * 2);
    parallel_for(played.size(), [&](size_t i) {
      std::vector<uint8_t> trial = plan;
      trial[idx(rest[i / 2])] = (uint8_t)actions[i % 2];
      cost(trial, &played[i].first, &played[i].second);
    });
    // first pass: changes that lower the peak, rated by the reduction; if there is none (two
    // moments share the peak): changes that do not raise it, rated by the tensor's size
    for (int plateau = 0; plateau < 2 && best < 0; ++plateau)
      for (size_t pos = 0; pos < rest.size(); ++pos)
        for (int ai = 0; ai < 2; ++ai) {
          const int a = actions[ai];
          const int64_t T1 = played[pos * 2 + (size_t)ai].first;
          const uint64_t P1 = played[pos * 2 + (size_t)ai].second;
          if (plateau ? P1 > P : P1 >= P) continue;
          const uint64_t saved = plateau ? slot_bytes(c, rest[pos].slot) : P - P1;
          const int64_t dt = std::max<int64_t>(T1 - T, 0);
          bool better = best < 0;
          if (!better) {
            const unsigned __int128 lhs = (unsigned __int128)saved * (unsigned __int128)(best_dt + 1);
            const unsigned __int128 rhs = (unsigned __int128)best_saved * (unsigned __int128)(dt + 1);
            better = lhs > rhs || (lhs == rhs && dt < best_dt);
          }
          if (better) { best = (int)pos; best_a = a; best_dt = dt; best_saved = saved; best_T = T1; best_P = P1; }
        }
    if (best < 0) { ok = false; break; }
    plan[idx(rest[(size_t)best])] = (uint8_t)best_a;
    T = best_T; P = best_P;
    if (best_a == DP_SWAP) ++n_paid; else ++n_rec;
    rest.erase(rest.begin() + best);
  }
  if (rep) {
    rep->feasible = ok ? 1 : 0; rep->base_ns = base; rep->moo_ns = T - base; rep->peak_bytes = P;
    rep->n_free_swaps = n_free; rep->n_paid_swaps = n_paid; rep->n_recomputed = n_rec;
  }
  return ok;
}

// MemOpt against the executor: the model sees saved tensors only, the executor also holds
// transient gradients, workspaces and fragmentation.  Plan for the model, ask the validator for
// the true peak, and hand the difference back to the model as a smaller budget until it fits.
// DP_OK, DP_E_BUDGET (plan and report of the last round) or a validator error.
dp_status memopt_validated(const Cfg &c, const dp_cost_model &cm, uint64_t budget_bytes, uint32_t inflight,
                                  std::vector<uint8_t> &plan, dp_memopt_report *r) {
  const size_t plan_len = (size_t)c.L * (size_t)c.nslots;
  dp_plan_report keep;
  plan.assign(plan_len, DP_KEEP);
  (void)validate(c, plan.data(), plan_len, 0, 1, &keep, env_mfma_enabled(), kFuseGeluDefault);
  const uint64_t fixed = keep.fixed_bytes;
  uint64_t model_budget = budget_bytes;
  for (int round = 1; round <= 6; ++round) {
    r->refine_rounds = round;
    const bool ok = memopt(c, cm, model_budget, inflight, fixed, plan, r);
    dp_plan_report vr;
    SwapPolicy hold;
    const dp_status vs = validate(c, plan.data(), plan_len, budget_bytes, inflight, &vr, env_mfma_enabled(), kFuseGeluDefault, &hold);
    r->validated_peak_bytes = vr.peak_bytes;
    if (vs == DP_OK) {
      r->feasible = 1;
      r->exact_step_ns = walk_cost(c, for_inflight(cm, inflight), plan.data(), true, hold).step_ns;
      return DP_OK;
    }
    if (vs != DP_E_BUDGET) return vs;
    if (!ok || budget_bytes == 0) break;
    const uint64_t excess = vr.peak_bytes > r->peak_bytes ? vr.peak_bytes - r->peak_bytes : 0;
    const uint64_t target = budget_bytes / inflight;
    const uint64_t next = target > excess ? (target - excess) * inflight : 0;
    if (next == 0 || next >= model_budget) { if (model_budget < 2) break; model_budget = std::min(model_budget - 1, next ? next : model_budget / 2); }
    else model_budget = next;
  }
  // The greedy phase can end a few percent above the smallest peak a plan can have.  Last resort:
  // recompute everything (each layer's input kept), the plan with the least saved memory that
  // moves nothing over the link.
  if (budget_bytes != 0) {
    std::vector<uint8_t> lean(plan_len, DP_RECOMPUTE);
    for (int l = 0; l < c.L; ++l) lean[(size_t)l * (size_t)c.nslots + DP_SLOT_X_IN] = DP_KEEP;
    dp_plan_report vr;
    SwapPolicy hold;
    if (validate(c, lean.data(), plan_len, budget_bytes, inflight, &vr, env_mfma_enabled(), kFuseGeluDefault, &hold) == DP_OK) {
      const dp_cost_model cmi = for_inflight(cm, inflight);
      const CostOut o = walk_cost(c, cmi, lean.data(), false, SwapPolicy{});
      plan = lean;
      r->feasible = 1;
      r->moo_ns = o.step_ns - r->base_ns;
      r->peak_bytes = fixed + o.slot_peak;
      r->n_free_swaps = r->n_paid_swaps = 0;
      r->n_recomputed = 0;
      for (size_t k = 0; k < plan_len; ++k) r->n_recomputed += lean[k] == DP_RECOMPUTE;
      r->validated_peak_bytes = vr.peak_bytes;
      r->exact_step_ns = walk_cost(c, cmi, lean.data(), true, hold).step_ns;
      return DP_OK;
    }
  }
  r->feasible = 0;
  return DP_E_BUDGET;
}

}  // namespace dpi
using namespace dpi;

// ------------------------------------------------------------------ partition search
// Section 4.2 (Algorithm 1: AdjacentPartition, BiPar) over a chain of identical layers, with
// Appendix B.1's balance walks (Algorithm 2) for the two ends of every traversal and memopt()
// above as the MemOpt step.  Cuts fall between layers.  Stage x of l keeps l - x + 1
// micro-batches and fits when (l - x + 1) * peak <= M.
namespace {

constexpr int64_t kNever = INT64_MAX;   // a stage MemOpt cannot fit

struct StageRes {
  int64_t t = 0, base = 0, moo = 0;     // t = T_x + T_x^moo, kNever if it cannot fit
  bool mopt = false;                    // memory optimisation was needed
  uint64_t peak = 0;
  std::vector<uint8_t> plan;
};
struct SearchRes {
  int64_t t = kNever;
  bool mopt = false;
  std::vector<int> cuts;
  std::vector<std::shared_ptr<const StageRes>> stages;
};

// Algorithm 2's walk: item i adds amounts[i]; stage x's share of the total is weights[x] / sum.
// The item that reaches the target closes the stage unless the boundary in front of it is
// nearer (items are whole layers); every stage keeps at least one item.
std::vector<int> balanced_cuts(const std::vector<uint64_t> &amounts, const std::vector<uint64_t> &weights) {
  typedef unsigned __int128 u128;
  const int n = (int)amounts.size(), k = (int)weights.size();
  u128 total = 0, wsum = 0;
  for (uint64_t a : amounts) total += a;
  for (uint64_t w : weights) wsum += w;
  std::vector<int> cuts;
  int x = 0, i = 0, start = 0;
  u128 cur = 0;
  while (i < n && x < k - 1) {
    const u128 a = amounts[(size_t)i], target = total * weights[(size_t)x];
    const bool reached = (cur + a) * wsum >= target;
    if (reached && i > start && (cur + a) * wsum - target > target - cur * wsum) {
      cuts.push_back(i);
      ++x; cur = 0; start = i;
      continue;   // item i opens the next stage
    }
    cur += a;
    const bool must = n - (i + 1) == k - (x + 1);
    if (reached || must) { cuts.push_back(i + 1); ++x; cur = 0; start = i + 1; }
    ++i;
  }
  return cuts;
}

struct Partitioner {
  Cfg layer;                    // the layer shape; L is set per stage
  const dp_cost_model *cm;
  int n, ell;
  uint64_t M, fixed_per_layer, fixed_per_stage;
  std::vector<int64_t> extra_ns;
  std::vector<uint64_t> extra_bytes;
  int64_t layer_ns = 0;
  uint64_t layer_saved = 0, lcm_depths = 1;
  bool validated = false;       // stage memory from the executor's validator instead of the model
  int n_memopt = 0, n_positions = 0;
  std::vector<std::pair<std::array<int, 3>, std::shared_ptr<const StageRes>>> cache;

  void prepare() {
    for (int i = 0; i < op_count(layer); ++i) layer_ns += node_fwd_ns(*cm, i) + node_bwd_ns(*cm, i);
    for (int s = 0; s < layer.nslots; ++s) layer_saved += slot_bytes(layer, s);
    for (uint64_t d = 1; d <= (uint64_t)ell; ++d) {
      uint64_t a = lcm_depths, b = d;
      while (b) { const uint64_t r = a % b; a = b; b = r; }
      lcm_depths = lcm_depths / a * d;
    }
  }
  uint64_t time_of(int l) const { return (uint64_t)(layer_ns + extra_ns[(size_t)l]); }
  uint64_t mem_of(int l) const { return fixed_per_layer + extra_bytes[(size_t)l] + layer_saved; }

  // rho_cb, rho_mb: the cut after stage `after` when layers [a, b) are divided among stages first..last
  void comp_mem_bal(int a, int b, int first, int last, int after, int *cb, int *mb) const {
    std::vector<uint64_t> t, m, we, wm;
    for (int l = a; l < b; ++l) { t.push_back(time_of(l)); m.push_back(mem_of(l)); }
    for (int x = first; x <= last; ++x) { we.push_back(1); wm.push_back(lcm_depths / (uint64_t)(ell - x + 1)); }
    *cb = a + balanced_cuts(t, we)[(size_t)(after - first)];
    *mb = a + balanced_cuts(m, wm)[(size_t)(after - first)];
  }

  std::shared_ptr<const StageRes> stage(int a, int b, int x) {
    const std::array<int, 3> key{a, b, x};
    for (const auto &e : cache) if (e.first == key) return e.second;
    auto r = std::make_shared<StageRes>();
    Cfg c = layer;
    c.L = b - a;
    const uint32_t k = (uint32_t)(ell - x + 1);
    uint64_t fixed = fixed_per_stage + (uint64_t)c.L * fixed_per_layer;
    int64_t extra = 0;
    for (int l = a; l < b; ++l) { fixed += extra_bytes[(size_t)l]; extra += extra_ns[(size_t)l]; }
    r->plan.assign((size_t)c.L * (size_t)c.nslots, DP_KEEP);
    if (validated) {
      // The validator accounts for the library's weight copies, the gradients and the stage's
      // buffers itself; only the caller's extras come on top, as bytes no plan can remove.
      uint64_t extras = 0;
      for (int l = a; l < b; ++l) extras += extra_bytes[(size_t)l];
      const unsigned __int128 held_extras = (unsigned __int128)k * extras;   // the extras of every micro-batch in flight
      const CostOut keep = walk_cost(c, *cm, r->plan.data(), false, SwapPolicy{});
      r->base = keep.step_ns + extra;
      dp_plan_report vr;
      if (M == 0 || held_extras < M) {
        const uint64_t bk = M == 0 ? 0 : M - (uint64_t)held_extras;   // what is left for the stage proper, k times over
        if (validate(c, r->plan.data(), r->plan.size(), bk, k, &vr, env_mfma_enabled(), kFuseGeluDefault) == DP_OK) {
          r->t = r->base; r->peak = vr.peak_bytes + extras;
          cache.emplace_back(key, r);
          return r;
        }
        ++n_memopt;
        dp_memopt_report rep;
        memset(&rep, 0, sizeof rep);
        const dp_status vs = memopt_validated(c, *cm, bk, k, r->plan, &rep);
        // time: the model's clocks on the executor's own arena and hold policy where the plan runs
        r->mopt = true; r->peak = rep.validated_peak_bytes + extras;
        r->t = vs == DP_OK ? std::max(rep.exact_step_ns, rep.base_ns) + extra : kNever;
        r->moo = vs == DP_OK ? r->t - r->base : rep.moo_ns;
      } else {
        r->mopt = true; r->t = kNever; r->peak = extras;
      }
      cache.emplace_back(key, r);
      return r;
    }
    const CostOut keep = walk_cost(c, *cm, r->plan.data(), false, SwapPolicy{});
    const uint64_t keep_peak = fixed + keep.slot_peak;
    if (M == 0 || (unsigned __int128)k * keep_peak <= M) {
      r->t = r->base = keep.step_ns + extra; r->moo = 0; r->mopt = false; r->peak = keep_peak;
    } else {
      ++n_memopt;
      dp_memopt_report rep;
      memset(&rep, 0, sizeof rep);
      const bool ok = memopt(c, *cm, M, k, fixed, r->plan, &rep);
      r->mopt = true; r->base = rep.base_ns + extra; r->moo = rep.moo_ns; r->peak = rep.peak_bytes;
      r->t = ok ? rep.base_ns + rep.moo_ns + extra : kNever;
    }
    cache.emplace_back(key, r);
    return r;
  }

  // The loop AdjacentPartition and BiPar share: positions from rho_cb to rho_mb, stop where no
  // memory optimisation was needed, keep the fastest (the first on ties).  Beyond the paper:
  // if nothing in the interval fits, go on past rho_mb in the same direction (towards fewer
  // layers in the earlier stages when the two coincide) to the first position that fits.
  template <typename At>
  SearchRes traverse(int cb, int mb, int lo, int hi, At at) {
    const int step = mb > cb ? 1 : -1;
    SearchRes best;
    bool have = false;
    int last_pos = 0;
    bool any_pos = false;
    for (int rho = cb; rho != mb + step; rho += step) {
      if (rho < lo || rho > hi) continue;
      any_pos = true; last_pos = rho;
      SearchRes r = at(rho);
      const bool stop = !r.mopt;
      if (!have || r.t < best.t) { best = std::move(r); have = true; }
      if (stop) break;
    }
    if (!have || best.t == kNever) {
      int rho = (any_pos ? last_pos : std::min(std::max(mb, lo), hi)) + step;
      for (; rho >= lo && rho <= hi; rho += step) {
        SearchRes r = at(rho);
        const bool fitted = r.t < kNever;
        if (!have || fitted) { best = std::move(r); have = true; }
        if (fitted) break;
      }
    }
    return best;
  }

  SearchRes adjacent(int a, int b, int sid) {
    int cb, mb;
    comp_mem_bal(a, b, sid, sid + 1, sid, &cb, &mb);
    return traverse(cb, mb, a + 1, b - 1, [&](int rho) {
      ++n_positions;
      SearchRes r;
      auto l = stage(a, rho, sid), rt = stage(rho, b, sid + 1);
      r.t = std::max(l->t, rt->t); r.mopt = l->mopt || rt->mopt;
      r.cuts = {rho}; r.stages = {l, rt};
      return r;
    });
  }

  SearchRes bipar(int a, int b, int first, int last) {
    if (first == last) {
      SearchRes r;
      auto s = stage(a, b, first);
      r.t = s->t; r.mopt = s->mopt; r.stages = {s};
      return r;
    }
    if (last - first == 1) return adjacent(a, b, first);
    const int count = last - first + 1, mid = first + count / 2 - 1;   // three stages split 1 + 2
    int cb, mb;
    comp_mem_bal(a, b, first, last, mid, &cb, &mb);
    const int n_left = mid - first + 1, n_right = last - mid;
    return traverse(cb, mb, a + n_left, b - n_right, [&](int rho) {
      ++n_positions;
      SearchRes l = bipar(a, rho, first, mid), rt = bipar(rho, b, mid + 1, last), r;
      r.t = std::max(l.t, rt.t); r.mopt = l.mopt || rt.mopt;
      r.cuts = l.cuts; r.cuts.push_back(rho); r.cuts.insert(r.cuts.end(), rt.cuts.begin(), rt.cuts.end());
      r.stages = l.stages; r.stages.insert(r.stages.end(), rt.stages.begin(), rt.stages.end());
      return r;
    });
  }
};

}  // namespace

// ====================================================================== C ABI
extern "C" {

dp_status dp_plan_cost(const dp_stage_config *cfg, const dp_cost_model *cm, const uint8_t *plan, size_t plan_len,
                       uint64_t fixed_bytes, dp_plan_cost_report *report) {
  Cfg c;
  dp_status s = parse_cfg(cfg, &c);
  if (s != DP_OK) return s;
  if ((s = check_cost_model(cm)) != DP_OK) return s;
  if (report == nullptr) return fail(DP_E_INVAL, "report is null");
  dp_plan_report pr;
  memset(&pr, 0, sizeof pr);
  if ((s = check_plan(c, plan, plan_len, &pr)) != DP_OK) return s;
  const CostOut o = walk_cost(c, *cm, plan, false, SwapPolicy{});
  report->step_ns = o.step_ns; report->peak_bytes = fixed_bytes + o.slot_peak;
  report->d2h_bytes = o.d2h; report->h2d_bytes = o.h2d; report->n_replayed_ops = o.replayed;
  return DP_OK;
}

dp_status dp_plan_generate(const dp_stage_config *cfg, const dp_cost_model *cm, uint64_t budget_bytes,
                           uint32_t inflight, uint64_t fixed_bytes, uint32_t flags, uint8_t *plan_out, size_t plan_len,
                           dp_memopt_report *report) {
  Cfg c;
  dp_status s = parse_cfg(cfg, &c);
  if (s != DP_OK) return s;
  if ((s = check_cost_model(cm)) != DP_OK) return s;
  if (plan_out == nullptr) return fail(DP_E_INVAL, "plan_out is null");
  if (plan_len != (size_t)c.L * (size_t)c.nslots) return fail(DP_E_INVAL, "plan_len must be n_layers * %d", c.nslots);
  if (inflight < 1) return fail(DP_E_INVAL, "inflight must be >= 1");
  dp_memopt_report local;
  dp_memopt_report *r = report ? report : &local;
  memset(r, 0, sizeof *r);
  std::vector<uint8_t> plan;
  if ((flags & DP_MEMOPT_VALIDATE) == 0) {
    const bool ok = memopt(c, *cm, budget_bytes, inflight, fixed_bytes, plan, r);
    memcpy(plan_out, plan.data(), plan_len);
    return ok ? DP_OK : fail(DP_E_BUDGET, "no plan of the model fits %llu bytes", (unsigned long long)budget_bytes);
  }
  const dp_status vs = memopt_validated(c, *cm, budget_bytes, inflight, plan, r);
  memcpy(plan_out, plan.data(), plan_len);
  if (vs == DP_E_BUDGET)
    return fail(DP_E_BUDGET, "no generated plan fits %llu bytes (last true peak %llu)", (unsigned long long)budget_bytes,
                (unsigned long long)r->validated_peak_bytes);
  return vs;
}

dp_status dp_partition(const dp_stage_config *chain_cfg, const dp_cost_model *cm, int32_t n_stages,
                       uint64_t budget_bytes, uint64_t fixed_per_layer, uint64_t fixed_per_stage,
                       const int64_t *extra_ns, const uint64_t *extra_bytes, uint32_t flags, int32_t *cuts_out,
                       uint8_t *plan_out, size_t plan_len, dp_partition_stage *stages_out,
                       dp_partition_report *report) {
  Cfg c;
  dp_status s = parse_cfg(chain_cfg, &c);
  if (s != DP_OK) return s;
  if ((s = check_cost_model(cm)) != DP_OK) return s;
  if (n_stages < 1 || n_stages > 32 || n_stages > c.L)
    return fail(DP_E_INVAL, "n_stages must be 1..min(32, n_layers)");
  if (plan_out == nullptr || stages_out == nullptr || (n_stages > 1 && cuts_out == nullptr))
    return fail(DP_E_INVAL, "null output argument");
  if (plan_len != (size_t)c.L * (size_t)c.nslots) return fail(DP_E_INVAL, "plan_len must be n_layers * %d", c.nslots);
  if ((flags & ~(uint32_t)DP_MEMOPT_VALIDATE) != 0) return fail(DP_E_INVAL, "unknown flag bits 0x%x", flags);
  Partitioner p;
  p.validated = (flags & DP_MEMOPT_VALIDATE) != 0;
  p.layer = c; p.cm = cm; p.n = c.L; p.ell = n_stages; p.M = budget_bytes;
  p.fixed_per_layer = fixed_per_layer; p.fixed_per_stage = fixed_per_stage;
  p.extra_ns.assign((size_t)c.L, 0); p.extra_bytes.assign((size_t)c.L, 0);
  for (int l = 0; l < c.L; ++l) {
    if (extra_ns) { if (extra_ns[l] < 0) return fail(DP_E_INVAL, "extra_ns[%d] is negative", l); p.extra_ns[(size_t)l] = extra_ns[l]; }
    if (extra_bytes) p.extra_bytes[(size_t)l] = extra_bytes[l];
  }
  p.prepare();
  const SearchRes r = p.bipar(0, c.L, 1, n_stages);
  dp_partition_report local;
  dp_partition_report *rep = report ? report : &local;
  memset(rep, 0, sizeof *rep);
  rep->feasible = r.t < kNever; rep->time_ns = r.t; rep->any_memopt = r.mopt;
  rep->n_memopt = p.n_memopt; rep->n_positions = p.n_positions;
  if (n_stages > 1) {
    int cb, mb;
    p.comp_mem_bal(0, c.L, 1, n_stages, n_stages / 2, &cb, &mb);
    rep->rho_cb = cb; rep->rho_mb = mb;
  }
  int first = 0;
  for (int x = 1; x <= n_stages; ++x) {
    const StageRes &st = *r.stages[(size_t)(x - 1)];
    const int end = x < n_stages ? r.cuts[(size_t)(x - 1)] : c.L;
    if (x < n_stages) cuts_out[x - 1] = end;
    dp_partition_stage &o = stages_out[x - 1];
    o.first_layer = first; o.n_layers = end - first; o.inflight = n_stages - x + 1; o.used_memopt = st.mopt;
    o.time_ns = st.t; o.base_ns = st.base; o.moo_ns = st.moo; o.peak_bytes = st.peak;
    memcpy(plan_out + (size_t)first * (size_t)c.nslots, st.plan.data(), st.plan.size());
    first = end;
  }
  return rep->feasible ? DP_OK : fail(DP_E_BUDGET, "no partition into %d stages fits %llu bytes a device", n_stages,
                                      (unsigned long long)budget_bytes);
}

}  // extern "C"
