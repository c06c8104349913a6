// Host-only driver for sanitizer builds: runs the library's pure host entry points (plan
// validation, plan cost, plan generation, partition search) over a few stage shapes and plans,
// so that AddressSanitizer/UBSan (and ThreadSanitizer for the planner's worker threads) see the
// dry walk, the offset allocator and the planners at work.  Never touches a GPU.
#include "../../include/dpstage.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

static dp_stage_config cfg_of(int L, int H, int nh, int F, int S, int B, int pre, int causal, int mem_seq) {
  dp_stage_config c;
  memset(&c, 0, sizeof c);
  c.n_layers = L; c.hidden = H; c.n_heads = nh; c.ffn = F; c.seq = S; c.micro_batch = B;
  c.norm_style = pre ? DP_PRE_LN : DP_POST_LN; c.causal = causal; c.gelu_kind = DP_GELU_ERF; c.dtype = DP_BF16;
  c.ln_eps = 1e-5f; c.mem_seq = mem_seq; c.norm_kind = DP_NORM_LAYER;
  return c;
}

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static uint32_t next_u32() {   // splitmix64
  uint64_t z = (rng_state += 0x9e3779b97f4a7c15ull);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return (uint32_t)((z ^ (z >> 31)) >> 16);
}

#define CHECK(cond)                                                                    \
  do {                                                                                 \
    if (!(cond)) { fprintf(stderr, "host_check: %s failed at line %d: %s\n", #cond, __LINE__, dp_last_error()); return 1; } \
  } while (0)

int main() {
  const dp_stage_config shapes[] = {
      cfg_of(3, 128, 2, 512, 64, 2, 1, 1, 0),   cfg_of(2, 256, 4, 1024, 128, 2, 0, 0, 0),
      cfg_of(6, 1024, 16, 4096, 512, 8, 0, 0, 0), cfg_of(8, 1600, 25, 6400, 1024, 4, 1, 1, 0),
      cfg_of(2, 128, 2, 256, 64, 2, 1, 1, 40),
  };
  dp_cost_model cm;
  memset(&cm, 0, sizeof cm);
  const int64_t f[8] = {8000, 300000, 190000, 120000, 8000, 380000, 60000, 380000};
  const int64_t b[8] = {760000, 70000, 760000, 12000, 240000, 520000, 600000, 12000};
  for (int i = 0; i < 8; ++i) { cm.fwd_ns[i] = f[i]; cm.bwd_ns[i] = b[i]; }
  for (int i = 0; i < 5; ++i) { cm.fwd_more_ns[i] = 100000 + 1000 * i; cm.bwd_more_ns[i] = 200000 + 1000 * i; }
  cm.d2h_bytes_per_us = cm.h2d_bytes_per_us = 57000;
  cm.d2h_duplex_bytes_per_us = 32000; cm.h2d_duplex_bytes_per_us = 28000;

  for (const dp_stage_config &c : shapes) {
    const size_t n = dp_plan_len(&c);
    CHECK(n > 0);
    const size_t per_layer = n / (size_t)c.n_layers;
    std::vector<uint8_t> plan(n, DP_KEEP);
    dp_plan_report keep;
    CHECK(dp_plan_validate(&c, plan.data(), n, 0, 1, &keep) == DP_OK);
    // seeded plans under no budget, a generous one and the keep-all peak (every policy tier of the validator)
    for (int trial = 0; trial < 40; ++trial) {
      for (size_t i = 0; i < n; ++i) plan[i] = (uint8_t)(next_u32() % 3);
      for (int l = 0; l < c.n_layers; ++l)
        if (plan[(size_t)l * per_layer + DP_SLOT_X_IN] == DP_RECOMPUTE && l == 0) plan[0] = DP_KEEP;
      dp_plan_report r;
      CHECK(dp_plan_validate(&c, plan.data(), n, 0, 1, &r) == DP_OK);
      CHECK(dp_plan_validate(&c, plan.data(), n, 4 * keep.peak_bytes, 1, &r) == DP_OK);
      const dp_status s = dp_plan_validate(&c, plan.data(), n, keep.peak_bytes, 2, &r);
      CHECK(s == DP_OK || s == DP_E_BUDGET);
      dp_plan_cost_report cr;
      CHECK(dp_plan_cost(&c, &cm, plan.data(), n, keep.fixed_bytes, &cr) == DP_OK);
      CHECK(cr.step_ns > 0);
    }
    // plan generation for shrinking budgets, model mode and validated mode, one and two micro-batches in flight
    std::vector<uint8_t> lean(n, DP_RECOMPUTE);
    for (int l = 0; l < c.n_layers; ++l) lean[(size_t)l * per_layer + DP_SLOT_X_IN] = DP_KEEP;
    dp_plan_report low;
    CHECK(dp_plan_validate(&c, lean.data(), n, 0, 1, &low) == DP_OK);
    for (int pct = 100; pct >= 0; pct -= 25) {
      const uint64_t budget = low.peak_bytes + (keep.peak_bytes - low.peak_bytes) * (uint64_t)pct / 100 + 4096;
      dp_memopt_report mr;
      for (uint32_t inflight = 1; inflight <= 2; ++inflight) {
        dp_status s = dp_plan_generate(&c, &cm, budget * inflight, inflight, keep.fixed_bytes, 0, plan.data(), n, &mr);
        CHECK(s == DP_OK || s == DP_E_BUDGET);
        s = dp_plan_generate(&c, &cm, budget * inflight, inflight, 0, DP_MEMOPT_VALIDATE, plan.data(), n, &mr);
        CHECK(s == DP_OK || s == DP_E_BUDGET);
      }
    }
  }
  // partition search over a chain of the second-widest shape
  {
    dp_stage_config chain = cfg_of(12, 1024, 16, 4096, 512, 8, 1, 1, 0);
    const size_t n = dp_plan_len(&chain);
    std::vector<uint8_t> plans(n);
    dp_stage_config one = chain;
    one.n_layers = 1;
    std::vector<uint8_t> p1(dp_plan_len(&one), DP_KEEP);
    dp_plan_report r1;
    CHECK(dp_plan_validate(&one, p1.data(), p1.size(), 0, 1, &r1) == DP_OK);
    const uint64_t fl = r1.weight_bytes + r1.grad_bytes, fs = r1.fixed_bytes - fl;
    for (int stages = 2; stages <= 4; ++stages)
      for (uint32_t flags = 0; flags <= DP_MEMOPT_VALIDATE; ++flags)
        for (uint64_t gb = 2; gb <= 8; gb *= 2) {
          std::vector<int32_t> cuts((size_t)stages - 1);
          std::vector<dp_partition_stage> st((size_t)stages);
          dp_partition_report pr;
          const dp_status s = dp_partition(&chain, &cm, stages, gb * 1000000000ull, fl, fs, nullptr, nullptr, flags,
                                           cuts.data(), plans.data(), n, st.data(), &pr);
          CHECK(s == DP_OK || s == DP_E_BUDGET);
        }
  }
  // argument errors leave nothing behind
  CHECK(dp_plan_validate(nullptr, nullptr, 0, 0, 1, nullptr) == DP_E_INVAL);
  CHECK(dp_plan_len(nullptr) == 0);
  printf("host_check ok\n");
  return 0;
}
