"""The boundary is a C ABI: include/dpstage.h must compile as plain C (C99, no C++), and a C program must be
able to link the library and call its host-only entry points without any Python or torch in between."""
import os
import shutil
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_DIR = os.path.join(ROOT, "paper_2505_05856_amd")

PROGRAM = r'''
#include "dpstage.h"
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int main(void) {
  dp_stage_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = 4; cfg.hidden = 64; cfg.n_heads = 2; cfg.ffn = 256; cfg.seq = 32; cfg.micro_batch = 2;
  cfg.norm_style = DP_PRE_LN; cfg.causal = 1; cfg.gelu_kind = DP_GELU_ERF; cfg.dtype = DP_BF16; cfg.ln_eps = 1e-5f;
  size_t n = dp_plan_len(&cfg);
  if (n != 4 * DP_SLOTS_PER_LAYER) return 1;
  uint8_t *plan = (uint8_t *)calloc(n, 1);
  dp_plan_report rep;
  if (dp_plan_validate(&cfg, plan, n, 0, 1, &rep) != DP_OK) { printf("%s\n", dp_last_error()); return 2; }
  const uint64_t keep_peak = rep.peak_bytes;
  if (dp_plan_validate(&cfg, plan, n, keep_peak - 1, 1, &rep) != DP_E_BUDGET) return 3;
  plan[DP_SLOT_X_IN] = DP_RECOMPUTE;                       /* the stage input has no producer */
  if (dp_plan_validate(&cfg, plan, n, 0, 1, &rep) != DP_E_PLAN || rep.first_bad_slot != DP_SLOT_X_IN) return 4;
  plan[DP_SLOT_X_IN] = DP_KEEP;
  dp_cost_model cm;
  memset(&cm, 0, sizeof cm);
  for (int i = 0; i < 8; ++i) { cm.fwd_ns[i] = 10000 + 1000 * i; cm.bwd_ns[i] = 20000 + 1500 * i; }
  cm.d2h_bytes_per_us = cm.h2d_bytes_per_us = 2000;
  /* a budget halfway between recomputing everything but the layer inputs and keeping everything */
  for (size_t i = 0; i < n; ++i) plan[i] = (i % DP_SLOTS_PER_LAYER == DP_SLOT_X_IN) ? DP_KEEP : DP_RECOMPUTE;
  if (dp_plan_validate(&cfg, plan, n, 0, 1, &rep) != DP_OK || rep.peak_bytes >= keep_peak) return 9;
  const uint64_t budget = (rep.peak_bytes + keep_peak) / 2;
  dp_memopt_report mr;
  if (dp_plan_generate(&cfg, &cm, budget, 1, 0, DP_MEMOPT_VALIDATE, plan, n, &mr) != DP_OK) {
    printf("%s\n", dp_last_error()); return 5;
  }
  if (dp_plan_validate(&cfg, plan, n, budget, 1, &rep) != DP_OK || rep.peak_bytes > budget) return 6;
  int32_t cuts[1];
  dp_partition_stage stages[2];
  dp_partition_report pr;
  if (dp_partition(&cfg, &cm, 2, 0, 1000, 1000, NULL, NULL, 0, cuts, plan, n, stages, &pr) != DP_OK) return 7;
  if (cuts[0] != 2 || stages[0].inflight != 2 || stages[1].inflight != 1) return 8;
  printf("ok peak=%llu generated_peak=%llu cut=%d\n", (unsigned long long)keep_peak,
         (unsigned long long)rep.peak_bytes, (int)cuts[0]);
  free(plan);
  return 0;
}
'''


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no C compiler")
def test_header_is_c99_and_the_library_links_from_c(tmp_path):
    lib = os.path.join(LIB_DIR, "libdpstage.so")
    if not os.path.exists(lib):
        pytest.skip("library not built")
    src = tmp_path / "use_dpstage.c"
    src.write_text(PROGRAM)
    exe = tmp_path / "use_dpstage"
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           str(src), "-o", str(exe), "-L", LIB_DIR, "-ldpstage", "-Wl,-rpath," + LIB_DIR,
           "-Wl,-rpath,/opt/rocm/lib", "-Wl,--allow-shlib-undefined"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert r.stdout.startswith("ok ")
