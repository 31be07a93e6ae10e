"""The tree attention normally starts from the QKV GEMM's partial sums (reduce + RoPE + cache write in its prologue).
The library also keeps the unfused order of the same steps (a RoPE + cache-write kernel, then the attention kernel on
rotated queries), which it falls back to when the partial sums do not come in 128-column bands.  A test hook of the
library (include/medusa_bench.h) forces that order, so these cases run the same layer parity checks with the hook
set: ragged and empty prefixes, both query-per-workgroup variants, 16-bit and 8-bit cache rows.  They run in a child
process so that the process-global hook can never leak into other tests."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r"""
import sys
sys.path.insert(0, {root!r})
import paper_2603_03383_amd as P
from tests import test_gpu_parity as TP, test_gpu_kv8 as TK
assert P.medusa_test_force_unfused_rope(True) is False
P.medusa_profile_begin(64)
TP.test_small_bf16_layer_ragged_and_empty_prefix([77], 100)
prof = P.medusa_profile_end()
assert prof.get("rope", dict(launches=0))["launches"] >= 1, prof   # the separate RoPE + cache-write kernel did run
print("unfused path taken", flush=True)
for S_list, max_prefix in [([0], 0), ([77], 100), ([300, 0, 45], 300), ([5000, 131], 5003), ([33], 33)]:
    TP.test_small_bf16_layer_ragged_and_empty_prefix(S_list, max_prefix)
    print("small layer", S_list, "ok", flush=True)
TP.test_cfg2_full_size_layer_bf16()
print("full-size layer ok", flush=True)
TK.test_7b_width_layer_8bit_rows([1024], 1024, 8, "fp16")
print("8-bit rows ok", flush=True)
"""


@pytest.mark.gpu
def test_layer_parity_with_the_unfused_rope_and_cache_write():
    r = subprocess.run([sys.executable, "-u", "-c", CHILD.format(root=ROOT)], cwd=ROOT, capture_output=True,
                       text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "unfused path taken" in r.stdout and "8-bit rows ok" in r.stdout
