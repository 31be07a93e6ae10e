"""The per-family timing that bench.py reports (include/medusa_bench.h: medusa_profile_begin / _end): launch counts of
one step are what the path's structure says, every duration is positive, and their sum does not exceed the wall
clock of the same steps."""
import time

import pytest
import torch

import workload as W
import paper_2603_03383_amd as P
from tests import gpu_util as G
from tests.test_gpu_parity import _i32

pytestmark = pytest.mark.gpu


def test_launch_counts_and_durations_of_a_two_layer_step():
    w = W.CONFIGS["cfg3_step_1k"].with_(name="profile_api", n_layers=2)
    L, S = w.n_layers, w.prefix[0]
    dm = G.device_model(w)
    T, K = dm.tree_info["T"], dm.tree_info["K"]
    kv = G.device_kv_random_prefix(dm, w, cap=S + T + 64)
    buf = P.StepBuffers(dm, 1, S + 32)
    hidden = W.hidden_state(w, "profile_h", 1, device=G.DEV).view(1, 1, w.d).contiguous()
    src_row = _i32([0])
    root = _i32([7])
    seq_len = _i32([S])

    def step():
        seq_len.copy_(_i32([S]))
        P.run_step(dm, kv, buf, hidden, src_row, root, seq_len)

    step()
    torch.cuda.synchronize()
    steps = 4
    P.medusa_profile_begin(steps * 64)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    prof = P.medusa_profile_end()
    torch.cuda.synchronize()
    wall_us = (time.perf_counter() - t0) * 1e6
    assert "dropped" not in prof
    per_step = {k: v["launches"] / steps for k, v in prof.items()}
    assert per_step["gemm_w64"] == 4 * L + 1                 # QKV, O, gate/up, down per layer + the LM head
    assert per_step["gemm_w32"] == 1 + K                     # the heads' stacked first layers + K vocabulary projections
    assert per_step["attention"] == 2 * L                    # tree kernel + merge of the key-splits (three at this prefix)
    assert per_step["rmsnorm"] == 2 * L + 1                  # first norm (+ RoPE table), two per layer
    assert per_step["accept"] == 1 and per_step["kv_compact"] == 1 and per_step["embed"] == 1
    assert all(v["total_us"] > 0 and v["min_us"] > 0 and v["max_us"] >= v["min_us"] for v in prof.values())
    assert sum(v["total_us"] for v in prof.values()) <= wall_us
    # a second recording starts from zero
    P.medusa_profile_begin(8)
    assert P.medusa_profile_end() == {}
