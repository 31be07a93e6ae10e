"""tree_verify_layer_static (the entry point that allocates nothing: its scratch is a fixed device buffer inside the
library) against tree_verify_layer with a caller workspace, through the C-ABI: bit-identical layer outputs and cache
rows on two calls in a row, the second on a smaller input (a shorter prefix, so other split counts and a smaller part
of the shared scratch), and a clear refusal of a shape beyond the buffer."""
import pytest
import torch

import workload as W
import paper_2603_03383_amd as P
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _run_both(dm, w, S, max_prefix, x_seed):
    T = w.tree.n_nodes
    outs = []
    for static in (False, True):
        kv = P.DeviceKV(dm, batch=1, cap=max_prefix + T, n_layers=1)
        if S:
            k, v = W.prefix_kv(w.with_(prefix=(S,)), 0, 0, G.DEV)
            kv.write(0, 0, 0, k, v)
        x = W.hidden_state(w, x_seed, T, device=G.DEV).float()
        seq_len = torch.tensor([S], dtype=torch.int32, device=G.DEV)
        if static:
            P.tree_verify_layer_static(dm.desc, dm.layer(0), 0, x, kv.desc, seq_len, 1, max_prefix)
        else:
            ws = dm.workspace(1, max_prefix)
            P.tree_verify_layer(dm.desc, dm.layer(0), 0, x, kv.desc, seq_len, 1, max_prefix, ws)
        torch.cuda.synchronize()
        k_rows, v_rows = kv.read(0, 0, S, T)
        outs.append((x.clone(), k_rows.clone(), v_rows.clone()))
    return outs


def test_static_scratch_layer_equals_workspace_layer_twice_second_call_smaller():
    w = W.CONFIGS["cfg2_layer_bf16"]
    dm = G.device_model(w.with_(vocab=1024), heads=False, n_layers=1)
    assert P.tree_verify_layer_static_scratch_bytes() >= 32 << 20
    for S, max_prefix, seed in [(512, 512, "static_x0"), (77, 100, "static_x1")]:      # second call: smaller input
        (x0, k0, v0), (x1, k1, v1) = _run_both(dm, w, S, max_prefix, seed)
        assert torch.isfinite(x0).all() and float(x0.abs().max()) > 1.0
        assert torch.equal(x0, x1), f"S={S}: layer output differs from tree_verify_layer"
        assert torch.equal(k0, k1) and torch.equal(v0, v1), f"S={S}: cache rows differ"
    # a batch whose scratch need exceeds the built-in buffer is refused, nothing is enqueued
    kv = P.DeviceKV(dm, batch=4, cap=1024 + w.tree.n_nodes, n_layers=1)
    x = torch.zeros(4 * w.tree.n_nodes, w.d, dtype=torch.float32, device=G.DEV)
    seq_len = torch.tensor([1024] * 4, dtype=torch.int32, device=G.DEV)
    with pytest.raises(P.MedusaError) as e:
        P.tree_verify_layer_static(dm.desc, dm.layer(0), 0, x, kv.desc, seq_len, 4, 1024)
    assert e.value.status == -4 and "built-in buffer" in str(e.value)
    torch.cuda.synchronize()
    assert float(x.abs().max()) == 0.0
