"""GPU parity in fp16 storage (Section 4.1 of the paper: inference runs in Float16): the same entry points and kernels
as bf16 with the element type switched, against the oracle with fp16 storage rounding.  The bound is the bf16 one
scaled by 2^-3 (see TOL in test_gpu_parity)."""
import numpy as np
import pytest
import torch

import workload as W
import paper_2603_03383_amd as P
from oracle import medusa as O
from tests import gpu_util as G
from tests import util as U
from tests.test_gpu_parity import TOL, _i32, _scale, check_argmax_near_tie, _layer_case, _check_layer, ragged_batch_case
from tests.test_gpu_gqa import two_layer_step_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("S_list,max_prefix", [([0], 0), ([77], 100), ([512], 512), ([300, 0, 45], 300), ([5000], 5003)])
@pytest.mark.parametrize("kv_heads", [0, 8], ids=["mha", "gqa8"])
def test_7b_width_layer_fp16(S_list, max_prefix, kv_heads):
    w = W.CONFIGS["cfg2_layer_bf16"].with_(name="layer_fp16", dtype="fp16", n_kv_heads=kv_heads, prefix=tuple(S_list))
    r = _layer_case(w, S_list, max_prefix, x_seed="fp16_layer_x")
    rel = _check_layer(r, S_list, "fp16")
    print(f"fp16 layer {S_list} kv_heads={kv_heads}: err/scale {rel:.3e}")


@pytest.mark.parametrize("S_list,max_prefix", [([0, 33, 1000], 1000), ([4097], 4100)])
def test_7b_width_autoregressive_layer_fp16(S_list, max_prefix):
    w = W.CONFIGS["cfg2_layer_bf16"].with_(name="ar_layer_fp16", dtype="fp16", tree=W.TREE1, prefix=tuple(S_list))
    r = _layer_case(w, S_list, max_prefix, x_seed="fp16_ar_x")
    rel = _check_layer(r, S_list, "fp16")
    print(f"fp16 AR layer {S_list}: err/scale {rel:.3e}")


def test_two_layer_step_fp16():
    two_layer_step_case(W.CONFIGS["cfg3_step_1k"].with_(name="step_fp16", n_layers=2, dtype="fp16"))


def test_ragged_batch_16_sequences_fp16():
    """rows = 1024: the many-row GEMM kernel in fp16, heads, selection, acceptance, per-sequence compaction."""
    ragged_batch_case(W.CONFIGS["cfg5_ragged_b16"].with_(name="ragged_fp16", n_layers=1, dtype="fp16"))


def test_small_shapes_take_the_portable_kernels_fp16():
    """head_dim 64 and a 15-node tree: neither MFMA attention kernel applies, so fp16 runs through the portable
    attention, RoPE and SwiGLU kernels (and the streaming GEMM where the shapes allow)."""
    w = W.CONFIGS["cfg1_tiny_fp32"].with_(name="tiny_fp16", dtype="fp16", ffn=704)   # gate/up tiles interleave in 32 rows
    S = w.prefix[0]
    tol = TOL["fp16"]
    model = U.oracle_model(w)
    tree = U.oracle_tree(w)
    T = tree["T"]
    kc, vc = U.oracle_prefix_cache(w, 0, S + T)
    dm = G.device_model(w)
    kv = G.device_kv_random_prefix(dm, w, cap=S + T)
    tokens = W.random_tokens(w, "fp16_tiny_tokens", (T,)).to(torch.int32)
    buf = P.StepBuffers(dm, 1, S, want_logits=True)
    buf.tree_tokens.copy_(tokens.view(1, T).to(G.DEV))
    seq_len = _i32([S])
    P.run_step(dm, kv, buf, None, None, None, seq_len, with_heads=False)
    torch.cuda.synchronize()
    ref = O.tree_verify_step(tokens.numpy(), model, kc, vc, S, tree)
    g = buf.logits[0].cpu().numpy()
    lscale = _scale(ref["logits"])
    err = np.abs(g - ref["logits"]).max()
    print(f"tiny fp16 step: logits err/scale {err / lscale:.3e}")
    assert err <= tol * lscale
    gpu_am = buf.node_argmax[0].cpu().numpy()
    check_argmax_near_tie(gpu_am, g, ref["logits"], tol * lscale)
    acc = O.accept_longest_prefix(tree, tokens.numpy(), gpu_am)
    assert int(buf.accept_len[0]) == acc["accept_len"] and int(seq_len[0]) == S + acc["accept_len"]
