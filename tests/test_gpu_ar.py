"""GPU parity of the autoregressive baseline step: the single-node tree (T = 1, K = 0) through the same C-ABI
calls, against the oracle's causal decoder / single-node tree step, and against the 64-node tree's root row."""
import numpy as np
import pytest
import torch

import workload as W
import paper_2603_03383_amd as P
from oracle import medusa as O
from oracle import tree as OT
from tests import gpu_util as G
from tests import util as U
from tests.test_gpu_parity import TOL, _i32, _scale, check_argmax_near_tie, _layer_case, _check_layer

pytestmark = pytest.mark.gpu


def test_ar_steps_tiny_fp32_chain_matches_causal_decode():
    w = W.CONFIGS["cfg1_tiny_fp32"].with_(tree=W.TREE1)
    S = w.prefix[0]
    tol = TOL["fp32"]
    model = U.oracle_model(w, heads=False)
    tree1 = OT.build_tree((), ())
    prefix_tokens = W.random_tokens(w, "prefix", (S,)).numpy()
    kc, vc = O.empty_cache(model["cfg"], S + 8)
    lg, _ = O.causal_decode(prefix_tokens, model, kc, vc, 0)
    dm = G.device_model(w, heads=False)
    assert dm.tree_info["T"] == 1 and dm.tree_info["K"] == 0
    kv = G.device_kv_from_oracle(dm, [kc], [vc], [S], cap=S + 8)
    buf = P.StepBuffers(dm, 1, S + 7, want_logits=True)
    seq_len = _i32([S])
    root = _i32([int(np.argmax(lg[-1]))])
    tok = int(root[0])
    for step in range(4):                                              # a chained greedy decode, no host logic
        ref_logits, ref_hidden = O.causal_decode([tok], model, kc, vc, S + step)
        dummy_h = torch.zeros(1, 1, w.d, device=G.DEV)
        P.run_step(dm, kv, buf, dummy_h, None, root, seq_len)
        torch.cuda.synchronize()
        assert buf.tree_tokens.cpu().numpy().tolist() == [[tok]]
        g = buf.logits[0].cpu().numpy()
        assert np.abs(g - ref_logits).max() <= tol * _scale(ref_logits)
        assert np.abs(buf.hidden[0].cpu().numpy() - ref_hidden).max() <= tol * _scale(ref_hidden)
        assert check_argmax_near_tie(buf.node_argmax[0].cpu().numpy(), g, ref_logits, tol * _scale(ref_logits)) == 0
        assert int(buf.accept_len[0]) == 1 and buf.acc_nodes.cpu().numpy().tolist() == [[0]]
        assert buf.acc_tokens.cpu().numpy().tolist() == [[tok]]
        assert buf.kv_src_slots.cpu().numpy().tolist() == [[S + step]] and int(seq_len[0]) == S + step + 1
        tok = int(buf.next_root[0])
        assert tok == int(O.argmax_lowest(ref_logits)[0])
        root = buf.next_root.clone()
    for l in range(w.n_layers):
        k, v = kv.read(l, 0, 0, S + 4)
        np.testing.assert_allclose(k.cpu().numpy(), kc[l][:, :S + 4], rtol=0, atol=2e-5)
        np.testing.assert_allclose(v.cpu().numpy(), vc[l][:, :S + 4], rtol=0, atol=2e-5)


@pytest.mark.parametrize("S_list,max_prefix", [([0], 0), ([31], 31), ([32], 40), ([33, 0, 1000], 1000), ([4097], 4100),
                                               ([517] * 9, 600)])
def test_ar_layer_bf16_decode_attention_ragged(S_list, max_prefix):
    """One 7B-width layer, one row per sequence: M = B GEMMs and the single-query attention kernel."""
    w = W.CONFIGS["cfg2_layer_bf16"].with_(tree=W.TREE1, prefix=tuple(S_list))
    r = _layer_case(w, S_list, max_prefix, x_seed="ar_layer_x")
    rel = _check_layer(r, S_list, "bf16")
    print(f"AR layer {S_list}: err/scale {rel:.3e}")


def test_ar_step_two_layers_bf16_matches_oracle_and_the_tree_root():
    """Full AR step at 7B width (2 layers): against the oracle, and against node 0 of the 64-node tree step from the
    same prefix (the root sees exactly what the AR token sees: tree verification is a re-arrangement of causal decoding)."""
    w64 = W.CONFIGS["cfg3_step_1k"].with_(n_layers=2)
    w1 = w64.with_(tree=W.TREE1)
    S = w64.prefix[0]
    tol = TOL["bf16"]
    model = U.oracle_model(w1, device=G.DEV, heads=False)
    tree1 = OT.build_tree((), ())
    kc, vc = U.oracle_prefix_cache(w1, 0, S + 1, device=G.DEV)
    tok = 4242
    ref = O.tree_verify_step(np.array([tok]), model, kc, vc, S, tree1)

    dm1 = G.device_model(w1, heads=False)
    kv1 = G.device_kv_random_prefix(dm1, w1, cap=S + 1)
    buf1 = P.StepBuffers(dm1, 1, S, want_logits=True)
    seq1 = _i32([S])
    P.run_step(dm1, kv1, buf1, torch.zeros(1, 1, w1.d, dtype=dm1.tdtype, device=G.DEV), None, _i32([tok]), seq1)
    torch.cuda.synchronize()
    g = buf1.logits[0].cpu().numpy()
    lscale = _scale(ref["logits"])
    err = np.abs(g - ref["logits"]).max()
    print(f"AR step, 2 layers: logits err/scale {err / lscale:.3e}")
    assert err <= tol * lscale
    check_argmax_near_tie(buf1.node_argmax[0].cpu().numpy(), g, ref["logits"], tol * lscale)
    assert int(buf1.accept_len[0]) == 1 and int(seq1[0]) == S + 1
    for l in range(2):
        k, v = kv1.read(l, 0, S, 1)
        assert np.abs(U.to_np(k) - kc[l][:, S:S + 1]).max() <= tol * _scale(kc[l][:, S:S + 1])
        assert np.abs(U.to_np(v) - vc[l][:, S:S + 1]).max() <= tol * _scale(vc[l][:, S:S + 1])
    del dm1, kv1

    dm64 = G.device_model(w64, heads=False)
    kv64 = G.device_kv_random_prefix(dm64, w64, cap=S + 64)
    buf64 = P.StepBuffers(dm64, 1, S, want_logits=True)
    tokens = W.random_tokens(w64, "ar_vs_tree_tokens", (64,)).to(torch.int32)
    tokens[0] = tok
    buf64.tree_tokens.copy_(tokens.view(1, 64).to(G.DEV))
    P.run_step(dm64, kv64, buf64, None, None, None, _i32([S]), with_heads=False)
    torch.cuda.synchronize()
    root_logits = buf64.logits[0, 0].cpu().numpy()
    assert np.abs(root_logits - g[0]).max() <= 2 * tol * lscale        # two bf16 kernel families, same mathematics
