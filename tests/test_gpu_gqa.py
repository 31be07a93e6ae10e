"""GPU parity with grouped-query attention (Table 1 of the paper: 32 query heads, 8 key/value heads): the same
entry points and kernels with n_kv_heads < n_heads, against the oracle."""
import numpy as np
import pytest
import torch

import workload as W
import paper_2603_03383_amd as P
from oracle import medusa as O
from tests import gpu_util as G
from tests import util as U
from tests.test_gpu_parity import TOL, _i32, _scale, check_argmax_near_tie, _layer_case, _check_layer

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("spec", [W.TREE15, W.TREE64K5], ids=lambda s: s.name)
def test_tiny_fp32_grouped_heads_full_path(spec):
    """Also the five-head tree (Table 2 trains five heads): heads, verification, acceptance up to depth 5, compaction."""
    w = W.CONFIGS["cfg1_tiny_fp32"].with_(name="tiny_gqa", n_kv_heads=2, tree=spec)
    S = w.prefix[0]
    tol = TOL["fp32"]
    model = U.oracle_model(w)
    tree = U.oracle_tree(w)
    T = tree["T"]
    prefix_tokens = W.random_tokens(w, "prefix", (S,)).numpy()
    kc, vc = O.empty_cache(model["cfg"], S + T)
    lg, hid = O.causal_decode(prefix_tokens, model, kc, vc, 0)
    h = hid[-1].astype(np.float32)
    heads = O.medusa_heads(h, model, tree)
    kc_o, vc_o = U.copy_cache(kc), U.copy_cache(vc)
    ref = O.tree_verify_step(heads["tree_tokens"], model, kc_o, vc_o, S, tree)
    acc = O.accept_longest_prefix(tree, heads["tree_tokens"], ref["node_argmax"])

    dm = G.device_model(w)
    kv = G.device_kv_from_oracle(dm, [kc], [vc], [S], cap=S + T)
    assert kv.desc.n_heads == 2
    buf = P.StepBuffers(dm, 1, S, want_logits=True)
    seq_len = _i32([S])
    P.run_step(dm, kv, buf, torch.tensor(h, device=G.DEV).view(1, 1, -1), None, None, seq_len)
    torch.cuda.synchronize()
    assert buf.tree_tokens[0].cpu().numpy().tolist() == heads["tree_tokens"].tolist()
    g = buf.logits[0].cpu().numpy()
    assert np.abs(g - ref["logits"]).max() <= tol * _scale(ref["logits"])
    assert check_argmax_near_tie(buf.node_argmax[0].cpu().numpy(), g, ref["logits"], tol * _scale(ref["logits"])) == 0
    assert int(buf.accept_len[0]) == acc["accept_len"] and buf.acc_nodes[0].cpu().numpy().tolist() == acc["acc_nodes"].tolist()
    src, S2 = O.kv_compact(kc_o, vc_o, S, acc["acc_nodes"], acc["accept_len"])
    assert int(seq_len[0]) == S2
    for l in range(w.n_layers):
        k, v = kv.read(l, 0, 0, S2)
        assert k.shape[0] == 2
        np.testing.assert_allclose(k.cpu().numpy(), kc_o[l][:, :S2], rtol=0, atol=2e-5)
        np.testing.assert_allclose(v.cpu().numpy(), vc_o[l][:, :S2], rtol=0, atol=2e-5)


@pytest.mark.parametrize("S_list,max_prefix", [([0], 0), ([77], 100), ([1024], 1024), ([300, 0, 45], 300), ([5000], 5003)])
def test_7b_width_layer_32_query_8_kv_heads(S_list, max_prefix):
    """The MFMA path (fused reduce + RoPE + KV write in the attention prologue) with four query heads per KV head."""
    w = W.CONFIGS["cfg2_layer_bf16"].with_(name="layer_gqa", n_kv_heads=8, prefix=tuple(S_list))
    r = _layer_case(w, S_list, max_prefix, x_seed="gqa_layer_x")
    rel = _check_layer(r, S_list, "bf16")
    print(f"GQA layer {S_list}: err/scale {rel:.3e}")


@pytest.mark.parametrize("S_list,max_prefix", [([0, 33, 1000], 1000), ([4097], 4100)])
def test_7b_width_autoregressive_layer_grouped_heads(S_list, max_prefix):
    w = W.CONFIGS["cfg2_layer_bf16"].with_(name="ar_layer_gqa", n_kv_heads=8, tree=W.TREE1, prefix=tuple(S_list))
    r = _layer_case(w, S_list, max_prefix, x_seed="gqa_ar_x")
    rel = _check_layer(r, S_list, "bf16")
    print(f"GQA AR layer {S_list}: err/scale {rel:.3e}")


def test_two_layer_step_grouped_heads_bf16():
    two_layer_step_case(W.CONFIGS["cfg3_step_1k"].with_(name="step_gqa", n_layers=2, n_kv_heads=8))


def two_layer_step_case(w):
    S = w.prefix[0]
    tol = TOL[w.dtype]
    tree = U.oracle_tree(w)
    T = tree["T"]
    model = U.oracle_model(w, device=G.DEV, heads=False)
    dm = G.device_model(w, heads=False)
    kc, vc = U.oracle_prefix_cache(w, 0, S + T, device=G.DEV)
    kv = G.device_kv_random_prefix(dm, w, cap=S + T)
    tokens = W.random_tokens(w, "gqa_tree_tokens", (T,)).to(torch.int32)
    buf = P.StepBuffers(dm, 1, S, want_logits=True)
    buf.tree_tokens.copy_(tokens.view(1, T).to(G.DEV))
    seq_len = _i32([S])
    P.run_step(dm, kv, buf, None, None, None, seq_len, with_heads=False)
    torch.cuda.synchronize()
    ref = O.tree_verify_step(tokens.numpy(), model, kc, vc, S, tree)
    g = buf.logits[0].cpu().numpy()
    lscale = _scale(ref["logits"])
    err = np.abs(g - ref["logits"]).max()
    print(f"{w.name} ({w.dtype}), 2 layers: logits err/scale {err / lscale:.3e}")
    assert err <= tol * lscale
    gpu_am = buf.node_argmax[0].cpu().numpy()
    check_argmax_near_tie(gpu_am, g, ref["logits"], tol * lscale)
    acc = O.accept_longest_prefix(tree, tokens.numpy(), gpu_am)
    assert int(buf.accept_len[0]) == acc["accept_len"] and int(seq_len[0]) == S + acc["accept_len"]


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_paper_shape_one_layer_step_with_heads_vocab_153600(dtype):
    """The paper's shape (Table 1: grouped heads, vocabulary ~153k; five heads; fp16 as in Section 4.1, and bf16) at
    one layer: the selection kernels run with more column chunks than at 128000, the LM-head GEMMs with 4800 tiles."""
    from tests.test_gpu_parity import check_topk_near_tie
    w = W.CONFIGS["next3_paper_shape_1k"].with_(n_layers=1, prefix=(200,), dtype=dtype)
    S = w.prefix[0]
    tol = TOL[dtype]
    tree = U.oracle_tree(w)
    T, K = tree["T"], tree["K"]
    model = U.oracle_model(w, device=G.DEV)
    dm = G.device_model(w)
    kc, vc = U.oracle_prefix_cache(w, 0, S + T, device=G.DEV)
    kv = G.device_kv_random_prefix(dm, w, cap=S + T)
    h = W.hidden_state(w, "heads_in", 1, device=G.DEV)
    heads = O.medusa_heads(U.to_np(h)[0], model, tree)
    buf = P.StepBuffers(dm, 1, S, want_logits=True, want_head_logits=True)
    seq_len = _i32([S])
    P.run_step(dm, kv, buf, h.view(1, 1, -1), None, None, seq_len)
    torch.cuda.synchronize()
    hl = buf.head_logits[0].cpu().numpy()
    hscale = _scale(heads["head_logits"])
    assert np.abs(hl - heads["head_logits"]).max() <= tol * hscale
    cand = buf.cand_flat[0].cpu().numpy()
    check_argmax_near_tie(cand[:1], hl[:1], heads["head_logits"][:1], tol * hscale)
    off = 1
    for k in range(K):
        c = tree["caps"][k]
        check_topk_near_tie(cand[off:off + c], hl[k + 1], heads["head_logits"][k + 1], c, tol * hscale)
        off += c
    gpu_tokens = buf.tree_tokens[0].cpu().numpy()
    assert gpu_tokens.tolist() == cand[tree["cand_slot"]].tolist()
    ref = O.tree_verify_step(gpu_tokens, model, kc, vc, S, tree)
    g = buf.logits[0].cpu().numpy()
    lscale = _scale(ref["logits"])
    assert np.abs(g - ref["logits"]).max() <= tol * lscale
    check_argmax_near_tie(buf.node_argmax[0].cpu().numpy(), g, ref["logits"], tol * lscale)
    print(f"paper shape, one layer, {dtype}: head logits err/scale {np.abs(hl - heads['head_logits']).max() / hscale:.3e}, "
          f"logits err/scale {np.abs(g - ref['logits']).max() / lscale:.3e}")
