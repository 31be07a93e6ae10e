"""Pins for oracle/medusa.py: the tree pass, the decoder maths, heads, compaction (CPU only).

The paper fixes that verification happens in one pass over all T candidates under the static
visibility matrix while the frozen backbone's outputs are unchanged (Sections 3.1, 3.2): hence a
node's logits must equal ordinary causal decoding along its root-to-node path.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workload as W
from oracle import medusa as O
from oracle import tree as OT
from tests import util as U

TINY = W.CONFIGS["cfg1_tiny_fp32"]


@pytest.fixture(scope="module")
def tiny():
    w = TINY
    model = U.oracle_model(w)
    tree = U.oracle_tree(w)
    cap = 160
    kc, vc = O.empty_cache(model["cfg"], cap)
    prefix_tokens = W.random_tokens(w, "prefix", (w.prefix[0],)).numpy()
    O.causal_decode(prefix_tokens, model, kc, vc, 0)          # config 1: prefix cache by causal prefill
    return dict(w=w, model=model, tree=tree, kc=kc, vc=vc, S=w.prefix[0], prefix_tokens=prefix_tokens)


# ---------------------------------------------------------------- P1: tree == causal

@pytest.mark.parametrize("spec", [W.TREE15, W.TreeSpec("tree7", (2, 2), (2, 4), 7, 4)], ids=lambda s: s.name)
def test_tree_pass_equals_causal_decoding_along_each_path(tiny, spec):
    model, S = tiny["model"], tiny["S"]
    tree = OT.build_tree(spec.caps, spec.budgets)
    T = tree["T"]
    tokens = W.random_tokens(TINY, f"treetok.{spec.name}", (T,)).numpy()
    kc, vc = U.copy_cache(tiny["kc"]), U.copy_cache(tiny["vc"])
    out = O.tree_verify_step(tokens, model, kc, vc, S, tree)
    scale = np.abs(out["logits"]).max()
    for n in range(T):
        chain = U.path_to(tree, n)
        kc2, vc2 = U.copy_cache(tiny["kc"]), U.copy_cache(tiny["vc"])
        logits, hidden = O.causal_decode(tokens[chain], model, kc2, vc2, S)
        assert np.abs(logits[-1] - out["logits"][n]).max() <= 1e-7 * scale     # fp32 cache rounding only
        assert np.abs(hidden[-1] - out["hidden"][n]).max() <= 1e-7 * np.abs(out["hidden"]).max()
        # the KV rows the tree pass wrote at slot S+n are the rows causal decoding wrote at S+depth
        for l in range(len(kc)):
            np.testing.assert_allclose(kc[l][:, S + n], kc2[l][:, S + len(chain) - 1], rtol=0, atol=1e-6)
            np.testing.assert_allclose(vc[l][:, S + n], vc2[l][:, S + len(chain) - 1], rtol=0, atol=1e-6)


def test_tree_pass_equals_causal_exactly_without_cache_rounding(tiny):
    """Same invariant with the cache kept in float64: agreement to 1e-9 relative."""
    w = TINY
    model = dict(tiny["model"], cfg=dict(tiny["model"]["cfg"], dtype="fp64"))
    tree = tiny["tree"]
    S = 5
    kc, vc = O.empty_cache(model["cfg"], 40)
    O.causal_decode(tiny["prefix_tokens"][:S], model, kc, vc, 0)
    tokens = W.random_tokens(w, "treetok.exact", (tree["T"],)).numpy()
    k1, v1 = U.copy_cache(kc), U.copy_cache(vc)
    out = O.tree_verify_step(tokens, model, k1, v1, S, tree)
    scale = np.abs(out["logits"]).max()
    for n in range(tree["T"]):
        k2, v2 = U.copy_cache(kc), U.copy_cache(vc)
        logits, _ = O.causal_decode(tokens[U.path_to(tree, n)], model, k2, v2, S)
        assert np.abs(logits[-1] - out["logits"][n]).max() <= 1e-9 * scale


def test_empty_prefix_and_sibling_relabelling(tiny):
    """S = 0 works (a node sees only its ancestors), and swapping two sibling subtrees' tokens
    swaps their logits and leaves every other node unchanged (P6)."""
    model, tree = tiny["model"], tiny["tree"]
    tokens = W.random_tokens(TINY, "treetok.perm", (tree["T"],)).numpy()
    kc, vc = O.empty_cache(model["cfg"], 16)
    a = O.tree_verify_step(tokens, model, kc, vc, 0, tree)
    row_sums_ok = np.isfinite(a["logits"]).all()
    assert row_sums_ok
    # swap the two depth-1 subtrees of tree15: nodes 1<->2, 3,4<->5,6, 7..10<->11..14
    perm = np.array([0, 2, 1, 5, 6, 3, 4, 11, 12, 13, 14, 7, 8, 9, 10])
    kc2, vc2 = O.empty_cache(model["cfg"], 16)
    b = O.tree_verify_step(tokens[perm], model, kc2, vc2, 0, tree)
    np.testing.assert_allclose(b["logits"], a["logits"][perm], rtol=0, atol=1e-9 * np.abs(a["logits"]).max())


# ---------------------------------------------------------------- P5: the decoder maths vs library ops

def _torch_layer_reference(x, lw, kpre, vpre, S, cfg):
    """A chain of n tokens after a prefix of S rows, written with PyTorch CPU library ops in float64.
    RoPE via complex multiplication (a different formulation from the oracle's real-pair form)."""
    H, hd = cfg["n_heads"], cfg["head_dim"]
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    x = t(x)
    n = x.shape[0]
    xn = F.rms_norm(x, (x.shape[1],), weight=t(lw["g_attn"]), eps=cfg["rms_eps"])
    q = F.linear(xn, t(lw["wq"])).view(n, H, hd).transpose(0, 1)
    k = F.linear(xn, t(lw["wk"])).view(n, H, hd).transpose(0, 1)
    v = F.linear(xn, t(lw["wv"])).view(n, H, hd).transpose(0, 1)

    def rope_c(a):
        half = hd // 2
        z = torch.complex(a[..., :half], a[..., half:])
        pos = torch.arange(S, S + n, dtype=torch.float64)
        theta = pos[:, None] * (cfg["rope_base"] ** (-torch.arange(half, dtype=torch.float64) * 2 / hd))[None, :]
        z = z * torch.polar(torch.ones_like(theta), theta)
        return torch.cat([z.real, z.imag], dim=-1)

    q, k = rope_c(q), rope_c(k)
    kk = torch.cat([t(kpre), k], dim=1)
    vv = torch.cat([t(vpre), v], dim=1)
    allow = torch.ones(n, S + n, dtype=torch.bool).tril(diagonal=S)          # causal with S prefix rows
    att = F.scaled_dot_product_attention(q, kk, vv, attn_mask=allow)
    att = att.transpose(0, 1).reshape(n, H * hd)
    x = x + F.linear(att, t(lw["wo"]))
    xn = F.rms_norm(x, (x.shape[1],), weight=t(lw["g_ffn"]), eps=cfg["rms_eps"])
    x = x + F.linear(F.silu(F.linear(xn, t(lw["wgate"]))) * F.linear(xn, t(lw["wup"])), t(lw["wdown"]))
    return x.numpy(), k.numpy(), v.numpy()


@pytest.mark.parametrize("S", [0, 9])
def test_chain_tree_layer_matches_torch_library_ops(S):
    """A chain-shaped tree (one child per node) is ordinary causal attention: compare one oracle layer
    against scaled_dot_product_attention / rms_norm / silu / linear on the CPU in float64."""
    w = TINY
    cfg = U.oracle_cfg(w, dtype="fp64")
    lw = U.oracle_layer(w, 0)
    lw["g_attn"] = W.normal(7, "gain_a", (w.d,), 0.3).numpy() + 1.0          # non-trivial gains
    lw["g_ffn"] = W.normal(7, "gain_f", (w.d,), 0.3).numpy() + 1.0
    chain = OT.build_tree((1, 1, 1, 1, 1), (1, 1, 1, 1, 1))
    assert chain["T"] == 6 and np.array_equal(chain["mask"], np.tril(np.ones((6, 6), dtype=bool)))
    x = W.hidden_state(w, "chain_x", 6).numpy()
    kpre = W.normal(3, "kpre", (w.n_heads, S, w.head_dim)).numpy()
    vpre = W.normal(3, "vpre", (w.n_heads, S, w.head_dim)).numpy()
    kc = np.zeros((w.n_heads, S + 6, w.head_dim)); kc[:, :S] = kpre
    vc = np.zeros((w.n_heads, S + 6, w.head_dim)); vc[:, :S] = vpre
    got = O.tree_verify_layer(x, lw, kc, vc, S, chain, cfg)
    ref, kref, vref = _torch_layer_reference(x, lw, kpre, vpre, S, cfg)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-11 * np.abs(ref).max())
    np.testing.assert_allclose(kc[:, S:], kref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(vc[:, S:], vref, rtol=0, atol=1e-12)


def test_chain_tree_whole_step_matches_torch_library_ops_end_to_end():
    """Embedding -> every layer -> final norm -> LM head -> argmax of a chain-shaped tree (ordinary causal decoding
    of 6 tokens after a prefix) against PyTorch CPU library ops in float64, with non-unit gains everywhere
    (final norm included) and an LM head that is a different tensor from the embedding."""
    w = TINY
    S = 9
    model = U.oracle_model(w, dtype="fp64")
    assert all(np.abs(lw[g] - 1.0).max() > 0.3 for lw in model["layers"] for g in ("g_attn", "g_ffn"))
    assert np.abs(model["g_final"] - 1.0).max() > 0.3 and not np.array_equal(model["lm_head"], model["embed"])
    chain = OT.build_tree((1, 1, 1, 1, 1), (1, 1, 1, 1, 1))
    T = chain["T"]
    tokens = W.random_tokens(w, "chain_step_tok", (T,)).numpy()
    kpre = [W.normal(3, f"kpre{l}", (w.n_heads, S, w.head_dim)).numpy() for l in range(w.n_layers)]
    vpre = [W.normal(3, f"vpre{l}", (w.n_heads, S, w.head_dim)).numpy() for l in range(w.n_layers)]
    kc, vc = O.empty_cache(model["cfg"], S + T)
    for l in range(w.n_layers):
        kc[l][:, :S] = kpre[l]
        vc[l][:, :S] = vpre[l]
    got = O.tree_verify_step(tokens, model, kc, vc, S, chain)
    # library-op reference
    x = F.embedding(torch.tensor(tokens, dtype=torch.long), torch.tensor(model["embed"], dtype=torch.float64)).numpy()
    for l in range(w.n_layers):
        x, kref, vref = _torch_layer_reference(x, model["layers"][l], kpre[l], vpre[l], S, model["cfg"])
        np.testing.assert_allclose(kc[l][:, S:], kref, rtol=0, atol=1e-11)
        np.testing.assert_allclose(vc[l][:, S:], vref, rtol=0, atol=1e-11)
    xt = torch.tensor(x)
    hidden = F.rms_norm(xt, (w.d,), weight=torch.tensor(model["g_final"], dtype=torch.float64), eps=w.rms_eps)
    logits = F.linear(hidden, torch.tensor(model["lm_head"], dtype=torch.float64))
    np.testing.assert_allclose(got["hidden"], hidden.numpy(), rtol=0, atol=1e-11 * float(hidden.abs().max()))
    np.testing.assert_allclose(got["logits"], logits.numpy(), rtol=0, atol=1e-11 * float(logits.abs().max()))
    assert got["node_argmax"].tolist() == torch.argmax(logits, dim=1).tolist()
    # the hidden the step returns is what the Medusa heads read: its base-head logits are the step's logits
    heads = O.medusa_heads(got["hidden"][2], model, U.oracle_tree(w))
    np.testing.assert_allclose(heads["head_logits"][0], logits[2].numpy(), rtol=0, atol=1e-11 * float(logits.abs().max()))


def test_heads_with_bias_against_torch_ops(tiny):
    """The optional bias of a head's residual block enters before the SiLU."""
    w = TINY.with_(head_bias_std=1.0)
    model, tree = U.oracle_model(w), tiny["tree"]
    assert all(hd["b1"] is not None and np.abs(hd["b1"]).max() > 1.0 for hd in model["medusa"])
    h = W.hidden_state(w, "heads_hb", 1).numpy()[0]
    out = O.medusa_heads(h, model, tree)
    ht = torch.tensor(h, dtype=torch.float64)
    for k, hd in enumerate(model["medusa"]):
        z = ht + F.silu(F.linear(ht, torch.tensor(hd["w1"], dtype=torch.float64), torch.tensor(hd["b1"], dtype=torch.float64)))
        lg = F.linear(z, torch.tensor(hd["lm"], dtype=torch.float64))
        np.testing.assert_allclose(out["head_logits"][k + 1], lg.numpy(), rtol=1e-12, atol=1e-12)


def test_rope_properties():
    hd = 64
    q = W.normal(1, "rq", (3, hd)).numpy().astype(np.float64)
    k = W.normal(1, "rk", (3, hd)).numpy().astype(np.float64)
    # position 0 is the identity; norms are preserved; <R_m q, R_n k> depends on m - n only
    np.testing.assert_allclose(O.rope(q, np.zeros(3), 1e4), q, atol=1e-15)
    np.testing.assert_allclose(np.linalg.norm(O.rope(q, np.array([5, 77, 1000]), 1e4), axis=1),
                               np.linalg.norm(q, axis=1), rtol=1e-13)
    a = (O.rope(q, np.array([10, 10, 10]), 1e4) * O.rope(k, np.array([7, 7, 7]), 1e4)).sum(1)
    b = (O.rope(q, np.array([103, 103, 103]), 1e4) * O.rope(k, np.array([100, 100, 100]), 1e4)).sum(1)
    np.testing.assert_allclose(a, b, rtol=1e-10)
    # first pair (i = 0) rotates by exactly pos radians; last pair by pos * base**(-(hd-2)/hd)
    e = np.zeros((1, hd)); e[0, 0] = 1.0
    r = O.rope(e, np.array([2.0]), 1e4)
    np.testing.assert_allclose([r[0, 0], r[0, hd // 2]], [np.cos(2.0), np.sin(2.0)], atol=1e-15)
    e = np.zeros((1, hd)); e[0, hd // 2 - 1] = 1.0
    r = O.rope(e, np.array([3.0]), 1e4)
    th = 3.0 * 1e4 ** (-(hd - 2) / hd)
    np.testing.assert_allclose([r[0, hd // 2 - 1], r[0, hd - 1]], [np.cos(th), np.sin(th)], atol=1e-15)


def test_round_to_storage_matches_torch_casts():
    x = np.concatenate([W.normal(5, "rnd", (20000,)).numpy().astype(np.float64) * s
                        for s in (1e-3, 1.0, 300.0)])
    x = np.concatenate([x, [0.0, 1.0, -1.0, 1.00390625, 1.01171875, 255.5, 3.3895313892515355e38 / 2]])
    t = torch.tensor(x)
    np.testing.assert_array_equal(O.round_to_storage(x, "bf16"), t.to(torch.bfloat16).to(torch.float64).numpy())
    np.testing.assert_array_equal(O.round_to_storage(x, "fp32"), t.to(torch.float32).to(torch.float64).numpy())
    # exact ties go to even: 1 + 2^-8 -> 1.0 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert O.round_to_storage(np.array([1.00390625, 1.01171875]), "bf16").tolist() == [1.0, 1.015625]


def test_round_to_fp16_binary16_grid_ties_subnormals_and_torch_cast():
    """fp16 (the paper's precision, Section 4.1): the result lies on the binary16 grid (11 significant bits above
    2^-14, multiples of 2^-24 below), is a nearest grid point, ties go to even; cross-checked with torch's cast."""
    x = np.concatenate([W.normal(6, "rnd16", (20000,)).numpy().astype(np.float64) * s for s in (1e-6, 1e-3, 1.0, 300.0)])
    r = O.round_to_storage(x, "fp16")
    np.testing.assert_array_equal(r, torch.tensor(x).to(torch.float16).to(torch.float64).numpy())
    # grid spacing at |x|: 2^(floor(log2|x|) - 10), at least 2^-24; the rounded value is a multiple of it within half a step
    e = np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** -14)))
    step = 2.0 ** (e - 10)
    assert np.all(np.abs(r - x) <= step / 2) and np.all(r / step == np.rint(r / step))
    # ties to even: 1 + 2^-11 -> 1 ; 1 + 3*2^-11 -> 1 + 2^-9 ; 2^-25 -> 0 ; 3*2^-25 -> 2^-23
    t = np.array([1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 2.0 ** -25, 3 * 2.0 ** -25, 65504.0, -2049.0])
    assert O.round_to_storage(t, "fp16").tolist() == [1.0, 1 + 2.0 ** -9, 0.0, 2.0 ** -23, 65504.0, -2048.0]


# ---------------------------------------------------------------- Medusa heads (O-2)

def test_heads_reduce_to_lm_head_when_w1_is_zero(tiny):
    model, tree = tiny["model"], tiny["tree"]
    h = W.hidden_state(TINY, "heads_h", 1).numpy()[0]
    m0 = dict(model, medusa=[dict(w1=np.zeros_like(hd["w1"]), b1=None, lm=hd["lm"]) for hd in model["medusa"]])
    out = O.medusa_heads(h, m0, tree)
    for k, hd in enumerate(model["medusa"]):
        np.testing.assert_allclose(out["head_logits"][k + 1], hd["lm"].astype(np.float64) @ h, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(out["head_logits"][0], model["lm_head"].astype(np.float64) @ h, rtol=1e-13, atol=1e-13)


def test_heads_against_torch_ops_and_full_sort(tiny):
    model, tree = tiny["model"], tiny["tree"]
    h = W.hidden_state(TINY, "heads_h2", 1).numpy()[0]
    out = O.medusa_heads(h, model, tree)
    ht = torch.tensor(h, dtype=torch.float64)
    flat = [int(torch.argmax(F.linear(ht, torch.tensor(model["lm_head"], dtype=torch.float64))))]
    for k, hd in enumerate(model["medusa"]):
        z = ht + F.silu(F.linear(ht, torch.tensor(hd["w1"], dtype=torch.float64)))
        lg = F.linear(z, torch.tensor(hd["lm"], dtype=torch.float64))
        np.testing.assert_allclose(out["head_logits"][k + 1], lg.numpy(), rtol=1e-12, atol=1e-12)
        srt = sorted(range(lg.numel()), key=lambda i: (-float(lg[i]), i))       # full sort, ties -> lower id
        flat += srt[:tree["caps"][k]]
    assert out["cand_flat"].tolist() == flat
    assert out["tree_tokens"].tolist() == [flat[s] for s in tree["cand_slot"]]
    assert out["tree_tokens"][0] == flat[0]


def test_topk_and_argmax_tie_break():
    a = np.array([1.0, 3.0, 3.0, 2.0, 3.0, -1.0])
    assert O.topk_lowest(a, 4).tolist() == [1, 2, 4, 3]
    assert O.argmax_lowest(a[None])[0] == 1
    b = np.array([0.5, 0.5, 0.5])
    assert O.topk_lowest(b, 2).tolist() == [0, 1]


# ---------------------------------------------------------------- P4: compaction and chaining

@pytest.mark.parametrize("m", [0, 1, 2, 3])
def test_planted_path_accept_compact_equals_causal_cache(tiny, m):
    """Plant the model's own greedy continuation g_1..g_m on a tree path: acceptance must return m+1
    tokens and, after compaction, the cache must be the one causal decoding of those tokens writes.
    A second chained step then agrees with causal decoding of everything accepted so far."""
    model, tree, S = tiny["model"], tiny["tree"], tiny["S"]
    K, T = tree["K"], tree["T"]
    # greedy continuation from the prefix: root = argmax after last prefix token
    kc, vc = O.empty_cache(model["cfg"], 160)
    lg, _ = O.causal_decode(tiny["prefix_tokens"], model, kc, vc, 0)
    greedy = [int(np.argmax(lg[-1]))]
    kg, vg = U.copy_cache(kc), U.copy_cache(vc)
    for i in range(K + 1):
        lg1, _ = O.causal_decode([greedy[-1]], model, kg, vg, S + i)
        greedy.append(int(np.argmax(lg1[-1])))
    # choose the path through the LAST child at each depth (node indices far from 0..m)
    path = [0]
    for d in range(K):
        path.append(max(n for n in range(T) if tree["parent"][n] == path[-1]))
    tokens = np.full(T, -7, dtype=np.int64)
    filler = (np.arange(T) * 37 + 11) % TINY.vocab
    for n in range(T):
        tokens[n] = filler[n]
    tokens[0] = greedy[0]
    for d in range(1, m + 1):
        tokens[path[d]] = greedy[d]
    # make sure no other node accidentally matches its parent's greedy prediction
    k1, v1 = U.copy_cache(kc), U.copy_cache(vc)
    out = O.tree_verify_step(tokens, model, k1, v1, S, tree)
    for n in range(1, T):
        if n not in path[:m + 1] and tokens[n] == out["node_argmax"][tree["parent"][n]]:
            tokens[n] = (tokens[n] + 1) % TINY.vocab
    k1, v1 = U.copy_cache(kc), U.copy_cache(vc)
    out = O.tree_verify_step(tokens, model, k1, v1, S, tree)
    acc = O.accept_longest_prefix(tree, tokens, out["node_argmax"])
    assert acc["accept_len"] == m + 1
    assert acc["acc_nodes"][:m + 1].tolist() == path[:m + 1]
    assert acc["acc_tokens"][:m + 1].tolist() == greedy[:m + 1]
    assert acc["next_root"] == greedy[m + 1] and acc["last_node"] == path[m]
    before = U.copy_cache(k1)
    src, S2 = O.kv_compact(k1, v1, S, acc["acc_nodes"], acc["accept_len"])
    assert S2 == S + m + 1
    assert src[:m + 1].tolist() == [S + n for n in path[:m + 1]] and (src[m + 1:] == -1).all()
    for l in range(len(k1)):
        for j in range(m + 1):
            assert np.array_equal(k1[l][:, S + j], before[l][:, S + path[j]])       # bit-for-bit moved rows
        assert np.array_equal(k1[l][:, :S], kc[l][:, :S])                              # prefix untouched
    # cache == causal decoding of the accepted tokens
    k2, v2 = U.copy_cache(kc), U.copy_cache(vc)
    O.causal_decode(greedy[:m + 1], model, k2, v2, S)
    for l in range(len(k1)):
        np.testing.assert_allclose(k1[l][:, :S2], k2[l][:, :S2], rtol=0, atol=1e-6)
        np.testing.assert_allclose(v1[l][:, :S2], v2[l][:, :S2], rtol=0, atol=1e-6)
    # chained second step from the compacted cache == causal decoding from the causal cache
    tokens2 = W.random_tokens(TINY, f"treetok.chain{m}", (T,)).numpy()
    tokens2[0] = acc["next_root"]
    o1 = O.tree_verify_step(tokens2, model, k1, v1, S2, tree)
    o2 = O.tree_verify_step(tokens2, model, k2, v2, S2, tree)
    np.testing.assert_allclose(o1["logits"], o2["logits"], rtol=0, atol=2e-6 * np.abs(o2["logits"]).max())
