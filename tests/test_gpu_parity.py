"""GPU parity: the HIP path, called through the C-ABI binding, against the CPU oracle on identical
seeded inputs.  Bit-exact for ids / lengths / indices, tolerance on floating point:
  fp32 storage: 1e-5 x max(1, max|oracle logits|);  bf16 storage: 2e-2 x the same scale.
Near-tie rule for ids derived from floating point: the argmax / top-k kernels are checked bit-exactly
against the oracle's selection applied to the GPU's own logits; against the oracle's logits they must
agree wherever the oracle's deciding gap exceeds twice the tolerance.
"""
import numpy as np
import pytest
import torch

import workload as W
import paper_2603_03383_amd as P
from oracle import medusa as O
from tests import gpu_util as G
from tests import util as U

pytestmark = pytest.mark.gpu

# bf16 and fp32: the stated bounds.  fp16 (the paper's own precision, Section 4.1) has no stated bound: it carries 3 more
# significant bits than bf16 through the same roundings (activations between kernels, K/V in the cache, softmax
# probabilities), so its bound is the bf16 one scaled by 2^-3.
TOL = {"fp32": 1e-5, "bf16": 2e-2, "fp16": 2e-2 / 8}


def _scale(a):
    return max(1.0, float(np.abs(a).max()))


def _i32(a, dev=G.DEV):
    return torch.tensor(np.asarray(a), dtype=torch.int32, device=dev)


def check_argmax_near_tie(gpu_ids, gpu_logits, ref_logits, tol_abs):
    """gpu_ids [R]; logits [R,V]."""
    assert np.array_equal(gpu_ids, O.argmax_lowest(gpu_logits.astype(np.float64))), "argmax kernel != argmax of its own logits"
    ref_ids = O.argmax_lowest(ref_logits)
    part = np.partition(ref_logits, -2, axis=1)
    gap = part[:, -1] - part[:, -2]
    decided = gap > 2 * tol_abs
    assert np.array_equal(gpu_ids[decided], ref_ids[decided])
    for r in np.nonzero(~decided)[0]:                                  # near ties: must pick one of the tied leaders
        assert ref_logits[r, gpu_ids[r]] >= part[r, -1] - 2 * tol_abs
    return int((~decided).sum())


def check_topk_near_tie(gpu_ids, gpu_logits, ref_logits, k, tol_abs):
    assert gpu_ids.tolist() == O.topk_lowest(gpu_logits.astype(np.float64), k).tolist()
    ref_ids = O.topk_lowest(ref_logits, k)
    srt = np.sort(ref_logits)[::-1]
    gaps = srt[:k] - srt[1:k + 1]
    if (gaps > 2 * tol_abs).all():
        assert gpu_ids.tolist() == ref_ids.tolist()
        return 0
    assert all(ref_logits[i] >= srt[k - 1] - 2 * tol_abs for i in gpu_ids)
    return 1


# ------------------------------------------------------------------------------------------------
# config 1: tiny fp32 model, 15-node tree, causal-prefill prefix of 64 tokens — the whole path
# ------------------------------------------------------------------------------------------------

def _cfg1_case(w):
    S = w.prefix[0]
    model = U.oracle_model(w)
    tree = U.oracle_tree(w)
    prefix_tokens = W.random_tokens(w, "prefix", (S,)).numpy()
    kc, vc = O.empty_cache(model["cfg"], S + 2 * tree["T"])
    lg, hid = O.causal_decode(prefix_tokens, model, kc, vc, 0)
    dm = G.device_model(w)
    return dict(w=w, S=S, model=model, tree=tree, kc=kc, vc=vc, dm=dm, last_hidden=hid[-1], last_logits=lg[-1])


@pytest.fixture(scope="module")
def cfg1():
    """Config 1 with a bias in every Medusa head (the ABI's optional b1), so that input is exercised too."""
    return _cfg1_case(W.CONFIGS["cfg1_tiny_fp32"].with_(head_bias_std=1.0))


@pytest.fixture(scope="module")
def cfg1_k5():
    """The tiny model under the 64-node tree with five heads (Table 2 trains five heads)."""
    return _cfg1_case(W.CONFIGS["cfg1_tiny_fp32"].with_(name="tiny_k5", tree=W.TREE64K5))


def test_cfg1_heads_verify_accept_compact(cfg1):
    w, S, model, tree, dm = cfg1["w"], cfg1["S"], cfg1["model"], cfg1["tree"], cfg1["dm"]
    T, K = tree["T"], tree["K"]
    tol = TOL["fp32"]
    h = cfg1["last_hidden"].astype(np.float32)                         # hidden after the last prefix token
    heads = O.medusa_heads(h, model, tree)
    kc, vc = U.copy_cache(cfg1["kc"]), U.copy_cache(cfg1["vc"])
    ref = O.tree_verify_step(heads["tree_tokens"], model, kc, vc, S, tree)
    acc = O.accept_longest_prefix(tree, heads["tree_tokens"], ref["node_argmax"])

    kv = G.device_kv_from_oracle(dm, [cfg1["kc"]], [cfg1["vc"]], [S], cap=S + T)
    buf = P.StepBuffers(dm, 1, S, want_logits=True, want_head_logits=True)
    seq_len = _i32([S])
    hid_in = torch.tensor(h, device=G.DEV).view(1, 1, -1)
    P.run_step(dm, kv, buf, hid_in, None, None, seq_len)
    torch.cuda.synchronize()

    # heads
    hl = buf.head_logits[0].cpu().numpy()
    assert np.abs(hl - heads["head_logits"]).max() <= tol * _scale(heads["head_logits"])
    assert buf.cand_flat[0].cpu().numpy().tolist() == heads["cand_flat"].tolist()
    assert buf.tree_tokens[0].cpu().numpy().tolist() == heads["tree_tokens"].tolist()
    # verify
    lg = buf.logits[0].cpu().numpy()
    assert np.abs(lg - ref["logits"]).max() <= tol * _scale(ref["logits"])
    assert np.abs(buf.hidden[0].cpu().numpy() - ref["hidden"]).max() <= tol * _scale(ref["hidden"])
    n_tie = check_argmax_near_tie(buf.node_argmax[0].cpu().numpy(), lg, ref["logits"], tol * _scale(ref["logits"]))
    assert n_tie == 0
    # accept + compact (bit exact)
    assert int(buf.accept_len[0]) == acc["accept_len"] and int(buf.best_path[0]) == acc["best_path"]
    assert buf.acc_nodes[0].cpu().numpy().tolist() == acc["acc_nodes"].tolist()
    assert buf.acc_tokens[0].cpu().numpy().tolist() == acc["acc_tokens"].tolist()
    assert int(buf.next_root[0]) == acc["next_root"] and int(buf.last_node[0]) == acc["last_node"]
    src, S2 = O.kv_compact(kc, vc, S, acc["acc_nodes"], acc["accept_len"])
    assert buf.kv_src_slots[0].cpu().numpy().tolist() == src.tolist() and int(seq_len[0]) == S2
    for l in range(w.n_layers):
        k, v = kv.read(l, 0, 0, S + T)
        np.testing.assert_allclose(k.cpu().numpy()[:, :S2], kc[l][:, :S2], rtol=0, atol=2e-5)
        np.testing.assert_allclose(v.cpu().numpy()[:, :S2], vc[l][:, :S2], rtol=0, atol=2e-5)


def test_cfg1_heads_with_separately_allocated_first_layers(cfg1, monkeypatch):
    """The heads' first-layer matrices may be separate allocations (one GEMM launch per head) or lie back to back (one
    launch for all, what DeviceModel arranges): both orders of work give the oracle's candidates and logits."""
    w, model, tree = cfg1["w"], cfg1["model"], cfg1["tree"]
    monkeypatch.setattr(P.DeviceModel, "_stack_head_w1", lambda self: None)
    dm = G.device_model(w)
    ptrs = [dm._w1[k] for k in range(tree["K"])]
    assert any(ptrs[k + 1] - ptrs[k] != P.medusa_packed_bytes(dm.dtype, w.d, w.d) for k in range(tree["K"] - 1))
    h = cfg1["last_hidden"].astype(np.float32)
    heads = O.medusa_heads(h, model, tree)
    buf = P.StepBuffers(dm, 1, cfg1["S"], want_head_logits=True)
    P.medusa_heads(dm.desc, dm.weights, torch.tensor(h, device=G.DEV).view(1, 1, -1), None, None, 1, 1, buf.cand_flat,
                   buf.tree_tokens, buf.head_logits, buf.ws)
    torch.cuda.synchronize()
    hl = buf.head_logits[0].cpu().numpy()
    assert np.abs(hl - heads["head_logits"]).max() <= TOL["fp32"] * _scale(heads["head_logits"])
    assert buf.cand_flat[0].cpu().numpy().tolist() == heads["cand_flat"].tolist()
    # and the stacked arrangement gives bit-identical logits
    buf2 = P.StepBuffers(cfg1["dm"], 1, cfg1["S"], want_head_logits=True)
    P.medusa_heads(cfg1["dm"].desc, cfg1["dm"].weights, torch.tensor(h, device=G.DEV).view(1, 1, -1), None, None, 1, 1,
                   buf2.cand_flat, buf2.tree_tokens, buf2.head_logits, buf2.ws)
    torch.cuda.synchronize()
    assert torch.equal(buf.head_logits, buf2.head_logits) and torch.equal(buf.cand_flat, buf2.cand_flat)


@pytest.mark.parametrize("m", [0, 1, 2, 3])
def test_cfg1_planted_acceptance_and_chained_step(cfg1, m):
    """Tree tokens carry the model's own greedy continuation along one path: A must be m+1, the compacted
    cache must equal the oracle's, and a second chained step must agree with the oracle's second step."""
    _planted_acceptance(cfg1, m)


@pytest.mark.parametrize("m", [0, 3, 4, 5])
def test_five_head_tree_planted_acceptance_up_to_six_tokens(cfg1_k5, m):
    _planted_acceptance(cfg1_k5, m)


def _planted_acceptance(cfg1, m):
    w, S, model, tree, dm = cfg1["w"], cfg1["S"], cfg1["model"], cfg1["tree"], cfg1["dm"]
    T, K = tree["T"], tree["K"]
    tol = TOL["fp32"]
    greedy = [int(np.argmax(cfg1["last_logits"]))]
    kg, vg = U.copy_cache(cfg1["kc"]), U.copy_cache(cfg1["vc"])
    for i in range(K + 1):
        lg1, _ = O.causal_decode([greedy[-1]], model, kg, vg, S + i)
        greedy.append(int(np.argmax(lg1[-1])))
    path = [int(n) for n in [r for r in tree["retrieve"] if r[K] >= 0][-1]]      # the last root-to-leaf path of full depth
    tokens = ((np.arange(T) * 37 + 11) % w.vocab).astype(np.int32)
    tokens[0] = greedy[0]
    for d in range(1, m + 1):
        tokens[path[d]] = greedy[d]
    kc, vc = U.copy_cache(cfg1["kc"]), U.copy_cache(cfg1["vc"])
    ref = O.tree_verify_step(tokens, model, kc, vc, S, tree)
    for n in range(1, T):                                              # remove accidental matches elsewhere
        if n not in path[:m + 1] and tokens[n] == ref["node_argmax"][tree["parent"][n]]:
            tokens[n] = (tokens[n] + 1) % w.vocab
    kc, vc = U.copy_cache(cfg1["kc"]), U.copy_cache(cfg1["vc"])
    ref = O.tree_verify_step(tokens, model, kc, vc, S, tree)
    acc = O.accept_longest_prefix(tree, tokens, ref["node_argmax"])
    assert acc["accept_len"] == m + 1
    _, S2 = O.kv_compact(kc, vc, S, acc["acc_nodes"], acc["accept_len"])

    kv = G.device_kv_from_oracle(dm, [cfg1["kc"]], [cfg1["vc"]], [S], cap=S + 2 * T)
    buf = P.StepBuffers(dm, 1, S + K + 1, want_logits=True)
    buf.tree_tokens.copy_(_i32(tokens).view(1, T))
    seq_len = _i32([S])
    P.run_step(dm, kv, buf, None, None, None, seq_len, with_heads=False)
    torch.cuda.synchronize()
    assert int(buf.accept_len[0]) == m + 1 and int(seq_len[0]) == S2
    assert buf.acc_nodes[0].cpu().numpy().tolist() == acc["acc_nodes"].tolist()
    assert buf.acc_tokens[0, :m + 1].cpu().numpy().tolist() == greedy[:m + 1]
    assert int(buf.next_root[0]) == greedy[m + 1]
    # second, chained step: device state only (seq_len and the compacted cache stay on the GPU)
    tokens2 = W.random_tokens(w, f"chain2.{m}", (T,)).numpy().astype(np.int32)
    tokens2[0] = acc["next_root"]
    ref2 = O.tree_verify_step(tokens2, model, kc, vc, S2, tree)
    buf.tree_tokens.copy_(_i32(tokens2).view(1, T))
    P.run_step(dm, kv, buf, None, None, None, seq_len, with_heads=False)
    torch.cuda.synchronize()
    assert np.abs(buf.logits[0].cpu().numpy() - ref2["logits"]).max() <= tol * _scale(ref2["logits"])
    acc2 = O.accept_longest_prefix(tree, tokens2, ref2["node_argmax"])
    assert int(buf.accept_len[0]) == acc2["accept_len"] and int(seq_len[0]) == S2 + acc2["accept_len"]


# ------------------------------------------------------------------------------------------------
# config 2: one full-size 7B-class layer, bf16, 64-node tree, prefix 512
# ------------------------------------------------------------------------------------------------

def _layer_case(w, S_list, max_prefix, x_seed="layer_x"):
    tree = U.oracle_tree(w)
    T = tree["T"]
    Bn = len(S_list)
    cfg = U.oracle_cfg(w)
    lw = U.oracle_layer(w, 0, device=G.DEV)
    dm = G.device_model(w.with_(vocab=1024), heads=False, n_layers=1)          # vocab irrelevant for one layer
    kv = P.DeviceKV(dm, batch=Bn, cap=max_prefix + T, n_layers=1, quant=w.kv_quant)
    x = W.hidden_state(w, x_seed, Bn * T, device=G.DEV).float()                # bf16-valued fp32 rows
    x_ref = x.cpu().numpy().astype(np.float64)
    outs, caches = [], []
    for b, S in enumerate(S_list):
        k, v = W.prefix_kv(w.with_(prefix=tuple(S_list)), 0, b, G.DEV)
        kc = np.zeros((w.kv_heads, S + T, w.head_dim)); vc = np.zeros_like(kc)
        kc[:, :S] = U.stored_rows(w, U.to_np(k)); vc[:, :S] = U.stored_rows(w, U.to_np(v))
        if S:
            kv.write(0, b, 0, k, v)
        outs.append(O.tree_verify_layer(x_ref[b * T:(b + 1) * T], lw, kc, vc, S, tree, cfg))
        caches.append((kc, vc))
    ws = dm.workspace(Bn, max_prefix)
    seq_len = _i32(S_list)
    P.tree_verify_layer(dm.desc, dm.layer(0), 0, x, kv.desc, seq_len, Bn, max_prefix, ws)
    torch.cuda.synchronize()
    return dict(x=x.cpu().numpy(), ref=np.concatenate(outs), caches=caches, kv=kv, T=T)


def _check_layer(r, S_list, dtype):
    tol = TOL[dtype]
    err = np.abs(r["x"] - r["ref"]).max()
    assert err <= tol * _scale(r["ref"]), f"layer output error {err} vs scale {_scale(r['ref'])}"
    T = r["T"]
    for b, S in enumerate(S_list):
        k, v = r["kv"].read(0, b, S, T)
        kc, vc = r["caches"][b]
        assert np.abs(U.to_np(k) - kc[:, S:]).max() <= tol * _scale(kc[:, S:])
        assert np.abs(U.to_np(v) - vc[:, S:]).max() <= tol * _scale(vc[:, S:])
        if S:                                                                   # prefix rows untouched, bit for bit
            k0, v0 = r["kv"].read(0, b, 0, S)
            assert np.array_equal(U.to_np(k0), kc[:, :S]) and np.array_equal(U.to_np(v0), vc[:, :S])
    return err / _scale(r["ref"])


def test_cfg2_full_size_layer_bf16():
    w = W.CONFIGS["cfg2_layer_bf16"]
    r = _layer_case(w, list(w.prefix), w.prefix[0])
    rel = _check_layer(r, list(w.prefix), "bf16")
    print(f"cfg2 layer: max error / scale = {rel:.3e}")


@pytest.mark.parametrize("S_list,max_prefix", [([0], 0), ([1], 5), ([77], 100), ([300, 0, 45], 300), ([5000, 131], 5003),
                                                ([31], 31), ([32], 40), ([33], 33),
                                                ([40000], 40000)])      # 13 key-splits: the merge kernel's second group
def test_small_bf16_layer_ragged_and_empty_prefix(S_list, max_prefix):
    w = W.CONFIGS["cfg2_layer_bf16"].with_(d=256, n_heads=2, head_dim=128, ffn=704, name="small_bf16")
    r = _layer_case(w, S_list, max_prefix, x_seed=f"small_x{len(S_list)}")
    _check_layer(r, S_list, "bf16")


@pytest.mark.parametrize("ffn,S_list", [(10240, [40]), (12288, [0, 70]), (32768, [33]), (10208, [40])])
def test_small_bf16_layer_wide_ffn_swiglu_in_the_gemm_epilogue(ffn, S_list):
    """Gate/up matrices of 160, 192 and 512 column bands run whole bands per workgroup (one band, or two in turn) with
    the SwiGLU in the GEMM's epilogue; 159.5 bands (ffn 10208) is the nearest width that takes the separate kernel."""
    w = W.CONFIGS["cfg2_layer_bf16"].with_(d=256, n_heads=2, head_dim=128, ffn=ffn, name=f"wide_ffn{ffn}")
    r = _layer_case(w, S_list, max(S_list), x_seed=f"wide_x{ffn}")
    _check_layer(r, S_list, "bf16")


def test_layer_is_deterministic_run_to_run():
    w = W.CONFIGS["cfg2_layer_bf16"].with_(d=512, n_heads=4, head_dim=128, ffn=1408, name="det_bf16")
    a = _layer_case(w, [130], 130)
    b = _layer_case(w, [130], 130)
    assert np.array_equal(a["x"], b["x"])


# ------------------------------------------------------------------------------------------------
# config 3 shapes with fewer layers: full widths, vocab 128000, 4 Medusa heads, prefix 1024
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("bias_std", [0.0, 1.0], ids=["no_bias", "head_bias"])
def test_cfg3_shapes_two_layers_full_step_bf16(bias_std):
    w = W.CONFIGS["cfg3_step_1k"].with_(n_layers=2, head_bias_std=bias_std)
    S = w.prefix[0]
    tol = TOL["bf16"]
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
    ties = check_argmax_near_tie(cand[:1], hl[:1], heads["head_logits"][:1], tol * hscale)
    off = 1
    for k in range(K):
        c = tree["caps"][k]
        ties += check_topk_near_tie(cand[off:off + c], hl[k + 1], heads["head_logits"][k + 1], c, tol * hscale)
        off += c
    gpu_tokens = buf.tree_tokens[0].cpu().numpy()
    assert gpu_tokens.tolist() == cand[tree["cand_slot"]].tolist()
    if ties == 0:
        assert gpu_tokens.tolist() == heads["tree_tokens"].tolist()

    # verify on the GPU's own tree tokens (identical inputs for the discrete stages)
    ref = O.tree_verify_step(gpu_tokens, model, kc, vc, S, tree)
    lg = buf.logits[0].cpu().numpy()
    lscale = _scale(ref["logits"])
    err = np.abs(lg - ref["logits"]).max()
    print(f"cfg3/2 layers: logits err/scale {err / lscale:.3e}, head logits err/scale "
          f"{np.abs(hl - heads['head_logits']).max() / hscale:.3e}")
    assert err <= tol * lscale
    assert np.abs(U.to_np(buf.hidden[0]) - ref["hidden"]).max() <= tol * _scale(ref["hidden"])
    gpu_am = buf.node_argmax[0].cpu().numpy()
    check_argmax_near_tie(gpu_am, lg, ref["logits"], tol * lscale)
    acc = O.accept_longest_prefix(tree, gpu_tokens, gpu_am)                   # oracle rule on the GPU's ids
    assert int(buf.accept_len[0]) == acc["accept_len"] and int(buf.best_path[0]) == acc["best_path"]
    assert buf.acc_nodes[0].cpu().numpy().tolist() == acc["acc_nodes"].tolist()
    assert buf.acc_tokens[0].cpu().numpy().tolist() == acc["acc_tokens"].tolist()
    assert int(seq_len[0]) == S + acc["accept_len"]
    assert buf.kv_src_slots[0].cpu().numpy().tolist() == [S + n if n >= 0 else -1 for n in acc["acc_nodes"]]


# ------------------------------------------------------------------------------------------------
# integer kernels in isolation: bit exact
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("spec,tid", [(W.TREE15, P.MDZ_TREE_15), (W.TREE64, P.MDZ_TREE_64),
                                      (W.TREE64K5, P.MDZ_TREE_64_K5)], ids=["tree15", "tree64", "tree64k5"])
@pytest.mark.parametrize("vocab", [2, 3, 5, 1000])
def test_accept_fuzz_bit_exact(spec, tid, vocab):
    from oracle import tree as OT
    tree = OT.build_tree(spec.caps, spec.budgets)
    T, K = tree["T"], tree["K"]
    Bn = 257
    toks = W.uniform_int(21, f"g.acc.tok.{spec.name}.{vocab}", (Bn, T), 0, vocab)
    ams = W.uniform_int(21, f"g.acc.am.{spec.name}.{vocab}", (Bn, T), 0, vocab)
    dev = lambda *s: torch.zeros(*s, dtype=torch.int32, device=G.DEV)
    out = dict(accept_len=dev(Bn), best_path=dev(Bn), acc_nodes=dev(Bn, K + 1), acc_tokens=dev(Bn, K + 1),
               next_root=dev(Bn), last_node=dev(Bn))
    P.accept_longest_prefix(tid, toks.to(G.DEV), ams.to(G.DEV), Bn, **out)
    torch.cuda.synchronize()
    out = {k: v.cpu().numpy() for k, v in out.items()}
    for b in range(Bn):
        a = O.accept_longest_prefix(tree, toks[b].numpy(), ams[b].numpy())
        assert out["accept_len"][b] == a["accept_len"] and out["best_path"][b] == a["best_path"]
        assert out["acc_nodes"][b].tolist() == a["acc_nodes"].tolist()
        assert out["acc_tokens"][b].tolist() == a["acc_tokens"].tolist()
        assert out["next_root"][b] == a["next_root"] and out["last_node"][b] == a["last_node"]


@pytest.mark.parametrize("dtype", ["bf16", "fp32", "fp16"])
def test_kv_compact_bit_exact_ragged_batch(dtype):
    from oracle import tree as OT
    spec = W.TREE64
    tree = OT.build_tree(spec.caps, spec.budgets)
    T, K = tree["T"], tree["K"]
    L, H, hd, Bn = 3, 2, 128, 5
    S_list = [0, 7, 33, 100, 64]
    max_prefix = 100
    cap = max_prefix + T
    dm = P.DeviceModel(d=H * hd, n_heads=H, head_dim=hd, ffn=64, vocab=64, n_layers=L, dtype=dtype, tree="tree64")
    kv = P.DeviceKV(dm, batch=Bn, cap=cap)
    kcs, vcs = [], []
    for b in range(Bn):
        kb, vb = [], []
        for l in range(L):
            k = W.normal(5, f"cmp.k.{b}.{l}", (H, cap, hd), 1.0, dm.tdtype)
            v = W.normal(5, f"cmp.v.{b}.{l}", (H, cap, hd), 1.0, dm.tdtype)
            kv.write(l, b, 0, k, v)
            kb.append(U.to_np(k).astype(np.float64)); vb.append(U.to_np(v).astype(np.float64))
        kcs.append(kb); vcs.append(vb)
    # accepted chains of every length, taken from retrieve rows
    rows = [0, 37, 20, 30, 36]
    lens = [1, 5, 3, 4, 2]
    acc_nodes = np.full((Bn, K + 1), -1, np.int32)
    for b in range(Bn):
        A = min(lens[b], int((tree["retrieve"][rows[b]] >= 0).sum()))
        lens[b] = A
        acc_nodes[b, :A] = tree["retrieve"][rows[b], :A]
    seq_len = _i32(S_list)
    slots = torch.zeros(Bn, K + 1, dtype=torch.int32, device=G.DEV)
    P.kv_compact(kv.desc, P.MDZ_TREE_64, _i32(acc_nodes), _i32(lens), seq_len, slots, Bn, max_prefix)
    torch.cuda.synchronize()
    for b in range(Bn):
        src, S2 = O.kv_compact(kcs[b], vcs[b], S_list[b], acc_nodes[b], lens[b])
        assert slots[b].cpu().numpy().tolist() == src.tolist() and int(seq_len[b]) == S2
        for l in range(L):
            k, v = kv.read(l, b, 0, cap)
            assert np.array_equal(U.to_np(k), kcs[b][l]) and np.array_equal(U.to_np(v), vcs[b][l])


def test_empty_batch_and_bad_arguments():
    w = W.CONFIGS["cfg1_tiny_fp32"]
    dm = G.device_model(w)
    kv = P.DeviceKV(dm, batch=1, cap=64 + 15)
    buf = P.StepBuffers(dm, 1, 64)
    seq_len = _i32([64])
    # B = 0: accepted, nothing happens
    P.tree_verify_step(dm.desc, dm.weights, buf.tree_tokens, kv.desc, seq_len, 0, 64, buf.node_argmax, None, None, buf.ws)
    P.accept_longest_prefix(dm.tree, buf.tree_tokens, buf.node_argmax, 0, buf.accept_len, buf.best_path, buf.acc_nodes,
                            buf.acc_tokens, buf.next_root, buf.last_node)
    P.kv_compact(kv.desc, dm.tree, buf.acc_nodes, buf.accept_len, seq_len, buf.kv_src_slots, 0, 64)
    # prefix bound beyond the cache, workspace too small, batch beyond the cache
    with pytest.raises(P.MedusaError) as e:
        P.tree_verify_step(dm.desc, dm.weights, buf.tree_tokens, kv.desc, seq_len, 1, 65, buf.node_argmax, None, None, buf.ws)
    assert e.value.status == -2
    with pytest.raises(P.MedusaError) as e:
        P.tree_verify_step(dm.desc, dm.weights, buf.tree_tokens, kv.desc, seq_len, 1, 64, buf.node_argmax, None, None,
                           buf.ws[:1024])
    assert e.value.status == -4
    with pytest.raises(P.MedusaError) as e:
        P.tree_verify_step(dm.desc, dm.weights, buf.tree_tokens, kv.desc, seq_len, 2, 64, buf.node_argmax, None, None, buf.ws)
    assert e.value.status == -2
    torch.cuda.synchronize()
    assert int(seq_len[0]) == 64


# ------------------------------------------------------------------------------------------------
# config 3 at full depth, config 4 (long prefix), config 5 (ragged batch), full-size properties
# ------------------------------------------------------------------------------------------------

def _oracle_step_streamed(w, tokens, S, tree, kv_rows=None):
    """The oracle's verify step for sequence 0 with layer weights generated one layer at a time."""
    assert S == w.prefix[0]
    return _oracle_steps_streamed(w, {0: tokens}, tree, kv_rows)[0]


def _oracle_steps_streamed(w, tokens_by_seq, tree, kv_rows=None):
    """The oracle's verify step for the sequences in ``tokens_by_seq`` (sequence index -> tree tokens), with layer
    weights generated one layer at a time and shared by the sequences (bounded host memory).  Per sequence:
    logits, hidden, node_argmax and the KV rows written by the layers in ``kv_rows``."""
    cfg = U.oracle_cfg(w)
    T = tree["T"]
    emb_t = W.embedding(w, G.DEV)
    xs = {b: U.to_np(emb_t[torch.as_tensor(np.asarray(t), device=G.DEV).long()]).astype(np.float64)
          for b, t in tokens_by_seq.items()}
    del emb_t
    kept = {b: {} for b in xs}
    for l in range(w.n_layers):
        lw = U.oracle_layer(w, l, device=G.DEV)
        for b in xs:
            S = w.prefix[b]
            k, v = W.prefix_kv(w, l, b, G.DEV)
            kc = np.zeros((w.kv_heads, S + T, w.head_dim)); vc = np.zeros_like(kc)
            kc[:, :S] = U.to_np(k); vc[:, :S] = U.to_np(v)
            xs[b] = O.tree_verify_layer(xs[b], lw, kc, vc, S, tree, cfg)
            if kv_rows is not None and l in kv_rows:
                kept[b][l] = (kc[:, S:].copy(), vc[:, S:].copy())
    fin = dict(cfg=cfg, g_final=U.to_np(W.norm_gain(w, "g_final", G.DEV)), lm_head=U.to_np(W.lm_head(w, G.DEV)))
    out = {}
    for b, x in xs.items():
        hidden, logits = O._final(x, fin)
        out[b] = dict(logits=logits, hidden=hidden, node_argmax=O.argmax_lowest(logits), kv=kept[b])
    return out


_FULL_DEPTH_REF = {}


def full_depth_reference(w, tokens, S, tree):
    """The oracle's 32-layer pass of one seed, computed once per test session (about a minute of CPU work)."""
    if w.seed not in _FULL_DEPTH_REF:
        _FULL_DEPTH_REF[w.seed] = _oracle_step_streamed(w, tokens, S, tree, kv_rows={0, 31})
    return _FULL_DEPTH_REF[w.seed]


@pytest.mark.parametrize("seed", [W.BASE_SEED, W.BASE_SEED + 1], ids=["base_seed", "second_seed"])
def test_cfg3_full_depth_32_layers_every_logit(seed):
    """The metric's own workload: 32 layers, prefix 1024, all 64 x 128000 logits against the oracle, on two seeds."""
    w = W.CONFIGS["cfg3_step_1k"].with_(seed=seed)
    S = w.prefix[0]
    tol = TOL["bf16"]
    tree = U.oracle_tree(w)
    T = tree["T"]
    tokens = W.random_tokens(w, "full_depth_tree", (T,)).numpy()
    ref = full_depth_reference(w, tokens, S, tree)
    dm = G.device_model(w, heads=False)
    kv = G.device_kv_random_prefix(dm, w, cap=S + T)
    buf = P.StepBuffers(dm, 1, S, want_logits=True)
    buf.tree_tokens.copy_(_i32(tokens).view(1, T))
    seq_len = _i32([S])
    P.run_step(dm, kv, buf, None, None, None, seq_len, with_heads=False)
    torch.cuda.synchronize()
    lg = buf.logits[0].cpu().numpy()
    scale = _scale(ref["logits"])
    err = np.abs(lg - ref["logits"]).max()
    print(f"cfg3 full depth (seed {seed}): logits err/scale {err / scale:.3e}")
    assert err <= tol * scale
    assert np.abs(U.to_np(buf.hidden[0]) - ref["hidden"]).max() <= tol * _scale(ref["hidden"])
    gpu_am = buf.node_argmax[0].cpu().numpy()
    n_tie = check_argmax_near_tie(gpu_am, lg, ref["logits"], tol * scale)
    print(f"cfg3 full depth (seed {seed}): {n_tie} of {T} argmax rows fall under the near-tie rule")
    acc = O.accept_longest_prefix(tree, tokens, gpu_am)
    assert int(buf.accept_len[0]) == acc["accept_len"] and int(seq_len[0]) == S + acc["accept_len"]
    if seed != W.BASE_SEED:
        return
    # compaction ran after the pass (node 0 stays in place): row S is the root's row
    for l, (kr, vr) in ref["kv"].items():
        k, v = kv.read(l, 0, S, 1)
        assert np.abs(U.to_np(k) - kr[:, :1]).max() <= tol * _scale(kr) and np.abs(U.to_np(v) - vr[:, :1]).max() <= tol * _scale(vr)
    # run-to-run determinism of the whole step at full size (fixed-order reductions everywhere)
    kv2 = G.device_kv_random_prefix(dm, w, cap=S + T)
    buf2 = P.StepBuffers(dm, 1, S, want_logits=True)
    buf2.tree_tokens.copy_(_i32(tokens).view(1, T))
    seq2 = _i32([S])
    P.run_step(dm, kv2, buf2, None, None, None, seq2, with_heads=False)
    torch.cuda.synchronize()
    assert torch.equal(buf.logits, buf2.logits) and torch.equal(buf.node_argmax, buf2.node_argmax)
    # sibling relabelling at full size: nodes 8 and 9 (each with one child: 39, 40) are isomorphic subtrees
    assert tree["parent"][39] == 8 and tree["parent"][40] == 9 and not (tree["parent"] == 39).any()
    perm = np.arange(T); perm[[8, 9, 39, 40]] = [9, 8, 40, 39]
    kv3 = G.device_kv_random_prefix(dm, w, cap=S + T)
    buf2.tree_tokens.copy_(_i32(tokens[perm]).view(1, T))
    seq2.copy_(_i32([S]))
    P.run_step(dm, kv3, buf2, None, None, None, seq2, with_heads=False)
    torch.cuda.synchronize()
    lg3 = buf2.logits[0].cpu().numpy()
    assert np.abs(lg3 - lg[perm]).max() <= 2e-3 * scale


def test_cfg3_full_depth_with_binary16_feed_forward_operands():
    """The same 32-layer pass with the feed-forward products on binary16 operands (a bf16 model's option): same
    oracle, same bound, and the error has to come out well under the plain bf16 path's (its two largest rounding terms
    shrink eightfold)."""
    w = W.CONFIGS["cfg3_step_1k"].with_(ffn_f16=True)
    S = w.prefix[0]
    tree = U.oracle_tree(w)
    T = tree["T"]
    tokens = W.random_tokens(w, "full_depth_tree", (T,)).numpy()
    ref = full_depth_reference(w, tokens, S, tree)
    dm = G.device_model(w, heads=False)
    kv = G.device_kv_random_prefix(dm, w, cap=S + T)
    buf = P.StepBuffers(dm, 1, S, want_logits=True)
    buf.tree_tokens.copy_(_i32(tokens).view(1, T))
    seq_len = _i32([S])
    P.run_step(dm, kv, buf, None, None, None, seq_len, with_heads=False)
    torch.cuda.synchronize()
    lg = buf.logits[0].cpu().numpy()
    scale = _scale(ref["logits"])
    err = np.abs(lg - ref["logits"]).max()
    print(f"cfg3 full depth, binary16 feed-forward operands: logits err/scale {err / scale:.3e}")
    assert err <= 8e-3 * scale
    assert np.abs(U.to_np(buf.hidden[0]) - ref["hidden"]).max() <= 8e-3 * _scale(ref["hidden"])
    gpu_am = buf.node_argmax[0].cpu().numpy()
    check_argmax_near_tie(gpu_am, lg, ref["logits"], 8e-3 * scale)
    acc = O.accept_longest_prefix(tree, tokens, gpu_am)
    assert int(buf.accept_len[0]) == acc["accept_len"] and int(seq_len[0]) == S + acc["accept_len"]


@pytest.mark.parametrize("S", [4096, 8192, 16384])
def test_cfg4_long_prefix_full_size_layer(S):
    w = W.CONFIGS["cfg4_step_16k"].with_(n_layers=1, prefix=(S,))
    r = _layer_case(w, [S], S, x_seed=f"long_x{S}")
    rel = _check_layer(r, [S], "bf16")
    print(f"cfg4 layer S={S}: max error / scale = {rel:.3e}")


def test_cfg5_ragged_batch_16_sequences():
    """16 sequences with seeded ragged prefixes (256..4096), one 7B-shaped layer + LM head + heads + accept +
    per-sequence compaction.  rows = 1024 > 64, so the GEMMs take the many-row kernel."""
    ragged_batch_case(W.CONFIGS["cfg5_ragged_b16"].with_(n_layers=1))


def ragged_batch_case(w):
    Bn = w.batch
    tol = TOL[w.dtype]
    tree = U.oracle_tree(w)
    T, K = tree["T"], tree["K"]
    max_prefix = max(w.prefix)
    dm = G.device_model(w)
    kv = G.device_kv_random_prefix(dm, w, cap=max_prefix + T)
    model = U.oracle_model(w, device=G.DEV)
    h = W.hidden_state(w, "ragged_h", Bn, device=G.DEV)
    buf = P.StepBuffers(dm, Bn, max_prefix, want_logits=True, want_head_logits=True)
    seq_len = _i32(list(w.prefix))
    P.run_step(dm, kv, buf, h.view(Bn, 1, -1), None, None, seq_len)
    torch.cuda.synchronize()
    hl = buf.head_logits.cpu().numpy()
    cand = buf.cand_flat.cpu().numpy()
    toks = buf.tree_tokens.cpu().numpy()
    lgs = buf.logits.cpu().numpy()
    ams = buf.node_argmax.cpu().numpy()
    worst = 0.0
    for b in range(Bn):
        S = w.prefix[b]
        heads = O.medusa_heads(U.to_np(h)[b], model, tree)
        hscale = _scale(heads["head_logits"])
        assert np.abs(hl[b] - heads["head_logits"]).max() <= tol * hscale
        off = 1
        check_argmax_near_tie(cand[b, :1], hl[b, :1], heads["head_logits"][:1], tol * hscale)
        for k in range(K):
            c = tree["caps"][k]
            check_topk_near_tie(cand[b, off:off + c], hl[b, k + 1], heads["head_logits"][k + 1], c, tol * hscale)
            off += c
        assert toks[b].tolist() == cand[b][tree["cand_slot"]].tolist()
        kc, vc = U.oracle_prefix_cache(w, b, S + T, device=G.DEV)
        ref = O.tree_verify_step(toks[b], model, kc, vc, S, tree)
        scale = _scale(ref["logits"])
        err = np.abs(lgs[b] - ref["logits"]).max()
        worst = max(worst, err / scale)
        assert err <= tol * scale
        check_argmax_near_tie(ams[b], lgs[b], ref["logits"], tol * scale)
        acc = O.accept_longest_prefix(tree, toks[b], ams[b])
        assert int(buf.accept_len[b]) == acc["accept_len"] and int(seq_len[b]) == S + acc["accept_len"]
        assert buf.acc_nodes[b].cpu().numpy().tolist() == acc["acc_nodes"].tolist()
        assert buf.kv_src_slots[b].cpu().numpy().tolist() == [S + n if n >= 0 else -1 for n in acc["acc_nodes"]]
        k, v = kv.read(0, b, S, 1)
        assert np.abs(U.to_np(k) - kc[0][:, S:S + 1]).max() <= tol * _scale(kc[0][:, S:S + T])
    print(f"cfg5 ragged batch: worst logits err/scale {worst:.3e}")


def test_cfg4_full_depth_32_layers_at_16k_prefix():
    """Config 4's longest point as a whole step: 32 layers at a 16384-token prefix (K and V of 4.3 GB each, so layer
    offsets pass 2^32 bytes; 64 queries per workgroup and 8 key-splits in every layer), every logit, the hidden
    states, node_argmax, acceptance, and the KV rows written by layers 0, 16 and 31 against the oracle."""
    w = W.CONFIGS["cfg4_step_16k"]
    S = w.prefix[0]
    tol = TOL["bf16"]
    tree = U.oracle_tree(w)
    T = tree["T"]
    tokens = W.random_tokens(w, "full_depth_tree_16k", (T,)).numpy()
    ref = _oracle_step_streamed(w, tokens, S, tree, kv_rows={0, 16, 31})
    dm = G.device_model(w, heads=False)
    kv = G.device_kv_random_prefix(dm, w, cap=S + T)
    buf = P.StepBuffers(dm, 1, S, want_logits=True)
    buf.tree_tokens.copy_(_i32(tokens).view(1, T))
    seq_len = _i32([S])
    P.tree_verify_step(dm.desc, dm.weights, buf.tree_tokens, kv.desc, seq_len, 1, S, buf.node_argmax, buf.hidden,
                       buf.logits, buf.ws)
    torch.cuda.synchronize()
    lg = buf.logits[0].cpu().numpy()
    scale = _scale(ref["logits"])
    err = np.abs(lg - ref["logits"]).max()
    print(f"cfg4 16K full depth: logits err/scale {err / scale:.3e}")
    assert err <= tol * scale
    assert np.abs(U.to_np(buf.hidden[0]) - ref["hidden"]).max() <= tol * _scale(ref["hidden"])
    gpu_am = buf.node_argmax[0].cpu().numpy()
    n_tie = check_argmax_near_tie(gpu_am, lg, ref["logits"], tol * scale)
    print(f"cfg4 16K full depth: {n_tie} of {T} argmax rows fall under the near-tie rule")
    for l, (kr, vr) in ref["kv"].items():                      # all T rows each layer wrote, before any compaction
        k, v = kv.read(l, 0, S, T)
        assert np.abs(U.to_np(k) - kr).max() <= tol * _scale(kr) and np.abs(U.to_np(v) - vr).max() <= tol * _scale(vr)
    k0, _ = kv.read(31, 0, S - 3, 3)                           # the prefix rows next to them are untouched
    kp, _ = W.prefix_kv(w, 31, 0, G.DEV)
    assert torch.equal(k0, kp[:, S - 3:])
    P.accept_longest_prefix(dm.tree, buf.tree_tokens, buf.node_argmax, 1, buf.accept_len, buf.best_path, buf.acc_nodes,
                            buf.acc_tokens, buf.next_root, buf.last_node)
    P.kv_compact(kv.desc, dm.tree, buf.acc_nodes, buf.accept_len, seq_len, buf.kv_src_slots, 1, S)
    torch.cuda.synchronize()
    acc = O.accept_longest_prefix(tree, tokens, gpu_am)
    assert int(buf.accept_len[0]) == acc["accept_len"] and int(seq_len[0]) == S + acc["accept_len"]
    assert buf.kv_src_slots[0].cpu().numpy().tolist() == [S + n if n >= 0 else -1 for n in acc["acc_nodes"]]


def test_cfg5_full_depth_32_layers_ragged_batch():
    """Config 5 as it is timed: 16 ragged sequences through all 32 layers, heads + verify + accept + per-sequence
    compaction.  The oracle follows the shortest, the longest and one middle sequence through the whole depth (every
    logit, hidden states, head logits); the integer outputs of all 16 sequences are checked bit for bit with the
    oracle's rules applied to the GPU's own ids (identical inputs for the discrete stages)."""
    w = W.CONFIGS["cfg5_ragged_b16"]
    Bn = w.batch
    tol = TOL["bf16"]
    tree = U.oracle_tree(w)
    T, K = tree["T"], tree["K"]
    max_prefix = max(w.prefix)
    order = sorted(range(Bn), key=lambda b: w.prefix[b])
    subset = [order[0], order[Bn // 2], order[-1]]
    dm = G.device_model(w)
    kv = G.device_kv_random_prefix(dm, w, cap=max_prefix + T)
    h = W.hidden_state(w, "ragged_h32", Bn, device=G.DEV)
    buf = P.StepBuffers(dm, Bn, max_prefix, want_logits=True, want_head_logits=True)
    seq_len = _i32(list(w.prefix))
    P.run_step(dm, kv, buf, h.view(Bn, 1, -1), None, None, seq_len)
    torch.cuda.synchronize()
    hl = buf.head_logits.cpu().numpy()
    cand = buf.cand_flat.cpu().numpy()
    toks = buf.tree_tokens.cpu().numpy()
    ams = buf.node_argmax.cpu().numpy()
    # every sequence: the discrete stages on the GPU's own values
    for b in range(Bn):
        S = w.prefix[b]
        assert cand[b, 0] == O.argmax_lowest(hl[b, :1].astype(np.float64))[0]
        off = 1
        for k in range(K):
            c = tree["caps"][k]
            assert cand[b, off:off + c].tolist() == O.topk_lowest(hl[b, k + 1].astype(np.float64), c).tolist()
            off += c
        assert toks[b].tolist() == cand[b][tree["cand_slot"]].tolist()
        lg_b = buf.logits[b].cpu().numpy()
        assert np.array_equal(ams[b], O.argmax_lowest(lg_b.astype(np.float64)))
        acc = O.accept_longest_prefix(tree, toks[b], ams[b])
        assert int(buf.accept_len[b]) == acc["accept_len"] and int(buf.best_path[b]) == acc["best_path"]
        assert int(seq_len[b]) == S + acc["accept_len"]
        assert buf.acc_nodes[b].cpu().numpy().tolist() == acc["acc_nodes"].tolist()
        assert buf.acc_tokens[b].cpu().numpy().tolist() == acc["acc_tokens"].tolist()
        assert int(buf.next_root[b]) == acc["next_root"] and int(buf.last_node[b]) == acc["last_node"]
        assert buf.kv_src_slots[b].cpu().numpy().tolist() == [S + n if n >= 0 else -1 for n in acc["acc_nodes"]]
    # the chosen sequences: floating point against the oracle through the whole depth
    refs = _oracle_steps_streamed(w, {b: toks[b] for b in subset}, tree, kv_rows={0, 31})
    heads_model = dict(lm_head=U.to_np(W.lm_head(w, G.DEV)),
                       medusa=[dict(w1=U.to_np(W.medusa_w1(w, k, G.DEV)), b1=None, lm=U.to_np(W.medusa_lm(w, k, G.DEV)))
                               for k in range(1, K + 1)])
    for b in subset:
        S, ref = w.prefix[b], refs[b]
        heads = O.medusa_heads(U.to_np(h)[b], heads_model, tree)
        hscale = _scale(heads["head_logits"])
        assert np.abs(hl[b] - heads["head_logits"]).max() <= tol * hscale
        check_argmax_near_tie(cand[b, :1], hl[b, :1], heads["head_logits"][:1], tol * hscale)
        lg = buf.logits[b].cpu().numpy()
        scale = _scale(ref["logits"])
        err = np.abs(lg - ref["logits"]).max()
        n_tie = check_argmax_near_tie(ams[b], lg, ref["logits"], tol * scale)
        print(f"cfg5 full depth, sequence {b} (prefix {S}): logits err/scale {err / scale:.3e}, {n_tie} near-tie rows")
        assert err <= tol * scale
        assert np.abs(U.to_np(buf.hidden[b]) - ref["hidden"]).max() <= tol * _scale(ref["hidden"])
        for l, (kr, vr) in ref["kv"].items():                  # the root's row stays at slot S through compaction
            k, v = kv.read(l, b, S, 1)
            assert np.abs(U.to_np(k) - kr[:, :1]).max() <= tol * _scale(kr)
            assert np.abs(U.to_np(v) - vr[:, :1]).max() <= tol * _scale(vr)


def test_sequence_length_beyond_max_prefix_sets_the_status_word():
    """Lengths live on the device; one beyond max_prefix cannot be refused by the call, so the kernels clamp it (every
    access stays inside the cache) and report it through the cache's status word."""
    w = W.CONFIGS["cfg1_tiny_fp32"]
    dm = G.device_model(w)
    T = w.tree.n_nodes
    kv = P.DeviceKV(dm, batch=2, cap=64 + T)
    buf = P.StepBuffers(dm, 2, 64)
    seq_len = _i32([64, 10])
    P.run_step(dm, kv, buf, None, None, None, seq_len, with_heads=False)
    torch.cuda.synchronize()
    assert int(kv.status.item()) == 0
    kv.check_status()
    seq_len.copy_(_i32([65, 10]))                     # one past the bound the call was given
    P.tree_verify_step(dm.desc, dm.weights, buf.tree_tokens, kv.desc, seq_len, 2, 64, buf.node_argmax, None, None, buf.ws)
    torch.cuda.synchronize()
    assert int(kv.status.item()) & P.MDZ_STATUS_SEQ_RANGE
    with pytest.raises(P.MedusaError):
        kv.check_status()
    kv.status.zero_()
    seq_len.copy_(_i32([-3, 10]))
    P.kv_compact(kv.desc, dm.tree, buf.acc_nodes, buf.accept_len, seq_len, buf.kv_src_slots, 2, 64)
    torch.cuda.synchronize()
    assert int(kv.status.item()) & P.MDZ_STATUS_SEQ_RANGE
