"""Chained speculative steps at 7B width (two layers, full vocabulary) with planted acceptance: the tree carries the
model's own greedy continuation along one root-to-leaf path down to a scheduled depth, so steps accept 1 .. K+1 tokens,
the cache is compacted by several rows, and the next step runs on the compacted cache: verification, acceptance,
compaction and chaining together, against the oracle, in bf16, with grouped heads + 8-bit cache rows, and in fp16 with
the five-head tree.  The planted tokens come from the GPU's own argmax (read back between verify-only runs), so the
accepted length is exact by construction; the oracle checks logits, acceptance outputs, the compacted rows and lengths."""
import numpy as np
import pytest
import torch

import workload as W
import paper_2603_03383_amd as P
from oracle import medusa as O
from tests import gpu_util as G
from tests import util as U
from tests.test_gpu_parity import TOL, _i32, _scale, check_argmax_near_tie
from tests.test_gpu_kv8 import KV8_DIRECT_TOL

pytestmark = pytest.mark.gpu

VARIANTS = {
    "bf16": dict(),
    "gqa8-kv8": dict(n_kv_heads=8, kv_quant="fp8e4m3"),
    "fp16-k5": dict(dtype="fp16", tree=W.TREE64K5, n_kv_heads=8),
}


def _rows_close(got, ref, w):
    """Compacted cache rows against the oracle's: the storage bound, or (8-bit rows) the neighbouring grid value."""
    tol = TOL[w.dtype]
    ref16 = O.round_to_storage(ref, w.dtype)
    d = np.abs(got - ref16)
    near = d <= tol * max(1.0, np.abs(ref).max())
    if not w.kv_quant:
        return bool(np.all(near))
    step = d <= 0.13 * np.abs(ref16) + tol * np.abs(ref).max(-1, keepdims=True)
    return bool(np.all(near | step)) and (1.0 - near.mean()) < 0.10


@pytest.mark.parametrize("variant", list(VARIANTS), ids=list(VARIANTS))
def test_chain_with_planted_acceptance_at_7b_width(variant):
    w = W.CONFIGS["cfg3_step_1k"].with_(name=f"chain7b_{variant}", n_layers=2, prefix=(100,), **VARIANTS[variant])
    tol = TOL[w.dtype]
    tree = U.oracle_tree(w)
    T, K = tree["T"], tree["K"]
    path = [int(n) for n in [r for r in tree["retrieve"] if r[K] >= 0][-1]]      # the last full-depth path
    schedule = [2, 0, K, 1]                                                         # planted depth per step -> A = depth + 1
    S = w.prefix[0]
    cap = S + sum(d + 1 for d in schedule) + T
    model = U.oracle_model(w, device=G.DEV, heads=False)
    dm = G.device_model(w, heads=False)
    kc, vc = U.oracle_prefix_cache(w, 0, cap, device=G.DEV)
    kv = G.device_kv_random_prefix(dm, w, cap=cap)
    buf = P.StepBuffers(dm, 1, cap - T, want_logits=True)
    seq_len = _i32([S])
    root = 17
    emitted = []
    for step, depth in enumerate(schedule):
        tokens = ((np.arange(T) * 7919 + 13 * step + 5) % w.vocab).astype(np.int32)     # fillers
        tokens[0] = root

        def verify_only():
            buf.tree_tokens.copy_(_i32(tokens).view(1, T))
            P.tree_verify_step(dm.desc, dm.weights, buf.tree_tokens, kv.desc, seq_len, 1, buf.max_prefix, buf.node_argmax,
                               buf.hidden, buf.logits, buf.ws)
            torch.cuda.synchronize()
            return buf.node_argmax[0].cpu().numpy()

        for j in range(1, depth + 1):                                                # plant level by level
            am = verify_only()
            tokens[path[j]] = am[path[j - 1]]
        for _ in range(4):                                                           # no accidental match anywhere else
            am = verify_only()
            bad = [n for n in range(1, T) if n not in path[:depth + 1] and tokens[n] == am[tree["parent"][n]]]
            if not bad:
                break
            for n in bad:
                tokens[n] = (tokens[n] + 1) % w.vocab
        assert not bad
        buf.tree_tokens.copy_(_i32(tokens).view(1, T))
        P.run_step(dm, kv, buf, None, None, None, seq_len, with_heads=False)
        torch.cuda.synchronize()
        # oracle: same tokens, its own cache
        ref = O.tree_verify_step(tokens, model, kc, vc, S, tree)
        g = buf.logits[0].cpu().numpy()
        lscale = _scale(ref["logits"])
        err = np.abs(g - ref["logits"]).max()
        assert err <= (KV8_DIRECT_TOL[w.dtype] if w.kv_quant else tol) * lscale, (step, err / lscale)   # 8-bit rows: see test_gpu_kv8
        gpu_am = buf.node_argmax[0].cpu().numpy()
        check_argmax_near_tie(gpu_am, g, ref["logits"], tol * lscale)
        acc = O.accept_longest_prefix(tree, tokens, gpu_am)
        A = acc["accept_len"]
        assert A == depth + 1 == int(buf.accept_len[0])
        assert buf.acc_nodes[0].cpu().numpy().tolist() == acc["acc_nodes"].tolist()
        assert buf.acc_tokens[0].cpu().numpy().tolist() == acc["acc_tokens"].tolist()
        assert int(buf.next_root[0]) == acc["next_root"] and int(buf.last_node[0]) == acc["last_node"]
        src, S2 = O.kv_compact(kc, vc, S, acc["acc_nodes"], A)
        assert int(seq_len[0]) == S2 and buf.kv_src_slots[0].cpu().numpy().tolist() == src.tolist()
        for l in range(w.n_layers):
            k, v = kv.read(l, 0, S, A)
            assert _rows_close(U.to_np(k), kc[l][:, S:S2], w) and _rows_close(U.to_np(v), vc[l][:, S:S2], w), (step, l)
            if S:                                                                    # the prefix stays as it was
                k0, v0 = kv.read(l, 0, 0, w.prefix[0])
                assert np.array_equal(U.to_np(k0), O.round_to_storage(kc[l][:, :w.prefix[0]], w.dtype))
        emitted += acc["acc_tokens"][:A].tolist()
        print(f"{variant} step {step}: planted depth {depth}, accepted {A}, logits err/scale {err / lscale:.3e}")
        S, root = S2, acc["next_root"]
    assert len(emitted) == sum(d + 1 for d in schedule) and int(seq_len[0]) == w.prefix[0] + len(emitted)
