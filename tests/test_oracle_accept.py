"""Pins for the oracle's acceptance and compaction rules (CPU only, integer work).

Section 3.2 (zero-copy retrieval): the best path is picked by the acceptance criterion and its tokens
are gathered through the [N_paths, K+1] table.  The criterion here is greedy exact match; the oracle
states it as brute force over the table rows, and these tests pin that statement against two other
formulations: a recursive walk from the root, and a vectorised cumulative-product form.
"""
from itertools import product

import numpy as np
import pytest

import workload as W
from oracle import medusa as O
from oracle import tree as OT


def _children(tree):
    ch = [[] for _ in range(tree["T"])]
    for n in range(1, tree["T"]):
        ch[tree["parent"][n]].append(n)
    return ch


def _longest_from(n, tokens, argmax, ch):
    """Recursive formulation: length of the longest matching chain that starts at accepted node n."""
    best = 1
    for c in ch[n]:
        if tokens[c] == argmax[n]:
            best = max(best, 1 + _longest_from(c, tokens, argmax, ch))
    return best


def _vectorised(tree, tokens, argmax):
    r = tree["retrieve"]
    valid = r >= 0
    rn = np.where(valid, r, 0)
    par = np.where(rn > 0, tree["parent"][rn], 0)
    ok = valid & ((rn == 0) | (np.asarray(tokens)[rn] == np.asarray(argmax)[par]))
    lens = np.cumprod(ok, axis=1).sum(axis=1)
    p = int(np.argmax(lens))                       # first maximum = lowest path index
    return int(lens[p]), p


def _check(tree, tokens, argmax, ch):
    acc = O.accept_longest_prefix(tree, tokens, argmax)
    A = acc["accept_len"]
    assert 1 <= A <= tree["K"] + 1
    assert A == _longest_from(0, tokens, argmax, ch)
    assert (A, acc["best_path"]) == _vectorised(tree, tokens, argmax)
    nodes = acc["acc_nodes"]
    assert nodes[0] == 0 and (nodes[A:] == -1).all() and (acc["acc_tokens"][A:] == -1).all()
    for j in range(1, A):                                                   # returned chain is valid
        assert tree["parent"][nodes[j]] == nodes[j - 1]
        assert tokens[nodes[j]] == argmax[nodes[j - 1]]
    assert acc["acc_tokens"][:A].tolist() == [int(tokens[n]) for n in nodes[:A]]
    assert nodes[:A].tolist() == tree["retrieve"][acc["best_path"], :A].tolist()
    assert acc["last_node"] == nodes[A - 1] and acc["next_root"] == argmax[nodes[A - 1]]
    # maximality: the last accepted node has no matching child
    assert all(tokens[c] != argmax[nodes[A - 1]] for c in ch[nodes[A - 1]])
    return acc


@pytest.mark.parametrize("caps,budgets,vocab", [((2, 1), (2, 2), 3), ((2, 2), (2, 4), 2), ((3,), (3,), 3),
                                                ((1, 1, 1), (1, 1, 1), 2), ((2, 2), (2, 2), 2)])
def test_exhaustive_on_tiny_trees(caps, budgets, vocab):
    tree = OT.build_tree(caps, budgets)
    T = tree["T"]
    assert T <= 7
    ch = _children(tree)
    n = 0
    for tokens in product(range(vocab), repeat=T):
        for argmax in product(range(vocab), repeat=T):
            _check(tree, np.array(tokens), np.array(argmax), ch)
            n += 1
    assert n == vocab ** (2 * T)


@pytest.mark.parametrize("spec", [W.TREE15, W.TREE64, W.TREE64K5], ids=lambda s: s.name)
@pytest.mark.parametrize("vocab", [2, 3, 4, 50])
def test_fuzz_on_static_trees(spec, vocab):
    tree = OT.build_tree(spec.caps, spec.budgets)
    ch = _children(tree)
    toks = W.uniform_int(11, f"acc.tok.{spec.name}.{vocab}", (300, tree["T"]), 0, vocab).numpy()
    ams = W.uniform_int(11, f"acc.am.{spec.name}.{vocab}", (300, tree["T"]), 0, vocab).numpy()
    lens = [_check(tree, toks[i], ams[i], ch)["accept_len"] for i in range(300)]
    if vocab <= 3:
        assert max(lens) == tree["K"] + 1                                   # full-depth acceptance occurs
    if vocab == 50:
        assert min(lens) == 1 and max(lens) >= 2                            # root-only acceptance occurs


def test_distinct_siblings_give_a_unique_chain():
    """With distinct sibling tokens (what top-k produces) the accepted node chain is the unique
    walk-down chain; only the path index needs a tie-break."""
    tree = OT.build_tree(W.TREE64.caps, W.TREE64.budgets)
    ch = _children(tree)
    T = tree["T"]
    for trial in range(200):
        tokens = np.zeros(T, dtype=np.int64)
        for p in range(T):                                     # distinct tokens among siblings
            for r, c in enumerate(ch[p]):
                tokens[c] = r
        argmax = W.uniform_int(13, f"acc.unique.{trial}", (T,), 0, 4).numpy()
        acc = O.accept_longest_prefix(tree, tokens, argmax)
        chain, n = [0], 0
        while True:
            nxt = [c for c in ch[n] if tokens[c] == argmax[n]]
            if not nxt:
                break
            assert len(nxt) == 1
            n = nxt[0]
            chain.append(n)
        assert acc["acc_nodes"][:acc["accept_len"]].tolist() == chain


def test_tie_break_lowest_path_index_by_hand():
    # tree7: root; 1,2; (0,0)=3,(0,1)=4,(1,0)=5,(1,1)=6.  paths: [0,1,3],[0,1,4],[0,2,5],[0,2,6]
    tree = OT.build_tree((2, 2), (2, 4))
    assert tree["retrieve"].tolist() == [[0, 1, 3], [0, 1, 4], [0, 2, 5], [0, 2, 6]]
    tokens = np.array([9, 5, 5, 1, 7, 7, 1])        # duplicate siblings 1,2 (token 5)
    argmax = np.array([5, 7, 7, 0, 0, 0, 0])        # root predicts 5; both children predict 7
    acc = O.accept_longest_prefix(tree, tokens, argmax)
    # paths 1 ([0,1,4]) and 2 ([0,2,5]) both have length 3 -> lowest index wins
    assert (acc["accept_len"], acc["best_path"]) == (3, 1)
    assert acc["acc_nodes"].tolist() == [0, 1, 4] and acc["acc_tokens"].tolist() == [9, 5, 7]
    # nothing matches: only the root is accepted, via path 0
    acc = O.accept_longest_prefix(tree, np.array([9, 1, 1, 1, 1, 1, 1]), np.zeros(7, dtype=int))
    assert (acc["accept_len"], acc["best_path"], acc["acc_nodes"].tolist()) == (1, 0, [0, -1, -1])
    assert acc["next_root"] == 0 and acc["last_node"] == 0


def test_compact_moves_rows_and_pads():
    H, cap, hd, L = 2, 40, 4, 3
    base = np.arange(H * cap * hd, dtype=np.float64).reshape(H, cap, hd)
    kc = [base + 1000 * l for l in range(L)]
    vc = [-(base + 1000 * l) for l in range(L)]
    k0 = [a.copy() for a in kc]
    S = 10
    acc_nodes = np.array([0, 2, 6, -1, -1], dtype=np.int32)
    src, S2 = O.kv_compact(kc, vc, S, acc_nodes, 3)
    assert src.tolist() == [10, 12, 16, -1, -1] and S2 == 13
    for l in range(L):
        assert np.array_equal(kc[l][:, 10], k0[l][:, 10])
        assert np.array_equal(kc[l][:, 11], k0[l][:, 12])
        assert np.array_equal(kc[l][:, 12], k0[l][:, 16])      # old row 12 was consumed before being overwritten
        assert np.array_equal(vc[l][:, 12], -k0[l][:, 16])
        assert np.array_equal(kc[l][:, :10], k0[l][:, :10])
        assert np.array_equal(kc[l][:, 13:], k0[l][:, 13:])    # rows beyond S+A are left as they were
