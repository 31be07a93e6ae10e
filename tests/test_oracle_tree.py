"""Pins for oracle/tree.py against what the paper and arithmetic fix (CPU only).

Section 3.2: the visibility matrix is [T,T] and encodes parent-child dependencies of all
candidate paths; the retrieve table is [N_paths, K+1], one row per candidate path.
"""
import numpy as np
import pytest

import workload as W
from oracle import tree as OT


def _tree(spec):
    return OT.build_tree(spec.caps, spec.budgets)


# closed-form counts.  tree15: the full binary-ish tree over caps (2,2,2): widths 1,2,4,8.
# tree64: width at depth m = #{(a_1..a_m) : 1 <= a_i <= caps_i, prod a_i <= B_m} with B = (10,12,4,3):
#   m=1: a <= 10 -> 10;  m=2: sum_{a=1..10} min(10, floor(12/a)) = 10+6+4+3+2+2+1+1+1+1 = 31
#   m=3: ordered triples with product <= 4: prod 1:1, 2:3, 3:3, 4:6 -> 13;  m=4: prod <= 3: 1+4+4 = 9
# tree64k5 (five heads), caps = B = (9,10,4,3,2): m=1: 9;  m=2: sum_{a=1..9} min(10, floor(10/a)) = 10+5+3+2+2+1+1+1+1 = 26
#   m=3: 13 as above;  m=4: 9 as above;  m=5: ordered 5-tuples with product <= 2: 1 + 5 = 6
# ones in the mask = sum_n (depth_n + 1).
EXPECT = {
    "tree15": dict(widths=[1, 2, 4, 8], leaves=8, ones=1 + 2 * 2 + 4 * 3 + 8 * 4),
    "tree64": dict(widths=[1, 10, 31, 13, 9], leaves=38, ones=1 + 10 * 2 + 31 * 3 + 13 * 4 + 9 * 5),
    "tree64k5": dict(widths=[1, 9, 26, 13, 9, 6], leaves=34, ones=1 + 9 * 2 + 26 * 3 + 13 * 4 + 9 * 5 + 6 * 6),
}


@pytest.mark.parametrize("spec", [W.TREE15, W.TREE64, W.TREE64K5], ids=lambda s: s.name)
def test_counts_and_shapes(spec):
    t = _tree(spec)
    e = EXPECT[spec.name]
    K = len(spec.caps)
    assert t["T"] == spec.n_nodes == sum(e["widths"])
    assert np.bincount(t["depth"], minlength=K + 1).tolist() == e["widths"]
    assert t["mask"].shape == (t["T"], t["T"])
    assert t["retrieve"].shape == (e["leaves"], K + 1) == (spec.n_paths, K + 1)
    assert int(t["mask"].sum()) == e["ones"]
    assert e["ones"] == {"tree15": 49, "tree64": 211, "tree64k5": 230}[spec.name]
    assert t["n_cand"] == 1 + sum(spec.caps)


@pytest.mark.parametrize("spec", [W.TREE15, W.TREE64, W.TREE64K5], ids=lambda s: s.name)
def test_mask_is_ancestor_relation(spec):
    """mask == reflexive-transitive closure of the parent relation, computed here by boolean matrix
    powers of the child->parent adjacency (a different route from walking pointers)."""
    t = _tree(spec)
    T = t["T"]
    P = np.zeros((T, T), dtype=np.int64)
    for n in range(1, T):
        P[n, t["parent"][n]] = 1
    closure = np.eye(T, dtype=np.int64)
    power = np.eye(T, dtype=np.int64)
    for _ in range(len(spec.caps)):
        power = power @ P
        closure += power
    assert np.array_equal(closure > 0, t["mask"])
    # row popcount = depth + 1; strictly lower-triangular apart from the diagonal; root column all ones
    assert np.array_equal(t["mask"].sum(1), t["depth"] + 1)
    assert not np.triu(t["mask"], 1).any()
    assert t["mask"][:, 0].all()
    # parents precede children, depth(parent) = depth - 1
    for n in range(1, T):
        p = t["parent"][n]
        assert 0 <= p < n and t["depth"][p] == t["depth"][n] - 1
    assert t["parent"][0] == -1 and t["depth"][0] == 0


@pytest.mark.parametrize("spec", [W.TREE15, W.TREE64, W.TREE64K5], ids=lambda s: s.name)
def test_retrieve_rows_are_root_to_leaf_chains(spec):
    t = _tree(spec)
    T = t["T"]
    children = [[] for _ in range(T)]
    for n in range(1, T):
        children[t["parent"][n]].append(n)
    leaves = [n for n in range(T) if not children[n]]
    seen_leaves = []
    covered = set()
    for row in t["retrieve"]:
        nodes = [int(n) for n in row if n >= 0]
        assert row.tolist() == nodes + [-1] * (len(row) - len(nodes))       # -1 padding only at the end
        assert nodes[0] == 0
        for a, b in zip(nodes, nodes[1:]):
            assert t["parent"][b] == a
        assert not children[nodes[-1]]
        seen_leaves.append(nodes[-1])
        covered.update(nodes)
    assert seen_leaves == leaves                                             # ascending leaf order, each once
    assert covered == set(range(T))                                          # every node lies on some path


def test_cand_slot_tree15_by_hand():
    # flat buffer [root | h1r0 h1r1 | h2r0 h2r1 | h3r0 h3r1]; nodes by depth then lexicographic ranks
    t = _tree(W.TREE15)
    assert t["cand_slot"].tolist() == [0, 1, 2, 3, 4, 3, 4, 5, 6, 5, 6, 5, 6, 5, 6]
    assert t["parent"].tolist() == [-1, 0, 0, 1, 1, 2, 2, 3, 3, 4, 4, 5, 5, 6, 6]


def test_cand_slot_tree64_properties():
    t = _tree(W.TREE64)
    caps = W.TREE64.caps
    offs = np.concatenate([[1], 1 + np.cumsum(caps)])
    for n in range(1, t["T"]):
        d = t["depth"][n]
        s = t["cand_slot"][n]
        assert offs[d - 1] <= s < offs[d]                    # slot lies in head d's segment
        assert s - offs[d - 1] == t["tuples"][n][-1]          # at the node's own rank
    # children of one parent use distinct slots (distinct candidates)
    for p in range(t["T"]):
        slots = [t["cand_slot"][n] for n in range(1, t["T"]) if t["parent"][n] == p]
        assert len(set(slots)) == len(slots)
    # max rank used per depth: 9, 9, 3, 2 (budget 10, 12/1, 4/1, 3/1 capped by caps)
    maxrank = [max(tp[-1] for tp in t["tuples"] if len(tp) == m) for m in range(1, 5)]
    assert maxrank == [9, 9, 3, 2]
    # first children always exist along the all-zero path (the "greedy" path)
    assert [t["tuples"].index((0,) * m) for m in range(5)] == [0, 1, 11, 42, 55]
