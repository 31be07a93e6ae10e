"""CPU oracle, part 1: the static candidate tree and its constant tensors.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file;
it exists so that tests, the smoke check and the bench's cpu_baseline leg have
an independent statement of what the HIP library must compute.

Follows the paper's "Tensorization of Tree Topology" and "Zero-Copy Retrieval
Strategy" paragraphs (Section 3.2): the tree is fixed offline and shipped as a
[T,T] visibility matrix that encodes parent-child dependencies, a node-index
mapping, and a [N_paths, K+1] lookup table of per-path offsets.  The paper does
not print a tree; the rule used here (rank tuples under per-depth budgets) is
this build's reading and is described in build_tree's docstring.
"""
from __future__ import annotations

from itertools import product

import numpy as np


def build_tree(caps, budgets):
    """Static tree from per-head top-k sizes ``caps`` and per-depth budgets.

    A node is a tuple of ranks (r_1, .., r_m), 1 <= m <= K = len(caps), where r_i
    is "the r_i-th best candidate of Medusa head i" (0-based, r_i < caps[i-1]).
    A tuple belongs to the tree iff prod(r_i + 1) <= budgets[m-1] and its parent
    tuple (r_1..r_{m-1}) belongs to the tree.  The empty tuple is the root (the
    base model's own next token, depth 0); head k supplies depth k (Section 3.1:
    head k predicts position t+k+1, the base head t+1).

    Node order: by depth, then lexicographic tuple; so node 0 is the root and a
    parent always precedes its children.

    Returns a dict of numpy arrays:
      tuples     list of rank tuples, one per node
      parent     [T] int32, -1 for the root
      depth      [T] int32
      cand_slot  [T] int32: index into the flat candidate buffer
                 [root | top-k of head 1 | top-k of head 2 | ...]
      mask       [T,T] bool: mask[i][j] <=> j is i or an ancestor of i
      retrieve   [N_paths, K+1] int32: node indices root->leaf for each leaf
                 (leaves in ascending node index), padded with -1
    """
    K = len(caps)
    assert len(budgets) == K
    nodes = {(): None}
    for m in range(1, K + 1):
        for tup in product(*[range(c) for c in caps[:m]]):
            if tup[:-1] not in nodes:
                continue
            p = 1
            for r in tup:
                p *= r + 1
            if p <= budgets[m - 1]:
                nodes[tup] = None
    tuples = sorted(nodes.keys(), key=lambda t: (len(t), t))
    index = {t: i for i, t in enumerate(tuples)}
    T = len(tuples)
    parent = np.full(T, -1, dtype=np.int32)
    depth = np.zeros(T, dtype=np.int32)
    cand_slot = np.zeros(T, dtype=np.int32)
    offs = [1]
    for c in caps:
        offs.append(offs[-1] + c)
    for i, t in enumerate(tuples):
        depth[i] = len(t)
        if t:
            parent[i] = index[t[:-1]]
            cand_slot[i] = offs[len(t) - 1] + t[-1]
    mask = np.zeros((T, T), dtype=bool)
    for i in range(T):
        j = i
        while j >= 0:
            mask[i, j] = True
            j = parent[j]
    has_child = np.zeros(T, dtype=bool)
    for i in range(1, T):
        has_child[parent[i]] = True
    leaves = [i for i in range(T) if not has_child[i]]
    retrieve = np.full((len(leaves), K + 1), -1, dtype=np.int32)
    for p, leaf in enumerate(leaves):
        chain = []
        j = leaf
        while j >= 0:
            chain.append(j)
            j = parent[j]
        chain.reverse()
        retrieve[p, :len(chain)] = chain
    return dict(tuples=tuples, parent=parent, depth=depth, cand_slot=cand_slot, mask=mask,
                retrieve=retrieve, n_cand=offs[-1], caps=tuple(caps), K=K, T=T)
