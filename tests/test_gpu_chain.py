"""GPU: the chained on-device decode loop (heads -> verify -> accept -> compact repeated with no host round trip),
eager and replayed from a HIP graph, against the oracle's loop and against plain greedy decoding."""
import numpy as np
import pytest
import torch

import workload as W
import paper_2603_03383_amd as P
from oracle import medusa as O
from tests import gpu_util as G
from tests import util as U
from tests.test_gpu_parity import _i32

pytestmark = pytest.mark.gpu

N_STEPS = 6


@pytest.fixture(scope="module")
def chain_case():
    w = W.CONFIGS["cfg1_tiny_fp32"]
    S = w.prefix[0]
    model = U.oracle_model(w)
    tree = U.oracle_tree(w)
    T, K = tree["T"], tree["K"]
    prefix_tokens = W.random_tokens(w, "prefix", (S,)).numpy()
    cap = S + N_STEPS * (K + 1) + T
    kc, vc = O.empty_cache(model["cfg"], cap)
    lg, hid = O.causal_decode(prefix_tokens, model, kc, vc, 0)
    # the oracle's loop
    kc_o, vc_o = U.copy_cache(kc), U.copy_cache(vc)
    h, root, S_run = hid[-1], int(O.argmax_lowest(lg[-1:])[0]), S
    steps = []
    for _ in range(N_STEPS):
        heads = O.medusa_heads(h, model, tree)             # its root is the base head's argmax on h ...
        toks = heads["tree_tokens"]
        assert int(toks[0]) == root                        # ... which is the token the previous step predicted
        ref = O.tree_verify_step(toks, model, kc_o, vc_o, S_run, tree)
        acc = O.accept_longest_prefix(tree, toks, ref["node_argmax"])
        _, S_run = O.kv_compact(kc_o, vc_o, S_run, acc["acc_nodes"], acc["accept_len"])
        steps.append((acc["acc_tokens"].tolist(), int(acc["accept_len"])))
        h, root = ref["hidden"][acc["last_node"]], int(acc["next_root"])
    # plain greedy decoding of as many tokens as the loop emitted
    emitted = [t for toks, n in steps for t in toks[:n]]
    kc_g, vc_g = U.copy_cache(kc), U.copy_cache(vc)
    greedy, tok = [], int(O.argmax_lowest(lg[-1:])[0])
    for i in range(len(emitted)):
        greedy.append(tok)
        l1, _ = O.causal_decode([tok], model, kc_g, vc_g, S + i)
        tok = int(O.argmax_lowest(l1)[0])
    return dict(w=w, S=S, cap=cap, kc=kc, vc=vc, steps=steps, emitted=emitted, greedy=greedy,
                h0=hid[-1].astype(np.float32), root0=int(O.argmax_lowest(lg[-1:])[0]), K=K, T=T)


def test_oracle_loop_emits_the_greedy_continuation(chain_case):
    """Speculative decoding with exact-match acceptance changes the schedule, never the text."""
    assert chain_case["emitted"] == chain_case["greedy"]


@pytest.mark.parametrize("use_graph", [False, True], ids=["eager", "graph"])
def test_chained_loop_matches_the_oracle_loop(chain_case, use_graph):
    c = chain_case
    w, S = c["w"], c["S"]
    dm = G.device_model(w)
    max_prefix = c["cap"] - c["T"]
    for attempt in range(3 if use_graph else 1):           # graph: replay the whole chain three times, eager work between
        kv = G.device_kv_from_oracle(dm, [c["kc"]], [c["vc"]], [S], cap=c["cap"])
        if attempt == 0:
            dec = P.ChainedDecoder(dm, kv, 1, max_prefix, use_graph=use_graph)
        else:
            dec.kv = kv                                    # same addresses are not guaranteed: rebuild the graph
            dec._graph = None
        dec.prime(torch.tensor(c["h0"], device=G.DEV).view(1, -1), _i32([c["root0"]]), _i32([S]))
        tokens, lens = dec.run(N_STEPS)
        torch.cuda.synchronize()
        got = [(tokens[i, 0].cpu().tolist(), int(lens[i, 0])) for i in range(N_STEPS)]
        assert got == c["steps"], f"attempt {attempt}"
        assert int(dec.seq_len[0]) == S + len(c["emitted"])
        _ = (torch.ones(1024, device=G.DEV) * 3).sum().item()      # unrelated eager work and a sync between replays
