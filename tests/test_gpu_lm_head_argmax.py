"""The verify pass's LM head with the per-row argmax in its epilogue (taken when the caller asks for no logits)
against the same pass with logits: identical node_argmax, bit for bit, including exact ties across tiles, waves and
workgroups (total order: value descending, then lowest column) and a vocabulary whose last band is ragged."""
import numpy as np
import pytest
import torch

import workload as W
import paper_2603_03383_amd as P
from tests import gpu_util as G
from tests.test_gpu_parity import _i32

pytestmark = pytest.mark.gpu


def _both_ways(dm, w, tokens, S):
    """node_argmax and logits of the pass that writes logits, and node_argmax of the pass that does not."""
    T = dm.tree_info["T"]
    Bn = tokens.shape[0]
    out = []
    for want in (True, False):
        kv = G.device_kv_random_prefix(dm, w, cap=S + T)
        buf = P.StepBuffers(dm, Bn, S, want_logits=want)
        buf.tree_tokens.copy_(_i32(tokens))
        buf.node_argmax.fill_(-7)
        buf.ws.fill_(0xA5)
        P.tree_verify_step(dm.desc, dm.weights, buf.tree_tokens, kv.desc, _i32([S] * Bn), Bn, S, buf.node_argmax, buf.hidden,
                           buf.logits, buf.ws)
        torch.cuda.synchronize()
        if not want and T == 64:
            # The pass without logits really took the epilogue argmax: the workspace's own [64, vocab] fp32 logits
            # region (which the other route fills when the caller passes no buffer) is still untouched.  Nothing else
            # the pass leaves alone is that large (the heads' logits are 5 rows).
            words = buf.ws[:buf.ws.numel() // 4 * 4].view(torch.int32)
            untouched = int((words == torch.tensor(0xA5A5A5A5 - (1 << 32), dtype=torch.int32, device=words.device)).sum()) * 4
            assert untouched >= Bn * T * dm.desc.vocab * 4
        out.append((buf.node_argmax.cpu().numpy().copy(), None if buf.logits is None else buf.logits.cpu().numpy()))
    return out


def _small(dtype, vocab, tree, **kw):
    return W.CONFIGS["cfg1_tiny_fp32"].with_(name=f"argmax_{dtype}_{vocab}", dtype=dtype, d=256, n_heads=2, head_dim=128,
                                             ffn=512, vocab=vocab, n_layers=1, tree=tree, prefix=(40,), **kw)


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
@pytest.mark.parametrize("tree", [W.TREE64, W.TREE15, W.TREE1], ids=lambda t: t.name)
@pytest.mark.parametrize("vocab", [16384, 16416, 40000])
def test_epilogue_argmax_equals_argmax_of_the_logits(dtype, tree, vocab):
    """64, 15 and 1 rows (both row-tile variants); vocabularies that end on a band, one tile into a band, and that
    give the workgroups uneven numbers of bands."""
    w = _small(dtype, vocab, tree)
    dm = G.device_model(w, heads=False)
    T = dm.tree_info["T"]
    tokens = W.random_tokens(w, "argmax_tree", (1, T)).numpy()
    (am_l, lg), (am_f, _) = _both_ways(dm, w, tokens, 40)
    assert np.array_equal(am_l[0], np.argmax(lg[0], axis=-1))        # numpy: the first of equal maxima
    assert np.array_equal(am_f, am_l)


@pytest.mark.parametrize("period", [1, 7, 4099])
def test_exact_ties_go_to_the_lowest_column(period):
    """An LM head whose rows repeat with a period: columns v and v + period have bit-identical logits (same operands,
    same accumulation order), so every row's maximum is attained many times, in different tiles, waves and workgroups."""
    w = _small("bf16", 16416, W.TREE64)
    dm = G.device_model(w, heads=False)
    base = W.lm_head(w, G.DEV)
    idx = torch.arange(w.vocab, device=G.DEV) % period
    dm.set_lm_head(base[idx].contiguous())
    dm.finalize()
    T = dm.tree_info["T"]
    tokens = W.random_tokens(w, "argmax_tie_tree", (1, T)).numpy()
    (am_l, lg), (am_f, _) = _both_ways(dm, w, tokens, 40)
    assert np.array_equal(lg[0][:, :w.vocab - period], lg[0][:, period:])   # the ties are exact
    assert (am_l < period).all()
    assert np.array_equal(am_l[0], np.argmax(lg[0], axis=-1))
    assert np.array_equal(am_f, am_l)


def test_full_size_lm_head_two_layers_batch_of_one():
    """The benchmark's shape: 64 rows x 128000 columns x 4096 features."""
    w = W.CONFIGS["cfg3_step_1k"].with_(name="argmax_full", n_layers=2)
    dm = G.device_model(w, heads=False)
    T = dm.tree_info["T"]
    tokens = W.random_tokens(w, "argmax_full_tree", (1, T)).numpy()
    (am_l, lg), (am_f, _) = _both_ways(dm, w, tokens, w.prefix[0])
    assert np.array_equal(am_l[0], np.argmax(lg[0], axis=-1))
    assert np.array_equal(am_f, am_l)
