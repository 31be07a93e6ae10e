"""Pins of the oracle's 8-bit KV cache format (oracle/kv8.py): the format's closed form and landmarks, brute-force
nearest-value rounding, hand-picked ties, torch's float8_e4m3fn cast as an independent library routine, error bounds,
idempotence, and the effect inside a decoder layer."""
import numpy as np
import pytest
import torch

import workload as W
from oracle import kv8
from oracle import medusa as O
from oracle import tree as OT
from tests import util as U


def test_table_landmarks_and_structure():
    t = kv8.e4m3_table()
    assert t[0x00] == 0.0 and t[0x80] == 0.0 and np.signbit(t[0x80])
    assert t[0x01] == 2.0 ** -9 and t[0x07] == 7 * 2.0 ** -9          # subnormals: m/8 * 2^-6
    assert t[0x08] == 2.0 ** -6                                        # smallest normal
    assert t[0x38] == 1.0 and t[0x3C] == 1.5 and t[0x40] == 2.0
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0                      # largest finite
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF])
    fin = t[:0x7F]
    assert np.all(np.diff(fin) > 0)                                    # monotone in the code
    np.testing.assert_array_equal(t[0x80:0xFF], -t[:0x7F])
    # every normal value has 4 significant bits: value / 2^floor(log2 value) is a multiple of 1/8 in [1, 2)
    nz = fin[8:]
    fr = nz / 2.0 ** np.floor(np.log2(nz))
    assert np.all((fr >= 1) & (fr < 2) & (fr * 8 == np.rint(fr * 8)))
    assert len(np.unique(fin)) == 127


def test_table_equals_torch_float8_e4m3fn_bit_patterns():
    codes = torch.arange(256, dtype=torch.uint8)
    tv = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    t = kv8.e4m3_table()
    np.testing.assert_array_equal(np.isnan(tv), np.isnan(t))
    ok = ~np.isnan(t)
    np.testing.assert_array_equal(tv[ok], t[ok])


def test_round_is_nearest_by_brute_force_with_ties_to_even():
    rng = np.random.default_rng(0)
    y = np.concatenate([rng.uniform(-460, 460, 4000), rng.normal(0, 1, 4000), rng.normal(0, 0.01, 2000),
                        kv8.e4m3_table()[:0x7F], [449.0, -470.0, 1e9]])
    fin = kv8.e4m3_table()[:0x7F]
    mids = (fin[:-1] + fin[1:]) / 2                                    # every exact tie, both signs
    y = np.concatenate([y, mids, -mids])
    got = kv8.e4m3_round(y)
    t = kv8.e4m3_table()
    cand = np.concatenate([np.arange(0x7F), 0x80 + np.arange(0x7F)])
    for yi, c in zip(np.clip(y, -448, 448), got):
        d = np.abs(t[cand] - yi)
        best = cand[d == d.min()]
        if len(best) > 1 and yi != 0:                                  # a tie: the even code wins
            best = best[best % 2 == 0]
        assert c in best or (yi == 0 and c == 0), (yi, c, best)


def test_round_hand_picked():
    # between 16 (0x58) and 18 (0x59): 17 ties to the even code 0x58; between 18 and 20 (0x5A): 19 ties to 0x5A
    assert kv8.e4m3_round(np.array([17.0, 19.0, -17.0, 1.0625, 1.1875])).tolist() == [0x58, 0x5A, 0xD8, 0x38, 0x3A]
    assert kv8.e4m3_round(np.array([448.0, 500.0, -1e6, 2.0 ** -10, 3 * 2.0 ** -10, 0.0, -0.0])).tolist() == \
        [0x7E, 0x7E, 0xFE, 0x00, 0x02, 0x00, 0x00]


def test_round_equals_torch_cast_inside_the_finite_range():
    x = np.concatenate([W.normal(8, "kv8.r", (30000,)).numpy().astype(np.float64) * s for s in (1e-3, 0.1, 1.0, 100.0)])
    x = x[np.abs(x) <= 448]
    got = kv8.e4m3_round(x)
    ref = torch.tensor(x, dtype=torch.float32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    same = got == ref
    # torch keeps the sign of values that round to zero; this format stores +0
    assert np.all(same | ((got == 0) & (ref == 0x80)))


def test_quantize_rows_scale_error_bound_idempotence_zero_rows():
    x = W.normal(9, "kv8.rows", (6, 50, 128)).numpy()
    x[0, 0] = 0.0
    x[1, 3, 17] = 37.5
    codes, scale = kv8.quantize_rows(x)
    assert codes.shape == x.shape and scale.shape == x.shape[:-1] and scale.dtype == np.float32
    amax = np.abs(x).max(-1)
    assert scale[0, 0] == 1.0 and np.all(codes[0, 0] == 0)
    np.testing.assert_array_equal(scale[amax > 0], (amax[amax > 0] / np.float32(448.0)).astype(np.float32))
    assert np.all((codes & 0x7F) <= 0x7E)                               # never a NaN code
    assert np.all((codes & 0x7F).max(-1)[amax > 0] == 0x7E)             # the row maximum maps to +-448
    xd = kv8.dequantize_rows(codes, scale)
    # nearest value with 3 mantissa bits: relative error <= 2^-4 above the subnormal range, absolute <= 2^-10 x scale below
    err = np.abs(xd - x)
    bound = np.maximum(np.abs(x) * 2.0 ** -4, scale[..., None].astype(np.float64) * 2.0 ** -10) * (1 + 1e-6)
    assert np.all(err <= bound)
    c2, s2 = kv8.quantize_rows(xd)                                      # written again: the same codes and scale
    np.testing.assert_array_equal(c2, codes)
    np.testing.assert_array_equal(s2, scale)


def test_layer_with_8bit_cache_equals_layer_on_roundtripped_rows_and_stays_close_to_16bit():
    """kv_quant changes exactly one thing: the rows the attention reads.  Feeding the plain layer a cache whose tree
    rows were replaced by round-tripped rows must give the same attention input; and the 8-bit layer stays within
    a few 1e-3 of the 16-bit layer on this workload's scale (the cost of the compression, reported, not a parity bound)."""
    w = W.CONFIGS["cfg1_tiny_fp32"].with_(name="kv8_tiny", dtype="bf16", ffn=704)
    cfg = U.oracle_cfg(w)
    cfg8 = dict(cfg, kv_quant="fp8e4m3")
    lw = U.oracle_layer(w, 0)
    tree = OT.build_tree(w.tree.caps, w.tree.budgets)
    T, S = tree["T"], 40
    x = W.hidden_state(w, "kv8_x", T).float().numpy().astype(np.float64)
    k0, v0 = W.prefix_kv(w.with_(prefix=(S,)), 0, 0)
    def cache(fn):
        kc = np.zeros((w.kv_heads, S + T, w.head_dim)); vc = np.zeros_like(kc)
        kc[:, :S] = fn(U.to_np(k0)); vc[:, :S] = fn(U.to_np(v0))
        return kc, vc
    kc8, vc8 = cache(kv8.roundtrip_rows)
    y8 = O.tree_verify_layer(x, lw, kc8, vc8, S, tree, cfg8)
    kc, vc = cache(lambda a: a.astype(np.float64))
    y = O.tree_verify_layer(x, lw, kc, vc, S, tree, cfg)
    # the tree rows of the 8-bit cache are the round trip of the 16-bit layer's unrounded rows: check via idempotence
    np.testing.assert_array_equal(kv8.roundtrip_rows(kc8[:, S:]), kc8[:, S:])
    assert np.all(np.abs(kc8[:, S:] - kc[:, S:]) <= np.abs(kc[:, S:]) * 2.0 ** -4 + np.abs(kc[:, S:]).max(-1, keepdims=True) * 2.0 ** -9)
    rel = np.abs(y8 - y).max() / max(1.0, np.abs(y).max())
    assert 0 < rel < 2e-2, rel
