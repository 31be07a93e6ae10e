"""Pins for grouped-query attention in the oracle (Table 1 of the paper: 32 query heads, 8 key/value heads):
tree == causal still holds, the layer equals PyTorch CPU library ops with the key/value heads repeated, and
duplicating the key/value projections of a grouped model gives the identical multi-head model."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workload as W
from oracle import medusa as O
from oracle import tree as OT
from tests import util as U

GQA = W.CONFIGS["cfg1_tiny_fp32"].with_(name="tiny_gqa", n_kv_heads=2)          # 4 query heads, 2 key/value heads


def test_tree_pass_equals_causal_decoding_with_grouped_heads():
    w = GQA
    model = U.oracle_model(w, dtype="fp64")
    assert model["layers"][0]["wk"].shape == (2 * w.head_dim, w.d)
    tree = U.oracle_tree(w)
    S = 11
    toks = W.random_tokens(w, "gqa_prefix", (S,)).numpy()
    kc, vc = O.empty_cache(model["cfg"], S + tree["T"])
    assert kc[0].shape == (2, S + tree["T"], w.head_dim)
    O.causal_decode(toks, model, kc, vc, 0)
    tree_tokens = W.random_tokens(w, "gqa_tree", (tree["T"],)).numpy()
    kt, vt = U.copy_cache(kc), U.copy_cache(vc)
    got = O.tree_verify_step(tree_tokens, model, kt, vt, S, tree)
    for n in range(tree["T"]):
        path = U.path_to(tree, n)
        k1, v1 = U.copy_cache(kc), U.copy_cache(vc)
        lg, _ = O.causal_decode(tree_tokens[path], model, k1, v1, S)
        np.testing.assert_allclose(got["logits"][n], lg[-1], rtol=0, atol=1e-9 * np.abs(lg).max())


def test_grouped_layer_matches_torch_library_ops_with_repeated_kv_heads():
    w = GQA
    cfg = U.oracle_cfg(w, dtype="fp64")
    lw = U.oracle_layer(w, 0)
    H, Hkv, hd, S, n = w.n_heads, w.kv_heads, w.head_dim, 7, 5
    chain = OT.build_tree((1, 1, 1, 1), (1, 1, 1, 1))
    x = W.hidden_state(w, "gqa_chain_x", n).numpy()
    kpre = W.normal(5, "gqa_kpre", (Hkv, S, hd)).numpy()
    vpre = W.normal(5, "gqa_vpre", (Hkv, S, hd)).numpy()
    kc = np.zeros((Hkv, S + n, hd)); kc[:, :S] = kpre
    vc = np.zeros((Hkv, S + n, hd)); vc[:, :S] = vpre
    got = O.tree_verify_layer(x, lw, kc, vc, S, chain, cfg)

    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    xt = t(x)
    xn = F.rms_norm(xt, (w.d,), weight=t(lw["g_attn"]), eps=cfg["rms_eps"])
    q = F.linear(xn, t(lw["wq"])).view(n, H, hd).transpose(0, 1)
    k = F.linear(xn, t(lw["wk"])).view(n, Hkv, hd).transpose(0, 1)
    v = F.linear(xn, t(lw["wv"])).view(n, Hkv, hd).transpose(0, 1)

    def rope_c(a):
        half = hd // 2
        z = torch.complex(a[..., :half], a[..., half:])
        pos = torch.arange(S, S + n, dtype=torch.float64)
        theta = pos[:, None] * (cfg["rope_base"] ** (-torch.arange(half, dtype=torch.float64) * 2 / hd))[None, :]
        z = z * torch.polar(torch.ones_like(theta), theta)
        return torch.cat([z.real, z.imag], dim=-1)

    q, k = rope_c(q), rope_c(k)
    kk = torch.cat([t(kpre), k], dim=1).repeat_interleave(H // Hkv, dim=0)      # query head h reads kv head h // group
    vv = torch.cat([t(vpre), v], dim=1).repeat_interleave(H // Hkv, dim=0)
    allow = torch.ones(n, S + n, dtype=torch.bool).tril(diagonal=S)
    att = F.scaled_dot_product_attention(q, kk, vv, attn_mask=allow).transpose(0, 1).reshape(n, H * hd)
    xr = xt + F.linear(att, t(lw["wo"]))
    xn2 = F.rms_norm(xr, (w.d,), weight=t(lw["g_ffn"]), eps=cfg["rms_eps"])
    ref = (xr + F.linear(F.silu(F.linear(xn2, t(lw["wgate"]))) * F.linear(xn2, t(lw["wup"])), t(lw["wdown"]))).numpy()
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-11 * np.abs(ref).max())
    np.testing.assert_allclose(kc[:, S:], k.numpy(), rtol=0, atol=1e-12)


def test_grouped_model_equals_multi_head_model_with_duplicated_kv_projections():
    w = GQA
    cfg_g = U.oracle_cfg(w, dtype="fp64")
    cfg_m = dict(cfg_g, n_kv_heads=w.n_heads)
    lw = U.oracle_layer(w, 0)
    H, Hkv, hd = w.n_heads, w.kv_heads, w.head_dim
    rep = lambda m: np.repeat(np.asarray(m).reshape(Hkv, hd, w.d), H // Hkv, axis=0).reshape(H * hd, w.d)
    lw_m = dict(lw, wk=rep(lw["wk"]), wv=rep(lw["wv"]))
    tree = U.oracle_tree(w)
    S, T = 6, tree["T"]
    x = W.hidden_state(w, "gqa_dup_x", T).numpy()
    kpre = W.normal(9, "dup_k", (Hkv, S, hd)).numpy()
    vpre = W.normal(9, "dup_v", (Hkv, S, hd)).numpy()
    kg = np.zeros((Hkv, S + T, hd)); kg[:, :S] = kpre
    vg = np.zeros((Hkv, S + T, hd)); vg[:, :S] = vpre
    km, vm = np.repeat(kg, H // Hkv, axis=0), np.repeat(vg, H // Hkv, axis=0)
    a = O.tree_verify_layer(x, lw, kg, vg, S, tree, cfg_g)
    b = O.tree_verify_layer(x, lw_m, km, vm, S, tree, cfg_m)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-12 * np.abs(b).max())
    np.testing.assert_allclose(np.repeat(kg, H // Hkv, axis=0), km, rtol=0, atol=0)
