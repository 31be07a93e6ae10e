"""Test helpers: turn a workload's named tensors into the oracle's plain-dict model."""
from __future__ import annotations

import numpy as np
import torch

import workload as W
from oracle import medusa as O
from oracle import tree as OT


def to_np(t: torch.Tensor) -> np.ndarray:
    """Exact float32 numpy view of a bf16/fp32 tensor (bf16 -> fp32 is exact)."""
    return t.detach().to("cpu", torch.float32).numpy()


def oracle_cfg(w: W.Workload, dtype=None) -> dict:
    return dict(n_layers=w.n_layers, d=w.d, n_heads=w.n_heads, n_kv_heads=w.kv_heads, head_dim=w.head_dim, ffn=w.ffn,
                vocab=w.vocab, rms_eps=w.rms_eps, rope_base=w.rope_base, dtype=dtype or w.dtype, kv_quant=w.kv_quant)


def oracle_tree(w: W.Workload) -> dict:
    return OT.build_tree(w.tree.caps, w.tree.budgets)


def oracle_layer(w: W.Workload, layer: int, device="cpu") -> dict:
    lw = {m: to_np(W.layer_weight(w, layer, m, device)) for m in W.LAYER_MATS}
    lw["g_attn"] = to_np(W.norm_gain(w, f"layer{layer}.g_attn", device))
    lw["g_ffn"] = to_np(W.norm_gain(w, f"layer{layer}.g_ffn", device))
    return lw


def oracle_model(w: W.Workload, device="cpu", heads=True, dtype=None) -> dict:
    m = dict(cfg=oracle_cfg(w, dtype),
             layers=[oracle_layer(w, l, device) for l in range(w.n_layers)],
             embed=to_np(W.embedding(w, device)), lm_head=to_np(W.lm_head(w, device)),
             g_final=to_np(W.norm_gain(w, "g_final", device)), medusa=[])
    if heads:
        for k in range(1, w.n_medusa + 1):
            b1 = W.medusa_b1(w, k, device)
            m["medusa"].append(dict(w1=to_np(W.medusa_w1(w, k, device)), b1=None if b1 is None else to_np(b1),
                                    lm=to_np(W.medusa_lm(w, k, device))))
    return m


def stored_rows(w: W.Workload, rows: np.ndarray) -> np.ndarray:
    """What the cache holds after rows (exact storage-dtype values) were written into it."""
    if w.kv_quant == "fp8e4m3":
        from oracle import kv8
        return kv8.roundtrip_rows(rows)
    return rows.astype(np.float64)


def oracle_prefix_cache(w: W.Workload, seq: int, cap: int, device="cpu"):
    """Per-layer [H,cap,hd] float64 caches whose first S rows are the workload's random prefix KV."""
    cfg = oracle_cfg(w)
    kc, vc = O.empty_cache(cfg, cap)
    S = w.prefix[seq]
    for l in range(w.n_layers):
        k, v = W.prefix_kv(w, l, seq, device)
        kc[l][:, :S] = stored_rows(w, to_np(k))
        vc[l][:, :S] = stored_rows(w, to_np(v))
    return kc, vc


def copy_cache(c):
    return [a.copy() for a in c]


def path_to(tree: dict, n: int):
    chain = []
    while n >= 0:
        chain.append(n)
        n = int(tree["parent"][n])
    return chain[::-1]
