"""CPU oracle, part 2: Medusa heads, static-tree verification, acceptance, KV compaction.

TEST INFRASTRUCTURE ONLY: a plain, slow, float64 numpy statement of what the
HIP library computes.  Only tests, the smoke check and the bench's
cpu_baseline leg may import it.  It shares no code with the HIP path.

What each function follows:
  medusa_heads          Section 3.1 (K parallel residual-MLP heads after the last
                        layer; head k predicts position t+k+1 from h_t)
  tree_verify_layer /   Section 3.2 "Tensorization of Tree Topology" (one forward
  tree_verify_step      pass of all T candidates under the static visibility
                        matrix) applied to a standard pre-RMSNorm / RoPE / SwiGLU
                        decoder
  accept_longest_prefix Section 3.2 "Zero-Copy Retrieval Strategy" (best path
                        chosen by the acceptance criterion, tokens gathered
                        through the [N_paths, K+1] table); the criterion is
                        greedy exact match, written as brute-force enumeration
                        of the table's rows
  kv_compact            Section 3.2 (node -> KV-cache position mapping): rows of
                        the accepted nodes become the next cache rows
  causal_decode         ordinary token-by-token decoding (Section 2.1), used to
                        pin the tree pass: a tree node's logits must equal those
                        of causal decoding along its root-to-node path

Parity pins (tests/test_oracle_*.py): tree == causal; mask == ancestors and the
closed-form node/leaf/ones counts; acceptance == an independent walk-down
formulation and exhaustive enumeration on tiny trees; compaction + chaining ==
causal decoding of the accepted tokens; the decoder maths == PyTorch CPU library
ops (scaled_dot_product_attention, rms_norm, silu) on chain trees; heads with
W1 = 0 == plain LM head; top-k == full sort.  Absolute logits of a trained 7B
model and the paper's accept-rate figures need weights that do not exist here:
parity unpinned for those.

Precision model: inputs (weights, embeddings, prefix KV) are exact values of the
storage dtype; all arithmetic is float64; K and V are rounded to the storage
dtype when written to the cache (the cache IS that dtype); nothing else is
rounded.
"""
from __future__ import annotations

import numpy as np

from . import kv8

F64 = np.float64


# ----------------------------------------------------------------------------
# storage rounding
# ----------------------------------------------------------------------------

def round_to_storage(a, dtype: str):
    """Round float64 values to the nearest (ties-to-even) bf16 / fp16 / fp32 value, returned as float64.
    fp16 is the paper's inference precision (Section 4.1): IEEE binary16, 11 significant bits, subnormals below 2**-14."""
    a = np.asarray(a, dtype=F64)
    if dtype == "fp64":                    # used only by pins that compare against float64 library ops
        return a
    if dtype == "fp32":
        return a.astype(np.float32).astype(F64)
    if dtype == "fp16":
        return a.astype(np.float16).astype(F64)
    if dtype == "bf16":
        m, e = np.frexp(a)                 # a = m * 2**e, 0.5 <= |m| < 1
        return np.ldexp(np.rint(m * 256.0), e - 8)   # 8 significant bits, rint = half-to-even
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# decoder building blocks
# ----------------------------------------------------------------------------

def rmsnorm(x, g, eps):
    x = np.asarray(x, dtype=F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, dtype=F64)


def silu(x):
    return x / (1.0 + np.exp(-x))


def rope(x, pos, base):
    """Rotate-half RoPE. x [..., n, hd] with positions pos [n]; pairs (i, i + hd/2),
    angle pos * base**(-2i/hd)."""
    x = np.asarray(x, dtype=F64)
    hd = x.shape[-1]
    half = hd // 2
    inv = base ** (-2.0 * np.arange(half, dtype=F64) / hd)
    ang = np.asarray(pos, dtype=F64)[:, None] * inv[None, :]
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def _attend(q, kc, vc, visible, head_dim):
    """q [H,n,hd]; kc,vc [Hkv,cap,hd]; visible [n, n_slots] bool over cache slots 0..n_slots-1.
    Grouped-query attention: query head h reads key/value head h // (H // Hkv) (Hkv == H: plain multi-head)."""
    n_slots = visible.shape[1]
    out = np.empty_like(q)
    scale = 1.0 / np.sqrt(float(head_dim))
    group = q.shape[0] // kc.shape[0]
    for h in range(q.shape[0]):
        hk = h // group
        sc = (q[h] @ kc[hk, :n_slots].T) * scale
        sc = np.where(visible, sc, -np.inf)
        sc = sc - sc.max(axis=1, keepdims=True)
        p = np.exp(sc)
        p = p / p.sum(axis=1, keepdims=True)
        out[h] = p @ vc[hk, :n_slots]
    return out


def _layer(x, lw, kc, vc, slots, pos, visible, cfg):
    """One pre-norm decoder layer over n rows.
    x [n,d]; kc,vc [Hkv,cap,hd] (this layer's cache, written in place at ``slots``);
    pos [n] RoPE positions; visible [n, n_slots] which cache slots each row attends.
    cfg["n_kv_heads"] (default n_heads) key/value heads: wk, wv are [Hkv*hd, d] (Table 1 of the paper: 32 query
    heads, 8 key/value heads).  cfg["kv_quant"] == "fp8e4m3": the rows are written as 8-bit codes with a scale per
    row (the KV compression the paper's Section 4.2 / 5 point to) and read back dequantised."""
    H, hd = cfg["n_heads"], cfg["head_dim"]
    Hkv = cfg.get("n_kv_heads") or H
    assert H % Hkv == 0
    n = x.shape[0]
    xn = rmsnorm(x, lw["g_attn"], cfg["rms_eps"])
    q = xn @ np.asarray(lw["wq"], dtype=F64).T
    k = xn @ np.asarray(lw["wk"], dtype=F64).T
    v = xn @ np.asarray(lw["wv"], dtype=F64).T
    q = rope(q.reshape(n, H, hd).transpose(1, 0, 2), pos, cfg["rope_base"])      # [H,n,hd]
    k = rope(k.reshape(n, Hkv, hd).transpose(1, 0, 2), pos, cfg["rope_base"])        # [Hkv,n,hd]
    v = v.reshape(n, Hkv, hd).transpose(1, 0, 2)
    if cfg.get("kv_quant") == "fp8e4m3":        # 8-bit cache rows (oracle/kv8.py states the format)
        kc[:, slots, :] = kv8.roundtrip_rows(k)
        vc[:, slots, :] = kv8.roundtrip_rows(v)
    else:
        kc[:, slots, :] = round_to_storage(k, cfg["dtype"])
        vc[:, slots, :] = round_to_storage(v, cfg["dtype"])
    att = _attend(q, kc, vc, visible, hd)                                          # [H,n,hd]
    att = att.transpose(1, 0, 2).reshape(n, H * hd)
    x = x + att @ np.asarray(lw["wo"], dtype=F64).T
    xn = rmsnorm(x, lw["g_ffn"], cfg["rms_eps"])
    gate = xn @ np.asarray(lw["wgate"], dtype=F64).T
    up = xn @ np.asarray(lw["wup"], dtype=F64).T
    x = x + (silu(gate) * up) @ np.asarray(lw["wdown"], dtype=F64).T
    return x


def tree_visibility(tree, S):
    """[T, S+T] bool: every node sees the whole prefix and its ancestors-or-self among the tree slots."""
    T = tree["T"]
    return np.concatenate([np.ones((T, S), dtype=bool), tree["mask"]], axis=1)


def tree_verify_layer(x, lw, kc, vc, S, tree, cfg):
    """Tree pass through one layer.  Node n: RoPE position S + depth[n], cache slot S + n."""
    T = tree["T"]
    slots = S + np.arange(T)
    pos = S + tree["depth"].astype(np.int64)
    return _layer(np.asarray(x, dtype=F64), lw, kc, vc, slots, pos, tree_visibility(tree, S), cfg)


def _final(x, model):
    hidden = rmsnorm(x, model["g_final"], model["cfg"]["rms_eps"])
    logits = hidden @ np.asarray(model["lm_head"], dtype=F64).T
    return hidden, logits


def argmax_lowest(a):
    """Row-wise argmax; ties -> lowest index (np.argmax returns the first maximum)."""
    return np.argmax(a, axis=-1).astype(np.int32)


def tree_verify_step(tree_tokens, model, kcache, vcache, S, tree):
    """Whole verify pass: embed the T tree tokens, run every layer under the tree mask,
    final norm, LM head, per-node argmax.
    kcache/vcache: lists (per layer) of [H,cap,hd] float64 arrays, written in place at S..S+T-1.
    Returns dict(logits [T,V], hidden [T,d], node_argmax [T])."""
    cfg = model["cfg"]
    x = np.asarray(model["embed"], dtype=F64)[np.asarray(tree_tokens, dtype=np.int64)]
    for l, lw in enumerate(model["layers"]):
        x = tree_verify_layer(x, lw, kcache[l], vcache[l], S, tree, cfg)
    hidden, logits = _final(x, model)
    return dict(logits=logits, hidden=hidden, node_argmax=argmax_lowest(logits))


def causal_decode(tokens, model, kcache, vcache, S):
    """Ordinary autoregressive decoding: feed ``tokens`` one at a time (M = 1) at positions
    S, S+1, ...; token i attends to cache slots 0..S+i.  Returns logits [len(tokens), V]
    and hidden [len(tokens), d]; the cache is extended in place."""
    cfg = model["cfg"]
    emb = np.asarray(model["embed"], dtype=F64)
    all_logits, all_hidden = [], []
    for i, tok in enumerate(tokens):
        p = S + i
        x = emb[int(tok)][None, :]
        vis = np.ones((1, p + 1), dtype=bool)
        for l, lw in enumerate(model["layers"]):
            x = _layer(x, lw, kcache[l], vcache[l], np.array([p]), np.array([p]), vis, cfg)
        hidden, logits = _final(x, model)
        all_logits.append(logits[0])
        all_hidden.append(hidden[0])
    return np.array(all_logits), np.array(all_hidden)


def empty_cache(cfg, cap):
    shape = (cfg.get("n_kv_heads") or cfg["n_heads"], cap, cfg["head_dim"])
    return ([np.zeros(shape, dtype=F64) for _ in range(cfg["n_layers"])],
            [np.zeros(shape, dtype=F64) for _ in range(cfg["n_layers"])])


# ----------------------------------------------------------------------------
# Medusa heads (Section 3.1)
# ----------------------------------------------------------------------------

def topk_lowest(logits, k):
    """Indices of the k largest entries, descending by value, ties -> lower index."""
    order = np.argsort(-np.asarray(logits, dtype=F64), kind="stable")
    return order[:k].astype(np.int32)


def medusa_heads(h, model, tree):
    """h [d]: the final-norm hidden state the base LM head reads at the current position.
    Head 0 is the base LM head (root token = its argmax).  Head k >= 1:
    z = h + SiLU(W1_k h + b1_k); logits_k = Wlm_k z; candidates = top-caps[k-1].
    Returns dict(head_logits [K+1,V], cand_flat [1+sum caps], tree_tokens [T])."""
    h = np.asarray(h, dtype=F64)
    logits = [np.asarray(model["lm_head"], dtype=F64) @ h]
    cand = [argmax_lowest(logits[0])[None]]
    for k, head in enumerate(model["medusa"]):
        pre = np.asarray(head["w1"], dtype=F64) @ h
        if head.get("b1") is not None:
            pre = pre + np.asarray(head["b1"], dtype=F64)
        z = h + silu(pre)
        lk = np.asarray(head["lm"], dtype=F64) @ z
        logits.append(lk)
        cand.append(topk_lowest(lk, tree["caps"][k]))
    cand_flat = np.concatenate(cand).astype(np.int32)
    tree_tokens = cand_flat[tree["cand_slot"]]
    return dict(head_logits=np.array(logits), cand_flat=cand_flat, tree_tokens=tree_tokens)


# ----------------------------------------------------------------------------
# Acceptance and compaction (Section 3.2, zero-copy retrieval)
# ----------------------------------------------------------------------------

def accept_longest_prefix(tree, tree_tokens, node_argmax):
    """Greedy exact-match acceptance by brute force over the retrieve table.
    A node n > 0 matches iff its token equals the model's argmax at its parent; the root always
    matches.  A path's length = number of leading matching nodes; the best path is the longest,
    ties -> lowest path index.  Returns accept_len A (1..K+1), best_path, acc_nodes [K+1] and
    acc_tokens [K+1] (-1 padded), next_root = argmax at the last accepted node, last_node."""
    retrieve, parent = tree["retrieve"], tree["parent"]
    K1 = retrieve.shape[1]
    best_len, best_p = 0, -1
    for p in range(retrieve.shape[0]):
        n_ok = 0
        for c in range(K1):
            n = retrieve[p, c]
            if n < 0:
                break
            if n != 0 and tree_tokens[n] != node_argmax[parent[n]]:
                break
            n_ok += 1
        if n_ok > best_len:
            best_len, best_p = n_ok, p
    acc_nodes = np.full(K1, -1, dtype=np.int32)
    acc_tokens = np.full(K1, -1, dtype=np.int32)
    acc_nodes[:best_len] = retrieve[best_p, :best_len]
    acc_tokens[:best_len] = np.asarray(tree_tokens)[acc_nodes[:best_len]]
    last = int(acc_nodes[best_len - 1])
    return dict(accept_len=best_len, best_path=best_p, acc_nodes=acc_nodes, acc_tokens=acc_tokens,
                next_root=int(node_argmax[last]), last_node=last)


def kv_compact(kcache, vcache, S, acc_nodes, accept_len):
    """Cache rows S..S+A-1 become the rows the accepted nodes wrote (node j's row sits at S+node_j),
    in every layer, for K and V.  Returns (kv_src_slots [K+1] with -1 padding, new length S + A)."""
    A = int(accept_len)
    src = np.full(len(acc_nodes), -1, dtype=np.int32)
    src[:A] = S + np.asarray(acc_nodes[:A])
    for c in list(kcache) + list(vcache):
        rows = c[:, src[:A], :].copy()
        c[:, S:S + A, :] = rows
    return src, S + A
