"""Seeded synthetic inputs for the Medusa static-tree verify path.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests/bench.  It holds NONE of the method's arithmetic: only a
counter-based random generator, the workload shapes, and helpers that name
tensors.  Everything is pure integer arithmetic followed by correctly rounded
float32 multiplications, so a tensor generated on the CPU and the same tensor
generated on the GPU agree bit for bit.

Generator
---------
element i of tensor ``name`` under ``seed``:
    key   = mix64(seed * GOLDEN + fnv1a64(name))
    h_j   = mix64(key + (4*i + j) * GOLDEN)            j = 0..3   (splitmix64 finaliser)
    s     = sum of the sixteen 16-bit fields of h_0..h_3          (Irwin-Hall, n = 16)
    z     = float32(s - 8*65535) * float32(1/sqrt(16*(65536^2-1)/12))
z has mean 0, variance 1 and is bell shaped (a 16-fold uniform sum; support
+-6.9 sigma, excess kurtosis -0.075).  It stands in for N(0,1) wherever the
workload recipe says "normal".  Values are then scaled by ``std`` in float32
and rounded (nearest-even) to the storage dtype.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, Tuple

import torch

BASE_SEED = 20260303

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(u: int) -> int:
    """Unsigned 64-bit value -> the int64 with the same bit pattern."""
    u &= _M64
    return u - (1 << 64) if u >= (1 << 63) else u


def fnv1a64(name: str) -> int:
    h = 0xCBF29CE484222325
    for b in name.encode("utf-8"):
        h ^= b
        h = (h * 0x100000001B3) & _M64
    return h


def _mix64_int(x: int) -> int:
    x &= _M64
    x ^= x >> 30
    x = (x * _C1) & _M64
    x ^= x >> 27
    x = (x * _C2) & _M64
    x ^= x >> 31
    return x


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    x = x ^ _lsr(x, 30)
    x = x * _s64(_C1)
    x = x ^ _lsr(x, 27)
    x = x * _s64(_C2)
    x = x ^ _lsr(x, 31)
    return x


def tensor_key(seed: int, name: str) -> int:
    return _mix64_int((seed * _GOLDEN + fnv1a64(name)) & _M64)


def _hash_block(key: int, start: int, count: int, lanes: int, device) -> torch.Tensor:
    """int64 tensor [count, lanes]: hash of counters (start+i)*lanes + j."""
    i = torch.arange(start, start + count, dtype=torch.int64, device=device)
    ctr = (i * lanes).unsqueeze(1) + torch.arange(lanes, dtype=torch.int64, device=device)
    return _mix64(ctr * _s64(_GOLDEN) + _s64(key))


_IH_SCALE = 1.0 / math.sqrt(16.0 * (65536.0 ** 2 - 1.0) / 12.0)


def _normal_block(key: int, start: int, count: int, device) -> torch.Tensor:
    h = _hash_block(key, start, count, 4, device)
    s = (h & 0xFFFF) + (_lsr(h, 16) & 0xFFFF) + (_lsr(h, 32) & 0xFFFF) + _lsr(h, 48)
    s = s.sum(dim=1) - 8 * 65535
    return s.to(torch.float32) * torch.tensor(_IH_SCALE, dtype=torch.float32, device=device)


def normal(seed: int, name: str, shape, std: float = 1.0, dtype=torch.float32,
           device="cpu") -> torch.Tensor:
    """Bell-shaped (Irwin-Hall 16) zero-mean values with the given std."""
    n = 1
    for s in shape:
        n *= int(s)
    key = tensor_key(seed, name)
    out = torch.empty(n, dtype=dtype, device=device)
    chunk = 1 << (25 if torch.device(device).type == "cuda" else 22)
    sc = torch.tensor(std, dtype=torch.float32, device=device)
    for a in range(0, n, chunk):
        c = min(chunk, n - a)
        z = _normal_block(key, a, c, device)
        if std != 1.0:
            z = z * sc
        out[a:a + c] = z.to(dtype)
    return out.view(*shape)


def uniform_int(seed: int, name: str, shape, lo: int, hi: int, device="cpu") -> torch.Tensor:
    """Uniform integers in [lo, hi) as int32 (modulo reduction of a 63-bit hash)."""
    n = 1
    for s in shape:
        n *= int(s)
    key = tensor_key(seed, name)
    h = _hash_block(key, 0, n, 1, device).view(-1)
    v = (_lsr(h, 1) % (hi - lo)) + lo
    return v.to(torch.int32).view(*shape)


# ---------------------------------------------------------------------------
# Workload shapes
# ---------------------------------------------------------------------------

@dataclass(frozen=True)
class TreeSpec:
    """A static candidate tree: node = rank tuple (r_1..r_m), r_i < caps[i], kept
    iff prod(r_i + 1) <= budgets[m-1].  Only the rule's parameters live here; the
    oracle and the HIP library each build their own tables from them."""
    name: str
    caps: Tuple[int, ...]
    budgets: Tuple[int, ...]
    n_nodes: int
    n_paths: int


TREE15 = TreeSpec("tree15", (2, 2, 2), (2, 4, 8), 15, 8)
TREE64 = TreeSpec("tree64", (10, 10, 4, 4), (10, 12, 4, 3), 64, 38)
TREE64K5 = TreeSpec("tree64k5", (9, 10, 4, 3, 2), (9, 10, 4, 3, 2), 64, 34)   # five heads, still 64 nodes
TREE1 = TreeSpec("tree1", (), (), 1, 1)   # the root alone: one autoregressive decode step


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                 # "bf16" | "fp16" | "fp32": storage type of weights, KV cache, activations at the boundary
    n_layers: int
    d: int
    n_heads: int
    head_dim: int
    ffn: int
    vocab: int
    tree: TreeSpec
    prefix: Tuple[int, ...]    # prefix length per sequence (len == batch)
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    weight_std: float = 0.02
    seed: int = BASE_SEED
    n_kv_heads: int = 0        # key/value heads (grouped-query attention); 0 = n_heads (plain multi-head attention)
    kv_quant: str = ""         # "" | "fp8e4m3": cache rows stored as 8-bit codes with one fp32 scale per row
    gain_std: float = 0.3      # RMSNorm gains are 1 + gain_std * z (0: all ones)
    head_bias_std: float = 0.0  # Medusa-head bias b1 ~ head_bias_std * z (0: the heads have no bias)
    ffn_f16: bool = False      # device-side option of a bf16 model (binary16 feed-forward operands); changes no input

    @property
    def kv_heads(self) -> int:
        return self.n_kv_heads or self.n_heads

    @property
    def batch(self) -> int:
        return len(self.prefix)

    @property
    def n_medusa(self) -> int:
        return len(self.tree.caps)

    @property
    def topk(self) -> Tuple[int, ...]:
        return self.tree.caps

    @property
    def torch_dtype(self):
        return {"bf16": torch.bfloat16, "fp16": torch.float16, "fp32": torch.float32}[self.dtype]

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


def _ragged_prefixes(seed: int, batch: int, lo: int, hi: int) -> Tuple[int, ...]:
    return tuple(int(v) for v in uniform_int(seed, "cfg5.prefix_len", (batch,), lo, hi + 1))


def _b7(name, n_layers, prefix) -> Workload:
    return Workload(name=name, dtype="bf16", n_layers=n_layers, d=4096, n_heads=32, head_dim=128,
                    ffn=11008, vocab=128000, tree=TREE64, prefix=tuple(prefix))


CONFIGS: Dict[str, Workload] = {
    # 1: tiny fp32 model, 15-node tree, prefix of 64 tokens produced by a causal prefill
    "cfg1_tiny_fp32": Workload(name="cfg1_tiny_fp32", dtype="fp32", n_layers=2, d=256, n_heads=4,
                               head_dim=64, ffn=688, vocab=1024, tree=TREE15, prefix=(64,)),
    # 2: one 7B-class decoder layer, bf16, prefix 512
    "cfg2_layer_bf16": _b7("cfg2_layer_bf16", 1, (512,)),
    # 3: full 32-layer 7B-class step, prefix 1024
    "cfg3_step_1k": _b7("cfg3_step_1k", 32, (1024,)),
    # 4: long prefixes
    "cfg4_step_4k": _b7("cfg4_step_4k", 32, (4096,)),
    "cfg4_step_8k": _b7("cfg4_step_8k", 32, (8192,)),
    "cfg4_step_16k": _b7("cfg4_step_16k", 32, (16384,)),
    # 5: 16 ragged sequences, prefix ~ UniformInt[256, 4096]
    "cfg5_ragged_b16": _b7("cfg5_ragged_b16", 32, _ragged_prefixes(BASE_SEED, 16, 256, 4096)),
    # the paper's own model shape where its Table 1 is readable: 34 layers, 32 query / 8 key-value heads, vocabulary
    # ~153k (153,600 here: a multiple of 128); its "hidden size 12,800" cannot be the model width of a 7B model and is
    # read as the FFN width; d = 4096 and head_dim = 128 as in the other configs; fp16 as in its Section 4.1;
    # five Medusa heads (its Table 2) on a 64-node tree of depth 5
    "next3_paper_shape_1k": Workload(name="next3_paper_shape_1k", dtype="fp16", n_layers=34, d=4096, n_heads=32,
                                     head_dim=128, ffn=12800, vocab=153600, tree=TREE64K5, prefix=(1024,), n_kv_heads=8),
}


# ---------------------------------------------------------------------------
# Named tensors of a workload.  Weights are [out_features, in_features] row-major.
# ---------------------------------------------------------------------------

LAYER_MATS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


def layer_shapes(w: Workload) -> Dict[str, Tuple[int, int]]:
    kvd = w.kv_heads * w.head_dim
    return {"wq": (w.d, w.d), "wk": (kvd, w.d), "wv": (kvd, w.d), "wo": (w.d, w.d),
            "wgate": (w.ffn, w.d), "wup": (w.ffn, w.d), "wdown": (w.d, w.ffn)}


def layer_weight(w: Workload, layer: int, mat: str, device="cpu") -> torch.Tensor:
    return normal(w.seed, f"layer{layer}.{mat}", layer_shapes(w)[mat], w.weight_std, w.torch_dtype, device)


def norm_gain(w: Workload, name: str, device="cpu") -> torch.Tensor:
    """RMSNorm gains [d]: 1 + gain_std * z, seeded per gain vector (``name`` = "layer3.g_attn", "g_final", ...),
    rounded to the storage dtype; all ones when gain_std is 0."""
    if w.gain_std == 0.0:
        return torch.ones(w.d, dtype=w.torch_dtype, device=device)
    z = normal(w.seed, f"gain.{name}", (w.d,), w.gain_std, torch.float32, device)
    return (z + 1.0).to(w.torch_dtype)


def embedding(w: Workload, device="cpu") -> torch.Tensor:
    # std 1 so that the residual stream has unit scale like the other configs' inputs
    return normal(w.seed, "embed", (w.vocab, w.d), 1.0, w.torch_dtype, device)


def lm_head(w: Workload, device="cpu") -> torch.Tensor:
    return normal(w.seed, "lm_head", (w.vocab, w.d), w.weight_std, w.torch_dtype, device)


def medusa_w1(w: Workload, k: int, device="cpu") -> torch.Tensor:
    return normal(w.seed, f"medusa{k}.w1", (w.d, w.d), w.weight_std, w.torch_dtype, device)


def medusa_b1(w: Workload, k: int, device="cpu"):
    """Bias [d] of Medusa head k's residual block, or None when the workload's heads have none."""
    if w.head_bias_std == 0.0:
        return None
    return normal(w.seed, f"medusa{k}.b1", (w.d,), w.head_bias_std, w.torch_dtype, device)


def medusa_lm(w: Workload, k: int, device="cpu") -> torch.Tensor:
    return normal(w.seed, f"medusa{k}.lm", (w.vocab, w.d), w.weight_std, w.torch_dtype, device)


def prefix_kv(w: Workload, layer: int, seq: int, device="cpu"):
    """Random prefix K and V, each [kv_heads, S, head_dim], N(0,1)-like, storage dtype."""
    S = w.prefix[seq]
    shape = (w.kv_heads, S, w.head_dim)
    k = normal(w.seed, f"kv.k.l{layer}.s{seq}", shape, 1.0, w.torch_dtype, device)
    v = normal(w.seed, f"kv.v.l{layer}.s{seq}", shape, 1.0, w.torch_dtype, device)
    return k, v


def hidden_state(w: Workload, name: str, rows: int, device="cpu") -> torch.Tensor:
    """[rows, d] unit-variance activations (layer input x, or the hidden the Medusa heads read)."""
    return normal(w.seed, f"hidden.{name}", (rows, w.d), 1.0, w.torch_dtype, device)


def random_tokens(w: Workload, name: str, shape, device="cpu") -> torch.Tensor:
    return uniform_int(w.seed, f"tokens.{name}", shape, 0, w.vocab, device)
