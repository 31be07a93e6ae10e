"""Holders for device memory around the C-ABI calls: packed model weights, KV cache, per-step buffers.

No arithmetic of the method lives here: tensors are allocated with torch, handed to the library's pack /
KV-write kernels, and their pointers are stored in the ctypes structs the entry points take.
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

import torch

from . import binding as B


def torch_dtype(dtype: int):
    return {B.MDZ_BF16: torch.bfloat16, B.MDZ_FP16: torch.float16, B.MDZ_FP32: torch.float32}[dtype]


class DeviceModel:
    """Packed weights of one decoder (+ Medusa heads) on one GPU."""

    def __init__(self, *, d, n_heads, head_dim, ffn, vocab, n_layers, dtype: str, tree: str, n_kv_heads: int = 0, rms_eps=1e-5,
                 rope_base=10000.0, device="cuda:0", ffn_f16: bool = False):
        self.desc = B.ModelDesc(d, n_heads, head_dim, ffn, vocab, n_layers, B.DTYPES[dtype], B.TREES[tree], rms_eps,
                                rope_base, n_kv_heads, int(ffn_f16))
        self.ffn_f16 = bool(ffn_f16)
        self.kv_heads = n_kv_heads or n_heads
        self.device = torch.device(device)
        self.dtype = B.DTYPES[dtype]
        self.tdtype = torch_dtype(self.dtype)
        self.tree = B.TREES[tree]
        self.tree_info = B.medusa_tree_info(self.tree)
        self.R = B.medusa_pack_tile_rows(self.dtype)
        self._keep: List[torch.Tensor] = []
        self._layers: List[B.LayerWeights] = []
        self._heads = []
        self.embed = self.lm_head = self.g_final = None
        self.weights: Optional[B.Weights] = None
        self.packed_bytes = 0

    # -- packing helpers -------------------------------------------------------------------------
    def _alloc_packed(self, n_rows, k) -> torch.Tensor:
        nbytes = B.medusa_packed_bytes(self.dtype, n_rows, k)
        t = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self._keep.append(t)
        self.packed_bytes += nbytes
        return t

    def _dev(self, t: torch.Tensor) -> torch.Tensor:
        return t.to(self.device, self.tdtype).contiguous()

    def pack(self, mats: Sequence[torch.Tensor], interleave: bool = False, as_f16: bool = False) -> torch.Tensor:
        """Stacks (or tile-interleaves) row-major [n_i, k] matrices into one packed matrix.  as_f16: a bf16 model's
        feed-forward matrices, stored as binary16."""
        pack_one = (lambda _dt, *a: B.medusa_pack_weight_bf16_as_f16(*a)) if as_f16 else B.medusa_pack_weight
        k = mats[0].shape[1]
        total = sum(m.shape[0] for m in mats)
        dst = self._alloc_packed(total, k)
        off = 0
        for i, m in enumerate(mats):
            m = self._dev(m)
            if interleave:
                pack_one(self.dtype, m, dst, total, i, len(mats))
            else:
                pack_one(self.dtype, m, dst, total, off // self.R, 1)
                off += m.shape[0]
        torch.cuda.synchronize(self.device)          # the row-major sources may be freed by the caller now
        return dst

    def _gain(self, g) -> torch.Tensor:
        g = self._dev(g)
        self._keep.append(g)
        return g

    # -- model assembly --------------------------------------------------------------------------
    def add_layer(self, wq, wk, wv, wo, wgate, wup, wdown, g_attn, g_ffn) -> None:
        lw = B.LayerWeights(self.pack([wq, wk, wv]).data_ptr(), self.pack([wo]).data_ptr(),
                            self.pack([wgate, wup], interleave=True, as_f16=self.ffn_f16).data_ptr(),
                            self.pack([wdown], as_f16=self.ffn_f16).data_ptr(),
                            self._gain(g_attn).data_ptr(), self._gain(g_ffn).data_ptr())
        self._layers.append(lw)

    def set_embed(self, e) -> None:
        self.embed = self._dev(e)

    def set_lm_head(self, w) -> None:
        self.lm_head = self.pack([w])

    def set_final_gain(self, g) -> None:
        self.g_final = self._gain(g)

    def add_medusa_head(self, w1, b1, lm) -> None:
        self._heads.append((self.pack([w1]), None if b1 is None else self._gain(b1), self.pack([lm])))

    def _stack_head_w1(self) -> None:
        """Moves the heads' packed first-layer matrices into one allocation, back to back: the library then runs them
        as a single launch (memory plumbing only: byte copies of what medusa_pack_weight wrote)."""
        if len(self._heads) < 2 or len({h[0].numel() for h in self._heads}) != 1:
            return
        n = self._heads[0][0].numel()
        both = torch.empty(n * len(self._heads), dtype=torch.uint8, device=self.device)
        for k, (w1, b1, lm) in enumerate(self._heads):
            both[k * n:(k + 1) * n].copy_(w1)
            self._keep = [t for t in self._keep if t is not w1]
            self._heads[k] = (both[k * n:(k + 1) * n], b1, lm)
        self._keep.append(both)
        torch.cuda.synchronize(self.device)

    def finalize(self) -> "DeviceModel":
        self._stack_head_w1()
        n = len(self._layers)
        self._layer_arr = (B.LayerWeights * max(n, 1))(*self._layers)
        nh = len(self._heads)
        self._w1 = (C.c_void_p * max(nh, 1))(*[h[0].data_ptr() for h in self._heads])
        self._lm = (C.c_void_p * max(nh, 1))(*[h[2].data_ptr() for h in self._heads])
        has_bias = any(h[1] is not None for h in self._heads)
        self._b1 = (C.c_void_p * max(nh, 1))(*[None if h[1] is None else h[1].data_ptr() for h in self._heads])
        self.weights = B.Weights(
            C.cast(self._layer_arr, C.POINTER(B.LayerWeights)),
            None if self.embed is None else self.embed.data_ptr(),
            None if self.lm_head is None else self.lm_head.data_ptr(),
            None if self.g_final is None else self.g_final.data_ptr(),
            nh, C.cast(self._w1, C.POINTER(C.c_void_p)),
            C.cast(self._b1, C.POINTER(C.c_void_p)) if has_bias else None,
            C.cast(self._lm, C.POINTER(C.c_void_p)))
        return self

    def view_with_tree(self, tree: str) -> "DeviceModel":
        """A second model over the SAME packed weights with another static tree (e.g. "tree1": the autoregressive
        baseline).  Medusa heads are kept only if the tree's depth matches their number."""
        import copy
        other = copy.copy(self)
        d = self.desc
        other.desc = B.ModelDesc(d.d, d.n_heads, d.head_dim, d.ffn, d.vocab, d.n_layers, d.dtype, B.TREES[tree],
                                 d.rms_eps, d.rope_base, d.n_kv_heads, d.ffn_f16)
        other.tree = B.TREES[tree]
        other.tree_info = B.medusa_tree_info(other.tree)
        keep = len(self._heads) if other.tree_info["K"] == len(self._heads) else 0
        w = self.weights
        other.weights = B.Weights(w.layers, w.embed, w.lm_head, w.g_final, keep, w.head_w1, w.head_b1, w.head_lm)
        return other

    def layer(self, l: int) -> B.LayerWeights:
        return self._layers[l]

    def workspace(self, batch: int, max_prefix: int) -> torch.Tensor:
        n = B.medusa_workspace_bytes(self.desc, batch, max_prefix)
        return torch.empty(n, dtype=torch.uint8, device=self.device)


class DeviceKV:
    """KV cache in the library's own layout.  quant="fp8e4m3": 8-bit rows (E4M3 codes + one fp32 scale per row)."""

    def __init__(self, model: DeviceModel, batch: int, cap: int, n_layers: Optional[int] = None, quant: str = ""):
        d = model.desc
        self.model = model
        self.desc = B.KvDesc(None, None, n_layers or d.n_layers, batch, model.kv_heads, d.head_dim, cap, model.dtype,
                             B.KV_QUANT[quant], None)
        nbytes = B.medusa_kv_bytes(self.desc)
        self.k = torch.empty(nbytes, dtype=torch.uint8, device=model.device)
        self.v = torch.empty(nbytes, dtype=torch.uint8, device=model.device)
        self.status = torch.empty(1, dtype=torch.int32, device=model.device)
        self.desc.k, self.desc.v, self.desc.status = self.k.data_ptr(), self.v.data_ptr(), self.status.data_ptr()
        self.bytes = 2 * nbytes
        B.medusa_kv_init(self.desc)                 # the library zero-fills its own layout (and the status word)

    def check_status(self) -> None:
        """Synchronises and raises if a kernel had to clamp a sequence length (see MDZ_STATUS_SEQ_RANGE)."""
        st = int(self.status.item())
        if st & B.MDZ_STATUS_SEQ_RANGE:
            raise B.MedusaError(-2, "a sequence length outside [0, max_prefix] reached the kernels and was clamped")

    def write(self, layer: int, seq: int, pos0: int, k_rows: torch.Tensor, v_rows: torch.Tensor) -> None:
        """k_rows, v_rows: [key/value heads, n, head_dim] storage dtype."""
        k_rows = k_rows.to(self.model.device, self.model.tdtype).contiguous()
        v_rows = v_rows.to(self.model.device, self.model.tdtype).contiguous()
        B.medusa_kv_write(self.desc, layer, seq, pos0, k_rows.shape[1], k_rows, v_rows)
        torch.cuda.synchronize(self.model.device)

    def read(self, layer: int, seq: int, pos0: int, n: int):
        d = self.desc
        k = torch.empty(d.n_heads, n, d.head_dim, dtype=self.model.tdtype, device=self.model.device)
        v = torch.empty_like(k)
        B.medusa_kv_read(self.desc, layer, seq, pos0, n, k, v)
        return k, v


class StepBuffers:
    """Device outputs of one heads -> verify -> accept -> compact step for a batch."""

    def __init__(self, model: DeviceModel, batch: int, max_prefix: int, want_logits: bool = False,
                 want_head_logits: bool = False):
        dev, ti, d = model.device, model.tree_info, model.desc
        T, K = ti["T"], ti["K"]
        i32 = dict(dtype=torch.int32, device=dev)
        self.batch, self.max_prefix = batch, max_prefix
        self.ws = model.workspace(batch, max_prefix)
        self.cand_flat = torch.zeros(batch, ti["n_cand"], **i32)
        self.tree_tokens = torch.zeros(batch, T, **i32)
        self.node_argmax = torch.zeros(batch, T, **i32)
        self.hidden = torch.zeros(batch, T, d.d, dtype=model.tdtype, device=dev)
        self.logits = torch.zeros(batch, T, d.vocab, dtype=torch.float32, device=dev) if want_logits else None
        self.head_logits = (torch.zeros(batch, K + 1, d.vocab, dtype=torch.float32, device=dev)
                            if want_head_logits else None)
        self.accept_len = torch.zeros(batch, **i32)
        self.best_path = torch.zeros(batch, **i32)
        self.acc_nodes = torch.zeros(batch, K + 1, **i32)
        self.acc_tokens = torch.zeros(batch, K + 1, **i32)
        self.next_root = torch.zeros(batch, **i32)
        self.last_node = torch.zeros(batch, **i32)
        self.kv_src_slots = torch.zeros(batch, K + 1, **i32)


def run_step(model: DeviceModel, kv: DeviceKV, buf: StepBuffers, hidden, src_row, root_token, seq_len,
             with_heads: bool = True, stream=None) -> None:
    """Enqueues heads -> verify -> accept -> compact (the four C-ABI calls, nothing else)."""
    Bn = buf.batch
    if with_heads:
        B.medusa_heads(model.desc, model.weights, hidden, src_row, root_token, Bn, hidden.shape[1], buf.cand_flat,
                       buf.tree_tokens, buf.head_logits, buf.ws, stream)
    B.tree_verify_step(model.desc, model.weights, buf.tree_tokens, kv.desc, seq_len, Bn, buf.max_prefix,
                       buf.node_argmax, buf.hidden, buf.logits, buf.ws, stream)
    B.accept_longest_prefix(model.tree, buf.tree_tokens, buf.node_argmax, Bn, buf.accept_len, buf.best_path,
                            buf.acc_nodes, buf.acc_tokens, buf.next_root, buf.last_node, stream)
    B.kv_compact(kv.desc, model.tree, buf.acc_nodes, buf.accept_len, seq_len, buf.kv_src_slots, Bn, buf.max_prefix,
                 stream)


class ChainedDecoder:
    """Speculative steps enqueued back to back with no host round trip (the paper's static-shape, device-resident
    decode loop, Section 3.2): step i's heads read step i-1's hidden state at `last_node`, its root is step i-1's
    `next_root`, and the sequence lengths live on the device.  With ``use_graph`` one step is captured in a HIP graph
    and replayed.  Only argument marshalling and buffer bookkeeping happen here; every step of the method runs in the
    library's kernels."""

    def __init__(self, model: DeviceModel, kv: DeviceKV, batch: int, max_prefix: int, use_graph: bool = True):
        self.model, self.kv, self.batch = model, kv, batch
        self.buf = StepBuffers(model, batch, max_prefix)
        self.seq_len = torch.zeros(batch, dtype=torch.int32, device=model.device)
        self.use_graph = use_graph
        self._graph = None

    def prime(self, hidden0: torch.Tensor, root0: torch.Tensor, seq_len: torch.Tensor) -> None:
        """hidden0 [B, d]: the hidden state the base model produced for the last prefix token; root0 [B]: its
        greedy next token; seq_len [B]: prefix lengths."""
        b = self.buf
        b.hidden.zero_()
        b.hidden[:, 0, :].copy_(hidden0)
        b.last_node.zero_()
        b.next_root.copy_(root0)
        self.seq_len.copy_(seq_len)

    def _step(self) -> None:
        b = self.buf
        run_step(self.model, self.kv, b, b.hidden, b.last_node, b.next_root, self.seq_len)

    def _capture(self) -> None:
        b = self.buf
        saved = [t.clone() for t in (b.hidden, b.last_node, b.next_root, self.seq_len)]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self._step()                                   # warm-up outside the capture (one-time kernel attributes)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for t, s in zip((b.hidden, b.last_node, b.next_root, self.seq_len), saved):
            t.copy_(s)
        torch.cuda.synchronize()
        self._graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self._graph, stream=side):
            self._step()
        for t, s in zip((b.hidden, b.last_node, b.next_root, self.seq_len), saved):
            t.copy_(s)                                     # capture does not run the kernels; restore anyway

    def run(self, n_steps: int):
        """Enqueues n_steps steps; returns device tensors (tokens [n_steps, B, K+1] with -1 padding,
        accept_len [n_steps, B]).  The caller synchronises when it wants to read them."""
        b = self.buf
        K1 = b.acc_tokens.shape[1]
        tokens = torch.empty(n_steps, self.batch, K1, dtype=torch.int32, device=self.model.device)
        lens = torch.empty(n_steps, self.batch, dtype=torch.int32, device=self.model.device)
        if self.use_graph and self._graph is None:
            self._capture()
        for i in range(n_steps):
            if self._graph is not None:
                self._graph.replay()
            else:
                self._step()
            tokens[i].copy_(b.acc_tokens)
            lens[i].copy_(b.accept_len)
        return tokens, lens

    def check_status(self) -> None:
        """After the caller has synchronised: raises if any step ran with a length beyond max_prefix."""
        self.kv.check_status()
