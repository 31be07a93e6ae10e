"""ctypes binding of libmedusa_hip.so: the same names as include/medusa.h, argument marshalling only.

Every computation runs inside the library's HIP kernels.  PyTorch appears here only as the owner of
device memory (``tensor.data_ptr()``) and of the current HIP stream.  If the shared library has not been
built (``python -c "import __graft_entry__ as g; g.build()"``) importing works but the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmedusa_hip.so")

MDZ_OK = 0
MDZ_BF16, MDZ_FP32, MDZ_FP16 = 0, 1, 2
MDZ_TREE_15, MDZ_TREE_64, MDZ_TREE_1, MDZ_TREE_64_K5 = 0, 1, 2, 3
MDZ_MAX_HEADS = 8
DTYPES = {"bf16": MDZ_BF16, "fp32": MDZ_FP32, "fp16": MDZ_FP16}
MDZ_KV_PLAIN, MDZ_KV_FP8E4M3 = 0, 1
KV_QUANT = {"": MDZ_KV_PLAIN, "fp8e4m3": MDZ_KV_FP8E4M3}
TREES = {"tree15": MDZ_TREE_15, "tree64": MDZ_TREE_64, "tree1": MDZ_TREE_1, "tree64k5": MDZ_TREE_64_K5}


class MedusaError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"libmedusa_hip status {status}: {msg}")
        self.status = status


class ModelDesc(C.Structure):
    _fields_ = [("d", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32),
                ("vocab", C.c_int32), ("n_layers", C.c_int32), ("dtype", C.c_int32), ("tree", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("n_kv_heads", C.c_int32),
                ("ffn_f16", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [("wqkv", C.c_void_p), ("wo", C.c_void_p), ("wgateup", C.c_void_p), ("wdown", C.c_void_p),
                ("g_attn", C.c_void_p), ("g_ffn", C.c_void_p)]


class Weights(C.Structure):
    _fields_ = [("layers", C.POINTER(LayerWeights)), ("embed", C.c_void_p), ("lm_head", C.c_void_p),
                ("g_final", C.c_void_p), ("n_medusa", C.c_int32), ("head_w1", C.POINTER(C.c_void_p)),
                ("head_b1", C.POINTER(C.c_void_p)), ("head_lm", C.POINTER(C.c_void_p))]


class KvDesc(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("n_layers", C.c_int32), ("batch", C.c_int32),
                ("n_heads", C.c_int32), ("head_dim", C.c_int32), ("cap", C.c_int32), ("dtype", C.c_int32), ("quant", C.c_int32),
                ("status", C.c_void_p)]


_lib = None

_SIGNATURES = {
    "medusa_tree_info": (C.c_int, [C.c_int] + [C.c_void_p] * 5),
    "medusa_tree_tables": (C.c_int, [C.c_int] + [C.c_void_p] * 5),
    "medusa_gemm_plan": (C.c_int, [C.c_int] * 5 + [C.c_void_p] * 4),
    "medusa_gemm_slot_count": (C.c_int, [C.c_int] * 6),
    "medusa_last_error": (C.c_char_p, []),
    "medusa_profile_begin": (C.c_int, [C.c_int]),
    "medusa_profile_end": (C.c_int, [C.c_char_p, C.c_int64]),
    "medusa_stream_read": (C.c_int, [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p]),
    "medusa_stream_read_bytes": (C.c_int64, [C.c_int64, C.c_int]),
    "medusa_stream_copy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]),
    "medusa_pack_tile_rows": (C.c_int, [C.c_int]),
    "medusa_packed_bytes": (C.c_int64, [C.c_int, C.c_int64, C.c_int64]),
    "medusa_pack_weight_bf16_as_f16": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64, C.c_int64,
                                                 C.c_int64, C.c_void_p]),
    "medusa_pack_weight": (C.c_int, [C.c_int, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64, C.c_int64,
                                     C.c_int64, C.c_void_p]),
    "medusa_kv_bytes": (C.c_int64, [C.POINTER(KvDesc)]),
    "medusa_kv_init": (C.c_int, [C.POINTER(KvDesc), C.c_void_p]),
    "medusa_test_force_unfused_rope": (C.c_int, [C.c_int]),
    "medusa_kv_write": (C.c_int, [C.POINTER(KvDesc), C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                  C.c_void_p]),
    "medusa_kv_read": (C.c_int, [C.POINTER(KvDesc), C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                 C.c_void_p]),
    "medusa_workspace_bytes": (C.c_int64, [C.POINTER(ModelDesc), C.c_int, C.c_int]),
    "medusa_heads": (C.c_int, [C.POINTER(ModelDesc), C.POINTER(Weights), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                               C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]),
    "tree_verify_layer": (C.c_int, [C.POINTER(ModelDesc), C.POINTER(LayerWeights), C.c_int, C.c_void_p,
                                    C.POINTER(KvDesc), C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int64,
                                    C.c_void_p]),
    "tree_verify_layer_static_scratch_bytes": (C.c_int64, []),
    "tree_verify_layer_static": (C.c_int, [C.POINTER(ModelDesc), C.POINTER(LayerWeights), C.c_int, C.c_void_p,
                                           C.POINTER(KvDesc), C.c_void_p, C.c_int, C.c_int, C.c_void_p]),
    "tree_verify_step": (C.c_int, [C.POINTER(ModelDesc), C.POINTER(Weights), C.c_void_p, C.POINTER(KvDesc), C.c_void_p,
                                   C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                   C.c_void_p]),
    "accept_longest_prefix": (C.c_int, [C.c_int, C.c_void_p, C.c_void_p, C.c_int] + [C.c_void_p] * 7),
    "kv_compact": (C.c_int, [C.POINTER(KvDesc), C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                             C.c_int, C.c_void_p]),
}

EXPORTED = tuple(_SIGNATURES)


def lib():
    """The loaded shared library; raises if it has not been built.  There is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MedusaError(-100, f"{LIB_PATH} is missing: build it with __graft_entry__.build()")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            f = getattr(l, name)
            f.restype, f.argtypes = res, args
        _lib = l
    return _lib


def _check(status: int):
    if status < 0:
        raise MedusaError(int(status), lib().medusa_last_error().decode("utf-8", "replace"))
    return status


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to the library must be contiguous"
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


# ---------------------------------------------------------------------------------------------
# introspection
# ---------------------------------------------------------------------------------------------

def medusa_tree_info(tree: int) -> dict:
    T, K, P, NC = (C.c_int32() for _ in range(4))
    topk = (C.c_int32 * MDZ_MAX_HEADS)()
    _check(lib().medusa_tree_info(tree, C.byref(T), C.byref(K), C.byref(P), C.byref(NC), topk))
    return dict(T=T.value, K=K.value, n_paths=P.value, n_cand=NC.value, topk=tuple(topk[:K.value]))


def medusa_gemm_plan(dtype: int, M: int, N: int, K: int, max_split: int) -> dict:
    vals = [C.c_int32() for _ in range(4)]
    _check(lib().medusa_gemm_plan(dtype, M, N, K, max_split, *[C.byref(v) for v in vals]))
    return dict(zip(("grid", "band_cols", "n_stages", "max_slots"), [v.value for v in vals]))


def medusa_gemm_slot_count(dtype: int, M: int, N: int, K: int, max_split: int, col: int) -> int:
    n = lib().medusa_gemm_slot_count(dtype, M, N, K, max_split, col)
    _check(n)
    return n


def medusa_tree_tables(tree: int) -> dict:
    info = medusa_tree_info(tree)
    T, K, P = info["T"], info["K"], info["n_paths"]
    parent = np.zeros(T, np.int32)
    depth = np.zeros(T, np.int32)
    cand_slot = np.zeros(T, np.int32)
    anc = np.zeros(T, np.uint64)
    retrieve = np.zeros((P, K + 1), np.int32)
    _check(lib().medusa_tree_tables(tree, parent.ctypes.data, depth.ctypes.data, cand_slot.ctypes.data,
                                    anc.ctypes.data, retrieve.ctypes.data))
    return dict(info, parent=parent, depth=depth, cand_slot=cand_slot, anc_mask=anc, retrieve=retrieve)


def medusa_profile_begin(max_launches: int) -> None:
    _check(lib().medusa_profile_begin(max_launches))


def medusa_profile_end() -> dict:
    """{family: dict(launches, total_us, min_us, max_us)}"""
    buf = C.create_string_buffer(4096)
    _check(lib().medusa_profile_end(buf, len(buf)))
    out = {}
    for line in buf.value.decode().splitlines():
        name, n, tot, mn, mx = line.split(",")
        out[name] = dict(launches=int(n), total_us=float(tot), min_us=float(mn), max_us=float(mx))
    return out


def medusa_stream_read(src: torch.Tensor, nbytes: int, n_workgroups: int, sink4: torch.Tensor, stream=None) -> int:
    """Enqueues the read stream over the first nbytes of src; returns the bytes actually read."""
    _check(lib().medusa_stream_read(_ptr(src), nbytes, n_workgroups, _ptr(sink4), _stream(stream)))
    return lib().medusa_stream_read_bytes(nbytes, n_workgroups)


def medusa_stream_copy(src: torch.Tensor, dst: torch.Tensor, nbytes: int, stream=None) -> None:
    _check(lib().medusa_stream_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)))


def medusa_pack_tile_rows(dtype: int) -> int:
    return _check(lib().medusa_pack_tile_rows(dtype))


def medusa_packed_bytes(dtype: int, n_rows: int, k: int) -> int:
    return _check(lib().medusa_packed_bytes(dtype, n_rows, k))


def medusa_pack_weight_bf16_as_f16(src: torch.Tensor, dst: torch.Tensor, dst_rows: int, tile_offset: int = 0,
                                   tile_stride: int = 1, stream=None) -> None:
    n_rows, k = src.shape
    _check(lib().medusa_pack_weight_bf16_as_f16(_ptr(src), n_rows, k, _ptr(dst), dst_rows, tile_offset, tile_stride,
                                                _stream(stream)))


def medusa_pack_weight(dtype: int, src: torch.Tensor, dst: torch.Tensor, dst_rows: int, tile_offset: int = 0,
                       tile_stride: int = 1, stream=None) -> None:
    n_rows, k = src.shape
    _check(lib().medusa_pack_weight(dtype, _ptr(src), n_rows, k, _ptr(dst), dst_rows, tile_offset, tile_stride,
                                    _stream(stream)))


def medusa_kv_bytes(kv: KvDesc) -> int:
    return _check(lib().medusa_kv_bytes(C.byref(kv)))


def medusa_kv_init(kv: KvDesc, stream=None) -> None:
    _check(lib().medusa_kv_init(C.byref(kv), _stream(stream)))


def medusa_test_force_unfused_rope(on: bool) -> bool:
    """Test hook (include/medusa_bench.h): returns the previous setting."""
    return bool(lib().medusa_test_force_unfused_rope(1 if on else 0))


MDZ_STATUS_SEQ_RANGE = 1


def medusa_kv_write(kv: KvDesc, layer: int, seq: int, pos0: int, n: int, k_rows, v_rows, stream=None) -> None:
    _check(lib().medusa_kv_write(C.byref(kv), layer, seq, pos0, n, _ptr(k_rows), _ptr(v_rows), _stream(stream)))


def medusa_kv_read(kv: KvDesc, layer: int, seq: int, pos0: int, n: int, k_rows, v_rows, stream=None) -> None:
    _check(lib().medusa_kv_read(C.byref(kv), layer, seq, pos0, n, _ptr(k_rows), _ptr(v_rows), _stream(stream)))


def medusa_workspace_bytes(model: ModelDesc, B: int, max_prefix: int) -> int:
    return _check(lib().medusa_workspace_bytes(C.byref(model), B, max_prefix))


# ---------------------------------------------------------------------------------------------
# the hot path
# ---------------------------------------------------------------------------------------------

def medusa_heads(model: ModelDesc, w: Weights, hidden, src_row, root_token, B: int, Tsrc: int, cand_flat, tree_tokens,
                 head_logits_opt, ws, stream=None) -> None:
    _check(lib().medusa_heads(C.byref(model), C.byref(w), _ptr(hidden), _ptr(src_row), _ptr(root_token), B, Tsrc,
                              _ptr(cand_flat), _ptr(tree_tokens), _ptr(head_logits_opt), _ptr(ws), ws.numel(),
                              _stream(stream)))


def tree_verify_layer(model: ModelDesc, lw: LayerWeights, layer: int, x_inout, kv: KvDesc, seq_len, B: int,
                      max_prefix: int, ws, stream=None) -> None:
    _check(lib().tree_verify_layer(C.byref(model), C.byref(lw), layer, _ptr(x_inout), C.byref(kv), _ptr(seq_len), B,
                                   max_prefix, _ptr(ws), ws.numel(), _stream(stream)))


def tree_verify_layer_static_scratch_bytes() -> int:
    return int(lib().tree_verify_layer_static_scratch_bytes())


def tree_verify_layer_static(model: ModelDesc, lw: LayerWeights, layer: int, x_inout, kv: KvDesc, seq_len, B: int,
                             max_prefix: int, stream=None) -> None:
    _check(lib().tree_verify_layer_static(C.byref(model), C.byref(lw), layer, _ptr(x_inout), C.byref(kv), _ptr(seq_len),
                                          B, max_prefix, _stream(stream)))


def tree_verify_step(model: ModelDesc, w: Weights, tree_tokens, kv: KvDesc, seq_len, B: int, max_prefix: int,
                     node_argmax, hidden_out, logits_opt, ws, stream=None) -> None:
    _check(lib().tree_verify_step(C.byref(model), C.byref(w), _ptr(tree_tokens), C.byref(kv), _ptr(seq_len), B,
                                  max_prefix, _ptr(node_argmax), _ptr(hidden_out), _ptr(logits_opt), _ptr(ws),
                                  ws.numel(), _stream(stream)))


def accept_longest_prefix(tree: int, tree_tokens, node_argmax, B: int, accept_len, best_path, acc_nodes, acc_tokens,
                          next_root, last_node, stream=None) -> None:
    _check(lib().accept_longest_prefix(tree, _ptr(tree_tokens), _ptr(node_argmax), B, _ptr(accept_len),
                                       _ptr(best_path), _ptr(acc_nodes), _ptr(acc_tokens), _ptr(next_root),
                                       _ptr(last_node), _stream(stream)))


def kv_compact(kv: KvDesc, tree: int, acc_nodes, accept_len, seq_len_inout, kv_src_slots, B: int, max_prefix: int,
               stream=None) -> None:
    _check(lib().kv_compact(C.byref(kv), tree, _ptr(acc_nodes), _ptr(accept_len), _ptr(seq_len_inout),
                            _ptr(kv_src_slots), B, max_prefix, _stream(stream)))
