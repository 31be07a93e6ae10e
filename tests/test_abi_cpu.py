"""CPU-only checks of the boundary: the library loads, exports every symbol the header declares, its
compiled-in tree tables equal the oracle's, and argument errors come back as status codes (no GPU work)."""
import os
import re

import numpy as np
import pytest

import workload as W
import paper_2603_03383_amd as P
from oracle import tree as OT

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(P.LIB_PATH):
        import __graft_entry__ as g
        g.build()


def test_header_symbols_are_exported():
    def declared_in(name):
        text = open(os.path.join(ROOT, "include", name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        return set(re.findall(r"\b(?:int|int64_t|const char\*)\s+(\w+)\s*\(", text))
    hot, bench = declared_in("medusa.h"), declared_in("medusa_bench.h")
    assert {"medusa_heads", "tree_verify_layer", "tree_verify_step", "accept_longest_prefix", "kv_compact"} <= hot
    # benchmark / test entry points live in the second header only
    assert not any(n.startswith(("medusa_profile", "medusa_stream", "medusa_gemm", "medusa_test")) for n in hot)
    declared = hot | bench
    assert declared == set(P.EXPORTED)
    lib = P.lib()
    for name in declared:
        assert hasattr(lib, name), name


@pytest.mark.parametrize("spec,tid", [(W.TREE15, P.MDZ_TREE_15), (W.TREE64, P.MDZ_TREE_64), (W.TREE1, P.MDZ_TREE_1),
                                      (W.TREE64K5, P.MDZ_TREE_64_K5)],
                         ids=["tree15", "tree64", "tree1", "tree64k5"])
def test_compiled_tables_equal_oracle_tree(spec, tid):
    t = P.medusa_tree_tables(tid)
    o = OT.build_tree(spec.caps, spec.budgets)
    assert (t["T"], t["K"], t["n_paths"], t["n_cand"], t["topk"]) == (o["T"], o["K"], len(o["retrieve"]), o["n_cand"], o["caps"])
    assert np.array_equal(t["parent"], o["parent"])
    assert np.array_equal(t["depth"], o["depth"])
    assert np.array_equal(t["cand_slot"], o["cand_slot"])
    assert np.array_equal(t["retrieve"], o["retrieve"])
    bits = (t["anc_mask"][:, None] >> np.arange(o["T"], dtype=np.uint64)[None, :]) & np.uint64(1)
    assert np.array_equal(bits.astype(bool), o["mask"])


def test_argument_errors_are_status_codes():
    m = P.ModelDesc(256, 4, 64, 688, 1024, 2, P.MDZ_FP32, P.MDZ_TREE_15, 1e-5, 1e4)
    assert P.medusa_workspace_bytes(m, 1, 64) > 0
    for field, bad in [("d", 255), ("dtype", 7), ("tree", 9), ("ffn", 690), ("head_dim", 0)]:
        mm = P.ModelDesc.from_buffer_copy(m)
        setattr(mm, field, bad)
        with pytest.raises(P.MedusaError) as e:
            P.medusa_workspace_bytes(mm, 1, 64)
        assert e.value.status in (-1, -2)
    # binary16 feed-forward operands are an option of bf16 models only
    ok = P.ModelDesc(256, 4, 64, 704, 1024, 2, P.MDZ_BF16, P.MDZ_TREE_15, 1e-5, 1e4, 0, 1)
    assert P.medusa_workspace_bytes(ok, 1, 64) > 0
    for dtype, flag in [(P.MDZ_FP32, 1), (P.MDZ_FP16, 1), (P.MDZ_BF16, 2)]:
        bad = P.ModelDesc(256, 4, 64, 704, 1024, 2, dtype, P.MDZ_TREE_15, 1e-5, 1e4, 0, flag)
        with pytest.raises(P.MedusaError) as e:
            P.medusa_workspace_bytes(bad, 1, 64)
        assert e.value.status == -1 and "ffn_f16" in str(e.value)
    with pytest.raises(P.MedusaError):
        P.medusa_tree_info(5)
    with pytest.raises(P.MedusaError):
        P.medusa_packed_bytes(P.MDZ_BF16, 0, 16)
    kv = P.KvDesc(None, None, 2, 1, 4, 64, 128, P.MDZ_FP32, 0, None)
    assert P.medusa_kv_bytes(kv) == 2 * 4 * 128 * 64 * 4
    lib = P.lib()
    # NULL buffers: rejected before anything is enqueued (safe without a GPU)
    assert lib.accept_longest_prefix(0, None, None, 1, None, None, None, None, None, None, None) == -1
    assert lib.kv_compact(kv, 0, None, None, None, None, 1, 10, None) == -1
    assert b"NULL" in lib.medusa_last_error()
    assert lib.medusa_pack_weight_bf16_as_f16(None, 32, 128, None, 32, 0, 1, None) == -1
    assert lib.medusa_pack_weight(P.MDZ_BF16, None, 32, 128, None, 32, 0, 1, None) == -1
    assert P.medusa_packed_bytes(P.MDZ_BF16, 4096, 4096) == 4096 * 4096 * 2
    assert P.medusa_pack_tile_rows(P.MDZ_BF16) == 32 and P.medusa_pack_tile_rows(P.MDZ_FP32) == 16
    # fp16 shares the 16-bit layouts
    assert P.medusa_pack_tile_rows(P.MDZ_FP16) == 32 and P.medusa_packed_bytes(P.MDZ_FP16, 4096, 4096) == 4096 * 4096 * 2
    with pytest.raises(P.MedusaError):
        P.medusa_pack_tile_rows(3)
