"""CPU tests of the weight-streaming GEMM's host-side work decomposition (no GPU work): the slot counts the
consumers compute by arithmetic must equal a brute-force walk over the workgroups' unit ranges."""
import pytest

import paper_2603_03383_amd as P

SHAPES = [
    # (M, N, K): the 7B layer matrices, the LM head, head W1, tiny shapes and ragged unit counts
    (64, 12288, 4096), (64, 4096, 4096), (64, 22016, 4096), (64, 4096, 11008), (64, 128000, 4096),
    (1, 4096, 4096), (1, 128000, 4096), (16, 4096, 4096), (32, 12288, 4096),
    (64, 256, 256), (15, 768, 256), (64, 1408, 256), (64, 96, 128), (7, 32, 128), (64, 32, 11008), (64, 4128, 384),
]


def brute_force_writers(n, band_cols, n_stages, grid):
    """For every band: which ranges [floor(w*U/G), floor((w+1)*U/G)) hold at least one of its units."""
    bands = (n + band_cols - 1) // band_cols
    U = bands * n_stages
    owner = [None] * U
    for w in range(grid):
        lo, hi = w * U // grid, (w + 1) * U // grid
        assert hi > lo, "an empty range would idle a workgroup"
        for u in range(lo, hi):
            assert owner[u] is None
            owner[u] = w
    assert all(o is not None for o in owner)
    return [sorted(set(owner[b * n_stages:(b + 1) * n_stages])) for b in range(bands)]


@pytest.mark.parametrize("M,N,K", SHAPES)
@pytest.mark.parametrize("max_split", [1, 2, 8, 12])
def test_slot_counts_equal_a_walk_over_the_ranges(M, N, K, max_split):
    plan = P.medusa_gemm_plan(P.MDZ_BF16, M, N, K, max_split)
    assert 1 <= plan["grid"] <= 256 and K % plan["n_stages"] == 0 and plan["band_cols"] % 32 == 0
    bands = (N + plan["band_cols"] - 1) // plan["band_cols"]
    if max_split == 1:                                     # whole bands: one slot everywhere, bands dealt evenly
        assert plan["max_slots"] == 1 and plan["grid"] <= bands
        for col in (0, N // 2, N - 1):
            assert P.medusa_gemm_slot_count(P.MDZ_BF16, M, N, K, max_split, col) == 1
        return
    writers = brute_force_writers(N, plan["band_cols"], plan["n_stages"], plan["grid"])
    most = 0
    for b, ws in enumerate(writers):
        assert ws == list(range(ws[0], ws[0] + len(ws))), "the writers of a band are consecutive ranges (slot = rank)"
        for col in {b * plan["band_cols"], min(N - 1, (b + 1) * plan["band_cols"] - 1)}:
            assert P.medusa_gemm_slot_count(P.MDZ_BF16, M, N, K, max_split, col) == len(ws)
        most = max(most, len(ws))
    assert most == plan["max_slots"] <= max_split


def test_7b_shapes_keep_the_cus_busy_and_smaller_grids_are_band_aligned():
    """One workgroup per CU, or at least three quarters of that when the equal ranges then line up with the bands."""
    expect = {(12288, 4096): 192, (4096, 4096): 256, (22016, 4096): 256, (4096, 11008): 256, (128000, 4096): 250,
              (6144, 4096): 192, (25600, 4096): 200, (4096, 12800): 256, (153600, 4096): 240}
    for (N, K), grid in expect.items():
        plan = P.medusa_gemm_plan(P.MDZ_BF16, 64, N, K, 12)
        assert plan["grid"] == grid
        if grid < 256:
            units = (N // plan["band_cols"]) * plan["n_stages"]
            assert units % grid == 0
            per = units // grid
            assert plan["n_stages"] % per == 0 or per % plan["n_stages"] == 0
            writers = brute_force_writers(N, plan["band_cols"], plan["n_stages"], grid)
            assert len({len(w) for w in writers}) == 1, "every band has the same number of writers"


def test_plan_rejects_shapes_the_streaming_kernel_does_not_take():
    for bad in [(65, 4096, 4096), (64, 4100, 4096), (64, 4096, 4000), (0, 4096, 4096)]:
        with pytest.raises(P.MedusaError):
            P.medusa_gemm_plan(P.MDZ_BF16, *bad, 8)
    with pytest.raises(P.MedusaError):
        P.medusa_gemm_plan(P.MDZ_FP32, 64, 4096, 4096, 8)
    with pytest.raises(P.MedusaError):
        P.medusa_gemm_slot_count(P.MDZ_BF16, 64, 4096, 4096, 8, 4096)
