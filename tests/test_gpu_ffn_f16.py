"""GPU parity of a bf16 model whose feed-forward products take binary16 operands (the model descriptor's ffn_f16):
what a layer computes (Section 3.2 of the paper: the ordinary decoder layer applied to the tree's rows) is unchanged,
so the oracle and the inputs are those of the plain bf16 cases; only the rounding of two activations differs."""
import numpy as np
import pytest
import torch

import workload as W
import paper_2603_03383_amd as P
from tests import gpu_util as G
from tests.test_gpu_parity import _layer_case, _check_layer, ragged_batch_case
from tests.test_gpu_gqa import two_layer_step_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("S_list,max_prefix", [([0], 0), ([77], 100), ([512], 512), ([300, 0, 45], 300)])
def test_7b_width_layer(S_list, max_prefix):
    """One and three sequences: the skinny GEMM with SwiGLU in its epilogue, and the split GEMM + separate SwiGLU."""
    w = W.CONFIGS["cfg2_layer_bf16"].with_(name="layer_ffn16", ffn_f16=True, prefix=tuple(S_list))
    r = _layer_case(w, S_list, max_prefix, x_seed="ffn16_layer_x")
    rel = _check_layer(r, S_list, "bf16")
    print(f"binary16 feed-forward layer {S_list}: err/scale {rel:.3e}")


@pytest.mark.parametrize("ffn", [10240, 10208])
def test_small_layer_other_ffn_widths(ffn):
    w = W.CONFIGS["cfg2_layer_bf16"].with_(name="layer_ffn16_w", ffn_f16=True, ffn=ffn, prefix=(40,))
    r = _layer_case(w, [40], 40, x_seed="ffn16_w_x")
    _check_layer(r, [40], "bf16")


def test_autoregressive_layer():
    w = W.CONFIGS["cfg2_layer_bf16"].with_(name="ar_layer_ffn16", ffn_f16=True, tree=W.TREE1, prefix=(0, 33, 1000))
    r = _layer_case(w, [0, 33, 1000], 1000, x_seed="ffn16_ar_x")
    _check_layer(r, [0, 33, 1000], "bf16")


def test_two_layer_step_with_heads():
    two_layer_step_case(W.CONFIGS["cfg3_step_1k"].with_(name="step_ffn16", n_layers=2, ffn_f16=True))


def test_ragged_batch_of_16_takes_the_many_row_gemm():
    ragged_batch_case(W.CONFIGS["cfg5_ragged_b16"].with_(n_layers=1, ffn_f16=True))


def test_packed_binary16_copy_holds_the_bf16_values():
    """medusa_pack_weight_bf16_as_f16 against medusa_pack_weight of the same matrix converted by torch: identical
    bytes, including values that land in binary16's subnormal range and the padding of a ragged shape."""
    g = torch.Generator(device="cpu").manual_seed(5)
    n, k = 96, 300
    src = (torch.randn(n, k, generator=g) * 0.02).to(torch.bfloat16)
    src[0, :8] = torch.tensor([0.0, -0.0, 2.0 ** -14, 2.0 ** -15, 3 * 2.0 ** -20, -2.0 ** -24, 1.0, -65280.0]).to(torch.bfloat16)
    src = src.to(G.DEV)
    nb = P.medusa_packed_bytes(P.MDZ_BF16, n, k)
    a = torch.zeros(nb, dtype=torch.uint8, device=G.DEV)
    b = torch.zeros(nb, dtype=torch.uint8, device=G.DEV)
    P.medusa_pack_weight_bf16_as_f16(src, a, n)
    P.medusa_pack_weight(P.MDZ_FP16, src.to(torch.float16).contiguous(), b, n)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
