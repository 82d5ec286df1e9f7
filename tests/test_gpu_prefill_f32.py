"""GPU parity: fp32 powattn_prefill vs the float64 oracle, element by element.
Bar: max abs error 1e-5 on the outputs, 1e-3 on the log-sum-exp."""
import math

import numpy as np
import pytest
import torch

from paper_2503_03588_amd import binding as pa
from paper_2503_03588_amd import synth
from gpu_util import check_prefill, gpu_prefill

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("sink", [1, 0])
def test_config1_tiny_prefill(sink):
    # batch 1, 2 heads, seq 1024, head_dim 64, block 64, window 2, fp32 N(0,1), seed 0
    check_prefill(pa.Pattern(64, 2, sink), 1, 2, 2, 1024, 64, "f32", seed=0)


@pytest.mark.parametrize("n,B,W,S,hq,hkv,d,batch", [
    (1000, 64, 2, 1, 2, 2, 64, 1),      # ragged tail
    (300, 16, 2, 1, 2, 1, 64, 2),       # small blocks, GQA, batch
    (777, 32, 3, 2, 4, 2, 128, 1),      # 32-token blocks, head_dim 128
    (2048, 128, 4, 1, 8, 2, 128, 1),    # two key tiles per block
    (1536, 256, 1, 0, 3, 3, 64, 1),     # four key tiles per block, pure power pattern
    (50, 64, 4, 1, 2, 2, 64, 1),        # shorter than one block
    (1024, 64, 0, 0, 2, 2, 64, 1),      # W = 0
    (500, 48, 2, 1, 2, 1, 64, 1),       # blocks of three 16-key tiles
    (1000, 192, 2, 1, 2, 1, 64, 1),     # blocks of three 64-key tiles
])
def test_shapes(n, B, W, S, hq, hkv, d, batch):
    check_prefill(pa.Pattern(B, W, S), batch, hq, hkv, n, d, "f32", seed=11)


def test_sliding_window_and_dense_flags():
    check_prefill(pa.Pattern(64, 3, 1, flags=0), 1, 2, 1, 1024, 64, "f32", seed=12)
    check_prefill(pa.Pattern(64, 3, 1, flags=pa.DENSE), 1, 2, 1, 1024, 64, "f32", seed=13)


def test_explicit_scale():
    check_prefill(pa.Pattern(64, 2, 1), 1, 2, 2, 512, 64, "f32", seed=14, scale=0.05)


def test_window_covering_everything_equals_dense_kernel():
    q, k, v = synth.qkv(1, 4, 2, 1024, 64, "f32", seed=15)
    o1, l1 = gpu_prefill(pa.Pattern(64, 16, 1), q, k, v)
    o2, l2 = gpu_prefill(pa.Pattern(64, 1, 0, flags=pa.DENSE), q, k, v)
    assert np.abs(o1 - o2).max() < 1e-6 and np.abs(l1 - l2).max() < 1e-5


def test_zero_keys_closed_form_pins_the_mask_through_the_kernel():
    n, B, W, S, d = 1024, 64, 2, 1, 64
    q, _, v = synth.qkv(1, 1, 1, n, d, "f32", seed=16)
    k = torch.zeros_like(v)
    o, lse = gpu_prefill(pa.Pattern(B, W, S), q, k, v)
    vv = v[0, 0].double().numpy()
    for i in (0, 1, 63, 64, 200, 511, 512, 1000, 1023):
        bi = i // B
        js = [j for j in range(i + 1) if (bi - j // B) < W or j // B < S or bin(bi - j // B).count("1") <= 1]
        assert abs(lse[0, 0, i] - math.log(len(js))) < 1e-5
        assert np.abs(o[0, 0, i] - vv[js].mean(axis=0)).max() < 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_a_query_block_with_an_empty_list_gives_zero_output_and_minus_infinity(dtype):
    # A caller's own list may leave a query block without any key block (Equation 1 over an empty attended
    # set): both kernels then write o = 0 and lse = -inf for its rows, and the other rows are unaffected.
    n, B = 512, 64
    pat = pa.Pattern(B, 2, 1)
    q, k, v = synth.qkv(1, 2, 2, n, 64, dtype, seed=17)
    cnt, idx, _ = pa.mask_build(pat, n)
    torch.cuda.synchronize()
    ref_o, ref_l = gpu_prefill(pat, q, k, v, lists=(cnt, idx))
    cnt2, idx2 = cnt.clone(), idx.clone()
    cnt2[3] = 0
    idx2[3] = -1
    o, lse = gpu_prefill(pat, q, k, v, lists=(cnt2, idx2))
    rows = slice(3 * B, 4 * B)
    assert (o[:, :, rows] == 0).all()
    assert np.isneginf(lse[:, :, rows]).all()
    keep = np.ones(n, dtype=bool)
    keep[rows] = False
    assert np.array_equal(o[:, :, keep], ref_o[:, :, keep]) and np.array_equal(lse[:, :, keep], ref_l[:, :, keep])
