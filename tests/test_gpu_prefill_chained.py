"""GPU parity for launches with more work items than compute units, where powattn_prefill chains items in
persistent workgroups (the tile stream, the block list and the Q rows of the next item are fetched during
the current one).  Reduced sizes that still give some thousand work items; rows are sampled so that the
float64 oracle stays fast: all rows of the first blocks (rows shorter than the ring), of blocks in the
middle and at the end, plus seeded random rows."""
import numpy as np
import pytest
import torch

from paper_2503_03588_amd import binding as pa
from paper_2503_03588_amd import synth
from gpu_util import check_prefill, gpu_prefill

pytestmark = pytest.mark.gpu


def rows_for(n, B, seed, extra_blocks=()):
    nb = -(-n // B)
    blocks = sorted(set([0, 1, 2, 3, 4, nb // 2, nb - 2, nb - 1] + list(extra_blocks)))
    rows = set()
    for b in blocks:
        if 0 <= b < nb:
            rows.update(range(b * B, min((b + 1) * B, n)))
    rng = np.random.default_rng(seed)
    rows.update(int(r) for r in rng.integers(0, n, size=96))
    return sorted(rows)


@pytest.mark.parametrize("n,B,W,S,hq,hkv,d,batch,flags", [
    (8192, 64, 4, 1, 16, 4, 128, 2, pa.POWER),      # 2*4*128 items, one workgroup each
    (8192, 64, 2, 0, 8, 8, 128, 1, pa.POWER),       # no GQA: half-empty workgroups (4 wavefronts)
    (6000, 64, 4, 1, 28, 4, 128, 1, pa.POWER),      # GQA 7 (an idle wavefront per item), ragged tail
    (16384, 128, 4, 1, 16, 4, 128, 1, pa.POWER),    # two 64-key tiles per block, two workgroups per query block
    (8192, 64, 0, 0, 8, 2, 128, 2, pa.POWER),       # W = 0: rows of one or two tiles at the start of every sequence
    (8192, 64, 3, 1, 8, 2, 128, 2, 0),              # sliding window + sink
    (12288, 64, 4, 1, 16, 4, 64, 2, pa.POWER),      # head_dim 64
    (4096, 256, 5, 1, 32, 4, 128, 2, pa.POWER),     # the paper's block size; four tiles per block
])
def test_chained_items(n, B, W, S, hq, hkv, d, batch, flags):
    rows = rows_for(n, B, seed=n + B)
    check_prefill(pa.Pattern(B, W, S, flags), batch, hq, hkv, n, d, "bf16", seed=41, rows=rows)


def test_chained_dense():
    n, B = 4096, 64
    check_prefill(pa.Pattern(B, 1, 0, pa.DENSE), 2, 16, 8, n, 128, "bf16", seed=42, rows=rows_for(n, B, 5))


def test_long_lists_are_not_chained_and_match_the_chained_result():
    # the same power-of-two lists, once with the row capacity the pattern needs (chained) and once padded to
    # 80 entries per row (too long for the look-ahead: one workgroup per item); both must give the same bits
    n, B, hq, hkv, d = 8192, 64, 16, 4, 128
    pat = pa.Pattern(B, 4, 1)
    q, k, v = synth.qkv(2, hq, hkv, n, d, "bf16", seed=43)
    cnt, idx, _ = pa.mask_build(pat, n)
    nb = n // B
    wide = torch.full((nb, 80), -1, dtype=torch.int32, device="cuda")
    wide[:, :idx.shape[1]] = idx
    o1, l1 = gpu_prefill(pat, q, k, v, lists=(cnt, idx))
    o2, l2 = gpu_prefill(pat, q, k, v, lists=(cnt, wide))
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_repeated_calls_are_deterministic():
    pat = pa.Pattern(64, 4, 1)
    q, k, v = synth.qkv(1, 16, 4, 8192, 128, "bf16", seed=44)
    o1, l1 = gpu_prefill(pat, q, k, v)
    o2, l2 = gpu_prefill(pat, q, k, v)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
