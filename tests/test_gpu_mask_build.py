"""GPU parity: powattn_mask_build vs the oracle's lists derived from the token
mask.  Integer work: the comparison is bit-exact."""
import numpy as np
import pytest
import torch

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa

pytestmark = pytest.mark.gpu

CASES = [
    # seq_len, B, W, S, flags
    (1024, 64, 2, 1, pa.POWER),            # config 1
    (1024, 64, 2, 0, pa.POWER),
    (32768, 64, 4, 1, pa.POWER),           # config 2
    (32768, 64, 4, 0, pa.POWER),
    (131072, 128, 4, 1, pa.POWER),         # config 3
    (65536, 64, 4, 1, pa.POWER),           # configs 4 and 5
    (32768, 256, 5, 1, pa.POWER),          # the paper's own setting (Section 4.1)
    (32768, 256, 9, 1, 0),                 # sliding window + sink baseline
    (1000, 64, 0, 0, pa.POWER),            # W = 0: diagonal still attended; ragged tail
    (5000, 16, 3, 5, pa.POWER),            # wide sink overlapping powers and window
    (64, 64, 4, 1, pa.POWER),              # a single block
    (37, 64, 4, 1, pa.POWER),              # shorter than one block
    (4096, 1, 1, 0, pa.POWER),             # token-level pattern of Theorem B.1
    (2048, 16, 2, 1, pa.DENSE),            # dense lists
]


@pytest.mark.parametrize("n,B,W,S,flags", CASES)
def test_lists_bit_exact(n, B, W, S, flags):
    pat = pa.Pattern(B, W, S, flags)
    opat = orc.Pattern(B, W, S, power=bool(flags & pa.POWER), dense=bool(flags & pa.DENSE))
    cnt, idx, mk = orc.block_lists(n, opat)
    nb = cnt.shape[0]
    want_bm = nb <= 2048
    g_cnt, g_idx, g_bm = pa.mask_build(pat, n, want_block_mask=want_bm)
    torch.cuda.synchronize()
    assert g_idx.shape == (nb, mk)
    assert np.array_equal(g_cnt.cpu().numpy(), cnt)
    assert np.array_equal(g_idx.cpu().numpy(), idx)
    if want_bm:
        assert np.array_equal(g_bm.cpu().numpy().astype(bool), orc.block_mask(n, opat))


def test_wider_row_capacity_is_padded():
    pat = pa.Pattern(64, 4, 1)
    n = 8192
    cnt, idx, mk = orc.block_lists(n, orc.Pattern(64, 4, 1))
    nb = cnt.shape[0]
    g_idx = torch.full((nb, mk + 3), 12345, dtype=torch.int32, device="cuda")
    g_cnt, g_idx, _ = pa.mask_build(pat, n, kv_idx=g_idx)
    torch.cuda.synchronize()
    got = g_idx.cpu().numpy()
    assert np.array_equal(got[:, :mk], idx)
    assert (got[:, mk:] == -1).all()


def test_short_capacity_is_refused():
    pat = pa.Pattern(64, 4, 1)
    g_idx = torch.empty((1024, 5), dtype=torch.int32, device="cuda")
    with pytest.raises(pa.PowattnError) as e:
        pa.mask_build(pat, 65536, kv_idx=g_idx)
    assert e.value.status == pa.WORKSPACE_TOO_SMALL
