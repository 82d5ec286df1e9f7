"""GPU tests of powattn_prefill_chunk_paged: a prompt processed in pieces against a KV cache kept as pages of one
block each gives, bit for bit, the rows of powattn_prefill on the sequence those pages spell out (same kernel, same
tile order; those rows are checked against the oracle here on a sample and in full elsewhere).  Unused pages, the
rows of a page beyond the context and table entries beyond the context are poisoned."""
import numpy as np
import pytest
import torch

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa
from paper_2503_03588_amd import synth
from gpu_util import TOL_LSE, TOL_O, oracle_pattern

pytestmark = pytest.mark.gpu


def to_pages(k, v, n_ctx, block, n_extra, seed):
    """Scatters the first n_ctx positions of [b, Hkv, N, D] over a shuffled pool [n_pages, Hkv, block, D]; everything
    else in the pool is NaN.  Returns the pools and the block table [b, ceil(N/block)] (entries of blocks that start
    at or beyond n_ctx hold a page number outside the pool)."""
    b, hkv, n, d = k.shape
    nbk = (n + block - 1) // block
    used = (n_ctx + block - 1) // block
    n_pages = b * used + n_extra
    rng = np.random.default_rng(seed)
    perm = rng.permutation(n_pages)[: b * used].reshape(b, used)
    table = np.full((b, nbk), 2 ** 30, dtype=np.int32)
    table[:, :used] = perm
    kp = torch.full((n_pages, hkv, block, d), float("nan"), dtype=k.dtype)
    vp = torch.full((n_pages, hkv, block, d), float("nan"), dtype=v.dtype)
    for bi in range(b):
        for j in range(used):
            lo, hi = j * block, min((j + 1) * block, n_ctx)
            kp[perm[bi, j], :, : hi - lo] = k[bi, :, lo:hi]
            vp[perm[bi, j], :, : hi - lo] = v[bi, :, lo:hi]
    return kp, vp, torch.from_numpy(table)


@pytest.mark.parametrize("n,B,W,S,hq,hkv,d,batch,cuts,flags", [
    (4096, 64, 4, 1, 8, 2, 128, 1, [0, 1024, 1088, 4096], pa.POWER),
    (3000, 64, 2, 1, 4, 4, 128, 2, [0, 64, 2047, 3000], pa.POWER),               # ragged end, a cut inside a block
    (4096, 128, 4, 1, 8, 2, 128, 1, [0, 2048, 2176, 3001, 4096], pa.POWER),      # two tiles per page
    (8192, 64, 4, 1, 16, 4, 128, 2, [0, 4096, 8192], pa.POWER),                  # many chained work items
    (2048, 64, 3, 1, 4, 2, 64, 1, [0, 1000, 2048], 0),                           # sliding window, head_dim 64
    (1900, 192, 2, 1, 4, 2, 128, 1, [0, 768, 1900], pa.POWER),                   # pages of 192 tokens
    (2500, 64, 4, 0, 7, 1, 128, 2, [0, 1, 2500], pa.POWER),                      # GQA 7, no sink, a one-token chunk
    (1024, 256, 5, 1, 8, 2, 128, 1, [0, 300, 1024], pa.POWER),                   # the paper's block size
])
def test_paged_chunks_equal_whole_prefill(n, B, W, S, hq, hkv, d, batch, cuts, flags):
    pat = pa.Pattern(B, W, S, flags)
    q, k, v = synth.qkv(batch, hq, hkv, n, d, "bf16", seed=61)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    cnt, idx, _ = pa.mask_build(pat, n)
    o_ref, l_ref = pa.prefill(pat, cnt, idx, qg, kg, vg)
    for a, b in zip(cuts[:-1], cuts[1:]):
        kp, vp, table = to_pages(k, v, b, B, n_extra=3, seed=62 + a)     # the pool holds exactly the first b positions
        o, l = pa.prefill_chunk_paged(pat, cnt, idx, qg[:, :, a:b].contiguous(), kp.cuda(), vp.cuda(), table.cuda(), a)
        torch.cuda.synchronize()
        assert torch.isfinite(o.float()).all() and torch.isfinite(l).all(), (a, b)
        assert torch.equal(o, o_ref[:, :, a:b]), (a, b)
        assert torch.equal(l, l_ref[:, :, a:b]), (a, b)


def test_paged_chunk_against_the_oracle():
    pat = pa.Pattern(64, 4, 1)
    n, hq, hkv, d, a = 3000, 8, 2, 128, 1111
    q, k, v = synth.qkv(2, hq, hkv, n, d, "bf16", seed=63)
    kp, vp, table = to_pages(k, v, n, 64, n_extra=7, seed=64)
    cnt, idx, _ = pa.mask_build(pat, n)
    o, l = pa.prefill_chunk_paged(pat, cnt, idx, q[:, :, a:].contiguous().cuda(), kp.cuda(), vp.cuda(), table.cuda(), a)
    torch.cuda.synchronize()
    rows = [a, a + 1, 1151, 1152, 2047, 2048, 2999]
    oo, ol = orc.attention_rows(synth.to_numpy_storage(q), synth.to_numpy_storage(k), synth.to_numpy_storage(v),
                                rows, oracle_pattern(pat))
    sel = [r - a for r in rows]
    assert np.abs(o.double().cpu().numpy()[:, :, sel] - oo).max() <= TOL_O["bf16"]
    assert np.abs(l.double().cpu().numpy()[:, :, sel] - ol).max() <= TOL_LSE


def test_bad_page_numbers_stay_inside_the_pool():
    # page numbers outside the pool are clamped into it: wrong numbers, finite, no stray access
    pat = pa.Pattern(64, 4, 1)
    n, hq, hkv, d = 1024, 4, 2, 128
    q, k, v = synth.qkv(1, hq, hkv, n, d, "bf16", seed=65)
    kp = k.reshape(1, hkv, n // 64, 64, d).permute(0, 2, 1, 3, 4).reshape(n // 64, hkv, 64, d).contiguous()
    vp = v.reshape(1, hkv, n // 64, 64, d).permute(0, 2, 1, 3, 4).reshape(n // 64, hkv, 64, d).contiguous()
    table = torch.tensor([[-5, 10 ** 9, 3, -(2 ** 31), 2 ** 31 - 1] + [7] * (n // 64 - 5)], dtype=torch.int32)
    cnt, idx, _ = pa.mask_build(pat, n)
    o, l = pa.prefill_chunk_paged(pat, cnt, idx, q.cuda(), kp.cuda(), vp.cuda(), table.cuda(), 0)
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all() and torch.isfinite(l).all()


def test_prompt_in_paged_chunks_then_paged_decode():
    # the serving flow on one pool: prompt in two chunks, then the next tokens through powattn_decode_paged
    pat = pa.Pattern(64, 4, 1)
    n, hq, hkv, d = 2200, 8, 2, 128
    q, k, v = synth.qkv(1, hq, hkv, n, d, "bf16", seed=66)
    kp, vp, table = to_pages(k, v, n, 64, n_extra=2, seed=67)
    kpg, vpg, tg, qg = kp.cuda(), vp.cuda(), table.cuda(), q.cuda()
    cnt, idx, _ = pa.mask_build(pat, n)
    o_ref, l_ref = pa.prefill(pat, cnt, idx, qg, k.cuda(), v.cuda())
    o1, l1 = pa.prefill_chunk_paged(pat, cnt, idx, qg[:, :, :1500].contiguous(), kpg, vpg, tg, 0)
    o2, l2 = pa.prefill_chunk_paged(pat, cnt, idx, qg[:, :, 1500:2100].contiguous(), kpg, vpg, tg, 1500)
    torch.cuda.synchronize()
    assert torch.equal(torch.cat([o1, o2], dim=2), o_ref[:, :, :2100])
    assert torch.equal(torch.cat([l1, l2], dim=2), l_ref[:, :, :2100])
    for t in (2100, 2111, 2112, 2199):
        od, ld = pa.decode_paged(pat, qg[:, :, t].contiguous(), kpg, vpg, tg, torch.tensor([t + 1], dtype=torch.int32).cuda())
        torch.cuda.synchronize()
        # a decode step and the prefill row round differently: both are within the bar of the oracle, hence 2x of each other
        assert (od.float() - o_ref[:, :, t].float()).abs().max().item() <= 2 * TOL_O["bf16"]
        assert (ld - l_ref[:, :, t]).abs().max().item() <= 2 * TOL_LSE
