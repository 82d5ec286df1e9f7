"""GPU parity: powattn_decode_paged (KV cache kept as pages of one block each, found through a block table)
vs the oracle on the cache the pages spell out, and vs powattn_decode on that cache (same kernel, same order of
operations: bit-identical).  Bar: max abs error 2e-2 on the outputs (bf16), 1e-3 on the log-sum-exp."""
import numpy as np
import pytest
import torch

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa
from paper_2503_03588_amd import synth
from gpu_util import TOL_LSE, TOL_O, oracle_pattern

pytestmark = pytest.mark.gpu


def to_pages(k, v, block, n_extra, seed):
    """Scatters contiguous caches [b, Hkv, cap, D] (cap a multiple of block) over a shuffled page pool
    [n_pages, Hkv, block, D] with n_extra unused pages; returns the pools and the block table [b, cap/block]."""
    b, hkv, cap, d = k.shape
    nbk = cap // block
    n_pages = b * nbk + n_extra
    rng = np.random.default_rng(seed)
    perm = torch.from_numpy(rng.permutation(n_pages)[: b * nbk].astype(np.int64))
    table = perm.reshape(b, nbk).to(torch.int32)
    kp = torch.full((n_pages, hkv, block, d), float("nan"), dtype=k.dtype)      # unused pages must not be read
    vp = torch.full((n_pages, hkv, block, d), float("nan"), dtype=v.dtype)
    kb = k.reshape(b, hkv, nbk, block, d).permute(0, 2, 1, 3, 4).reshape(b * nbk, hkv, block, d)
    vb = v.reshape(b, hkv, nbk, block, d).permute(0, 2, 1, 3, 4).reshape(b * nbk, hkv, block, d)
    kp[perm] = kb
    vp[perm] = vb
    return kp, vp, table


@pytest.mark.parametrize("B,W,S,hq,hkv,d,cap,kv_len", [
    (64, 4, 1, 8, 2, 128, 4096, [4096, 4095, 1, 64, 65, 2049, 3000, 100]),
    (128, 4, 1, 8, 2, 128, 4096, [4096, 129, 128, 127]),          # two 64-token chunks per page
    (256, 5, 1, 4, 2, 64, 8192, [8192, 5000, 300]),               # paper's block size; head_dim 64
    (64, 2, 0, 7, 1, 128, 3008, [3008, 2999, 777]),               # GQA 7, no sink
    (192, 3, 1, 4, 2, 128, 2304, [2304, 1000, 193]),              # pages of 192 tokens: three chunks per page
])
def test_paged_matches_oracle_and_contiguous(B, W, S, hq, hkv, d, cap, kv_len):
    pat = pa.Pattern(B, W, S)
    batch = len(kv_len)
    q, k, v = synth.decode_inputs(batch, hq, hkv, cap, d, "bf16", seed=41)
    kp, vp, table = to_pages(k, v, B, n_extra=5, seed=42)
    lens = torch.tensor(kv_len, dtype=torch.int32)
    # entries of blocks beyond a sequence's length are not read: poison them
    for bi, n in enumerate(kv_len):
        table[bi, (n - 1) // B + 1:] = -12345
    qd, ld = q.cuda(), lens.cuda()
    o, lse = pa.decode_paged(pat, qd, kp.cuda(), vp.cuda(), table.cuda(), ld)
    oc, lsec = pa.decode(pat, qd, k.cuda(), v.cuda(), ld)
    torch.cuda.synchronize()
    go, glse = o.double().cpu().numpy(), lse.double().cpu().numpy()
    assert np.isfinite(go).all() and np.isfinite(glse).all()
    assert np.array_equal(go, oc.double().cpu().numpy())
    assert np.array_equal(glse, lsec.double().cpu().numpy())
    oo, olse = orc.decode(synth.to_numpy_storage(q), synth.to_numpy_storage(k), synth.to_numpy_storage(v),
                          np.asarray(kv_len), oracle_pattern(pat), None)
    assert np.abs(go - oo).max() <= TOL_O["bf16"]
    assert np.abs(glse - olse).max() <= TOL_LSE


def test_generation_appends_into_fresh_pages():
    # a sequence grows token by token across a block boundary: the new block's page is taken from the pool and
    # entered in the table; every step must equal the oracle on the tokens written so far
    pat = pa.Pattern(64, 2, 1)
    hq, hkv, d, cap = 4, 2, 128, 512
    q, k, v = synth.decode_inputs(1, hq, hkv, cap, d, "bf16", seed=43)
    n_pages = 16
    kp = torch.zeros((n_pages, hkv, 64, d), dtype=torch.bfloat16).cuda()
    vp = torch.zeros_like(kp)
    table = torch.full((1, cap // 64), -1, dtype=torch.int32)
    free = [9, 3, 14, 0, 7, 11, 2, 5]
    kn, vn = synth.to_numpy_storage(k), synth.to_numpy_storage(v)
    for t in range(0, 200):
        blk, off = divmod(t, 64)
        if off == 0:
            table[0, blk] = free[blk]
        page = int(table[0, blk])
        kp[page, :, off] = k[0, :, t].cuda()
        vp[page, :, off] = v[0, :, t].cuda()
        if t in (0, 1, 62, 63, 64, 65, 127, 128, 129, 191, 192, 199):
            lens = torch.tensor([t + 1], dtype=torch.int32).cuda()
            o, lse = pa.decode_paged(pat, q.cuda(), kp, vp, table.cuda(), lens)
            torch.cuda.synchronize()
            oo, olse = orc.decode(synth.to_numpy_storage(q), kn, vn, np.asarray([t + 1]), oracle_pattern(pat), None)
            assert np.abs(o.double().cpu().numpy() - oo).max() <= TOL_O["bf16"], t
            assert np.abs(lse.double().cpu().numpy() - olse).max() <= TOL_LSE, t


def test_bad_page_numbers_stay_inside_the_pool():
    # page numbers outside the pool are clamped by the kernel: the call completes and reads only the pool
    pat = pa.Pattern(64, 4, 1)
    q, k, v = synth.decode_inputs(2, 4, 2, 1024, 128, "bf16", seed=44)
    kp, vp, table = to_pages(k, v, 64, n_extra=0, seed=45)
    kp = torch.nan_to_num(kp); vp = torch.nan_to_num(vp)
    table[0, 3] = 10**9
    table[1, 0] = -7
    lens = torch.tensor([1024, 700], dtype=torch.int32).cuda()
    o, lse = pa.decode_paged(pat, q.cuda(), kp.cuda(), vp.cuda(), table.cuda(), lens)
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all() and torch.isfinite(lse).all()


def test_paged_large_batch_on_persistent_workgroups():
    # enough work items for the persistent workgroups; pages are looked up one item ahead there
    B, W, S, hq, hkv, d, cap, batch = 64, 4, 1, 8, 4, 128, 2048, 272
    pat = pa.Pattern(B, W, S)
    rng = np.random.default_rng(71)
    kv_len = [int(x) for x in rng.integers(1, cap + 1, size=batch)]
    kv_len[:4] = [1, B, B + 1, cap]
    q, k, v = synth.decode_inputs(batch, hq, hkv, cap, d, "bf16", seed=72)
    kp, vp, table = to_pages(k, v, B, n_extra=7, seed=73)
    for bi, n in enumerate(kv_len):
        table[bi, (n - 1) // B + 1:] = -12345
    lens = torch.tensor(kv_len, dtype=torch.int32).cuda()
    qd = q.cuda()
    o, lse = pa.decode_paged(pat, qd, kp.cuda(), vp.cuda(), table.cuda(), lens)
    oc, lsec = pa.decode(pat, qd, k.cuda(), v.cuda(), lens)
    torch.cuda.synchronize()
    assert torch.equal(o, oc) and torch.equal(lse, lsec)
    go, glse = o.double().cpu().numpy(), lse.double().cpu().numpy()
    assert np.isfinite(go).all() and np.isfinite(glse).all()
    oo, olse = orc.decode(synth.to_numpy_storage(q), synth.to_numpy_storage(k), synth.to_numpy_storage(v),
                          np.asarray(kv_len), oracle_pattern(pat), None)
    assert np.abs(go - oo).max() <= TOL_O["bf16"]
    assert np.abs(glse - olse).max() <= TOL_LSE
