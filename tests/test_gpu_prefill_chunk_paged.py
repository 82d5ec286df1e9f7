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


def pool_for(k, v, ctx, block, n_extra, seed):
    """One pool for a batch whose sequence b holds its first ctx[b] positions; returns pools and table [b, nbk]."""
    b, hkv, n, d = k.shape
    nbk = (n + block - 1) // block
    used = [(c + block - 1) // block for c in ctx]
    n_pages = sum(used) + n_extra
    perm = np.random.default_rng(seed).permutation(n_pages)
    table = np.full((b, nbk), -7, dtype=np.int32)
    kp = torch.full((n_pages, hkv, block, d), float("nan"), dtype=k.dtype)
    vp = torch.full((n_pages, hkv, block, d), float("nan"), dtype=v.dtype)
    at = 0
    for bi in range(b):
        for j in range(used[bi]):
            pg = int(perm[at]); at += 1
            table[bi, j] = pg
            lo, hi = j * block, min((j + 1) * block, ctx[bi])
            kp[pg, :, : hi - lo] = k[bi, :, lo:hi]
            vp[pg, :, : hi - lo] = v[bi, :, lo:hi]
    return kp, vp, torch.from_numpy(table)


@pytest.mark.parametrize("n,B,W,S,hq,hkv,d,pieces,q_rows,flags", [
    # (q_start, q_len) per sequence
    (3000, 64, 4, 1, 8, 2, 128, [(0, 700), (1024, 512), (2999, 1), (100, 0), (1500, 777)], 800, pa.POWER),
    (2048, 128, 4, 1, 8, 2, 128, [(0, 2048), (1000, 1048), (2047, 1)], 2048, pa.POWER),       # whole prompts and a decode-like row
    (2500, 64, 2, 0, 7, 1, 128, [(63, 130), (64, 64), (0, 1), (2400, 100)], 130, pa.POWER),    # GQA 7, no sink
    (1900, 192, 3, 1, 4, 2, 64, [(191, 500), (192, 384), (5, 1000)], 1000, 0),                 # sliding window, pages of 192, head_dim 64
    (1024, 256, 5, 1, 8, 2, 128, [(0, 0), (0, 0)], 16, pa.POWER),                              # nothing to do
])
def test_batch_of_pieces_equals_each_piece_alone(n, B, W, S, hq, hkv, d, pieces, q_rows, flags):
    pat = pa.Pattern(B, W, S, flags)
    batch = len(pieces)
    q, k, v = synth.qkv(batch, hq, hkv, n, d, "bf16", seed=71)
    ctx = [a + ln for a, ln in pieces]
    kp, vp, table = pool_for(k, v, ctx, B, n_extra=4, seed=72)
    kpg, vpg, tg = kp.cuda(), vp.cuda(), table.cuda()
    cnt, idx, _ = pa.mask_build(pat, table.shape[1] * B)
    qb = torch.full((batch, hq, q_rows, d), float("nan"), dtype=torch.bfloat16)          # padding rows must not be read
    for bi, (a, ln) in enumerate(pieces):
        qb[bi, :, :ln] = q[bi, :, a:a + ln]
    sentinel = 12345.0
    ob = torch.full((batch, hq, q_rows, d), sentinel, dtype=torch.bfloat16, device="cuda")
    lb = torch.full((batch, hq, q_rows), sentinel, dtype=torch.float32, device="cuda")
    starts = torch.tensor([a for a, _ in pieces], dtype=torch.int32).cuda()
    lens = torch.tensor([ln for _, ln in pieces], dtype=torch.int32).cuda()
    pa.prefill_batch_paged(pat, cnt, idx, qb.cuda(), kpg, vpg, tg, starts, lens, o=ob, lse=lb)
    torch.cuda.synchronize()
    for bi, (a, ln) in enumerate(pieces):
        assert (ob[bi, :, ln:] == sentinel).all() and (lb[bi, :, ln:] == sentinel).all(), bi   # rows behind a piece untouched
        if ln == 0:
            continue
        o1, l1 = pa.prefill_chunk_paged(pat, cnt, idx, q[bi:bi + 1, :, a:a + ln].contiguous().cuda(), kpg, vpg,
                                        tg[bi:bi + 1].contiguous(), a)
        torch.cuda.synchronize()
        assert torch.isfinite(o1.float()).all()
        assert torch.equal(ob[bi:bi + 1, :, :ln], o1), (bi, a, ln)
        assert torch.equal(lb[bi:bi + 1, :, :ln], l1), (bi, a, ln)


def test_batch_of_pieces_against_the_oracle():
    pat = pa.Pattern(64, 4, 1)
    n, hq, hkv, d = 2200, 8, 2, 128
    pieces = [(0, 300), (1000, 300), (1900, 300)]
    q, k, v = synth.qkv(3, hq, hkv, n, d, "bf16", seed=73)
    kp, vp, table = pool_for(k, v, [a + ln for a, ln in pieces], 64, n_extra=1, seed=74)
    cnt, idx, _ = pa.mask_build(pat, table.shape[1] * 64)
    qb = torch.stack([q[bi, :, a:a + ln] for bi, (a, ln) in enumerate(pieces)])
    o, l = pa.prefill_batch_paged(pat, cnt, idx, qb.cuda(), kp.cuda(), vp.cuda(), table.cuda(),
                                  torch.tensor([a for a, _ in pieces], dtype=torch.int32).cuda(),
                                  torch.tensor([ln for _, ln in pieces], dtype=torch.int32).cuda())
    torch.cuda.synchronize()
    for bi, (a, ln) in enumerate(pieces):
        rows = [a, a + 63, a + 64, a + ln - 1]
        oo, ol = orc.attention_rows(synth.to_numpy_storage(q[bi:bi + 1]), synth.to_numpy_storage(k[bi:bi + 1]),
                                    synth.to_numpy_storage(v[bi:bi + 1]), rows, oracle_pattern(pat))
        sel = [r - a for r in rows]
        assert np.abs(o[bi:bi + 1].double().cpu().numpy()[:, :, sel] - oo).max() <= TOL_O["bf16"]
        assert np.abs(l[bi:bi + 1].double().cpu().numpy()[:, :, sel] - ol).max() <= TOL_LSE


def test_batch_lengths_out_of_range_are_clamped():
    # a length beyond the slab of Q/O, a start beyond the table, a negative start, a length that runs past the table:
    # clamped, finite, no stray access
    pat = pa.Pattern(64, 4, 1)
    n, hq, hkv, d, q_rows = 1024, 4, 2, 128, 200
    q, k, v = synth.qkv(4, hq, hkv, n, d, "bf16", seed=75)
    kp, vp, table = pool_for(k, v, [n, n, n, n], 64, n_extra=0, seed=76)
    kpg, vpg, tg = kp.cuda(), vp.cuda(), table.cuda()
    cnt, idx, _ = pa.mask_build(pat, n)
    qb = q[:, :, :q_rows].contiguous()
    qb[3, :, :24] = q[3, :, 1000:1024]
    o = torch.zeros((4, hq, q_rows, d), dtype=torch.bfloat16, device="cuda")
    starts = torch.tensor([0, 10 ** 9, -50, 1000], dtype=torch.int32).cuda()
    lens = torch.tensor([10 ** 9, 200, 200, 10 ** 9], dtype=torch.int32).cuda()
    pa.prefill_batch_paged(pat, cnt, idx, qb.cuda(), kpg, vpg, tg, starts, lens, o=o, want_lse=False)
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all()
    assert (o[1] == 0).all()                      # start clamped to the end of the table: no rows left
    assert (o[3, :, 24:] == 0).all()              # 1000 + length clamped to 1024: 24 rows
    for bi, piece in enumerate([(0, 200), None, (0, 200), (1000, 24)]):
        if piece is None:
            continue
        a, ln = piece
        o1, _ = pa.prefill_chunk_paged(pat, cnt, idx, q[bi:bi + 1, :, a:a + ln].contiguous().cuda(), kpg, vpg,
                                       tg[bi:bi + 1].contiguous(), a)
        torch.cuda.synchronize()
        assert torch.equal(o[bi:bi + 1, :, :ln], o1), bi


def test_batch_of_pieces_replayed_from_a_hip_graph_with_new_lengths():
    # Starts and lengths are read by the kernel, so one captured launch serves successive serving steps: capture
    # once, then replay with other (start, length) pairs written into the same device arrays, with eager calls in
    # between, and compare every replay with the eager result of the same step.
    pat = pa.Pattern(64, 4, 1)
    n, hq, hkv, d, q_rows, batch = 2600, 8, 2, 128, 512, 3
    q, k, v = synth.qkv(batch, hq, hkv, n, d, "bf16", seed=81)
    kp, vp, table = pool_for(k, v, [n] * batch, 64, n_extra=2, seed=82)
    kpg, vpg, tg, qg = kp.cuda(), vp.cuda(), table.cuda(), q.cuda()
    cnt, idx, _ = pa.mask_build(pat, table.shape[1] * 64)
    steps = [[(0, 512), (100, 300), (2000, 1)], [(512, 512), (400, 512), (2001, 1)], [(1024, 77), (912, 0), (2002, 511)]]
    qb = torch.zeros((batch, hq, q_rows, d), dtype=torch.bfloat16, device="cuda")
    starts = torch.zeros(batch, dtype=torch.int32, device="cuda")
    lens = torch.zeros(batch, dtype=torch.int32, device="cuda")
    o_g = torch.zeros_like(qb)
    l_g = torch.zeros((batch, hq, q_rows), dtype=torch.float32, device="cuda")

    def load(step):
        qb.zero_()
        for bi, (a, ln) in enumerate(step):
            qb[bi, :, :ln] = qg[bi, :, a:a + ln]
        starts.copy_(torch.tensor([a for a, _ in step], dtype=torch.int32))
        lens.copy_(torch.tensor([ln for _, ln in step], dtype=torch.int32))

    load(steps[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm up on the capture stream (one-time launch set-up)
        pa.prefill_batch_paged(pat, cnt, idx, qb, kpg, vpg, tg, starts, lens, o=o_g, lse=l_g, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        pa.prefill_batch_paged(pat, cnt, idx, qb, kpg, vpg, tg, starts, lens, o=o_g, lse=l_g)
    for rep in range(6):
        step = steps[rep % 3]
        load(step)
        o_e = torch.full_like(qb, 7.0)
        l_e = torch.full_like(l_g, 7.0)
        pa.prefill_batch_paged(pat, cnt, idx, qb, kpg, vpg, tg, starts, lens, o=o_e, lse=l_e)   # eager, between replays
        o_g.fill_(7.0); l_g.fill_(7.0)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(o_g, o_e) and torch.equal(l_g, l_e), rep
        for bi, (a, ln) in enumerate(step):
            assert (o_g[bi, :, ln:] == 7.0).all(), (rep, bi)
            if ln:
                assert torch.isfinite(o_g[bi, :, :ln].float()).all() and (o_g[bi, :, :ln] != 7.0).any(), (rep, bi)
