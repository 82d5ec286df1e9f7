"""GPU tests of powattn_prefill_chunk: a prompt processed in pieces against a KV cache gives, bit for bit, the
rows of the whole-sequence prefill (same kernel, same tile order), and those are checked against the oracle
elsewhere; a chunk followed by decode steps reproduces the corresponding prefill rows within the decode bar."""
import numpy as np
import pytest
import torch

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa
from paper_2503_03588_amd import synth

pytestmark = pytest.mark.gpu


def caches_from(k, v, cap):
    kc = torch.zeros(k.shape[0], k.shape[1], cap, k.shape[3], dtype=k.dtype, device="cuda")
    vc = torch.full_like(kc, float("nan"))          # positions beyond the context must never be read into a result
    kc[:] = float("nan")
    n = k.shape[2]
    kc[:, :, :n] = k
    vc[:, :, :n] = v
    return kc, vc


@pytest.mark.parametrize("n,B,W,S,hq,hkv,d,batch,cap,cuts,flags", [
    (4096, 64, 4, 1, 8, 2, 128, 1, 4096, [0, 1024, 1088, 4096], pa.POWER),
    (3000, 64, 2, 1, 4, 4, 128, 2, 5000, [0, 64, 2048, 3000], pa.POWER),          # ragged end, capacity > context
    (4096, 128, 4, 1, 8, 2, 128, 1, 8192, [0, 2048, 2176, 4096], pa.POWER),       # two tiles per block
    (8192, 64, 4, 1, 16, 4, 128, 2, 8192, [0, 4096, 8192], pa.POWER),             # chained work items inside a chunk
    (2048, 64, 3, 1, 4, 2, 64, 1, 2048, [0, 1024, 2048], 0),                      # sliding window, head_dim 64
    (2048, 64, 1, 0, 4, 2, 128, 1, 4096, [0, 512, 2048], pa.DENSE),               # dense
    (1900, 192, 2, 1, 4, 2, 128, 1, 2304, [0, 768, 1900], pa.POWER),              # blocks of 192 tokens
    (4096, 64, 4, 1, 8, 2, 128, 1, 4096, [0, 1000, 1001, 1023, 1100, 3003, 4096], pa.POWER),   # cuts inside blocks
    (3000, 128, 2, 1, 6, 2, 128, 2, 3000, [0, 129, 255, 2049, 3000], pa.POWER),   # the same with two tiles per block, ragged end
    (2500, 64, 3, 1, 4, 2, 64, 1, 2560, [0, 7, 1999, 2500], 0),                   # sliding window, head_dim 64, unaligned cuts
    (2048, 64, 1, 0, 4, 2, 128, 1, 2048, [0, 500, 2048], pa.DENSE),               # dense, unaligned cut
])
def test_chunks_equal_whole_prefill(n, B, W, S, hq, hkv, d, batch, cap, cuts, flags):
    pat = pa.Pattern(B, W, S, flags)
    q, k, v = synth.qkv(batch, hq, hkv, n, d, "bf16", seed=51)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    dense = bool(flags & pa.DENSE)
    cnt = idx = None
    if not dense:
        cnt, idx, _ = pa.mask_build(pat, n)
    o_ref, l_ref = pa.prefill(pat, cnt, idx, qg, kg, vg)
    # lists built for the whole cache capacity: rows are indexed by the block number in the sequence
    ccnt = cidx = None
    if not dense:
        ccnt, cidx, _ = pa.mask_build(pat, cap)
    for a, b in zip(cuts[:-1], cuts[1:]):
        kc, vc = caches_from(kg[:, :, :b], vg[:, :, :b], cap)     # the cache holds exactly the first b positions
        o, l = pa.prefill_chunk(pat, ccnt, cidx, qg[:, :, a:b].contiguous(), kc, vc, a)
        torch.cuda.synchronize()
        assert torch.equal(o, o_ref[:, :, a:b]), (a, b)
        assert torch.equal(l, l_ref[:, :, a:b]), (a, b)


def test_chunk_then_decode_matches_the_oracle():
    # serving flow: prompt of 3000 tokens in two chunks, then the next tokens one by one through powattn_decode
    pat = pa.Pattern(64, 4, 1)
    n, hq, hkv, d, cap = 3200, 8, 2, 128, 4096
    q, k, v = synth.qkv(1, hq, hkv, n, d, "bf16", seed=52)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    ccnt, cidx, _ = pa.mask_build(pat, cap)
    kc, vc = caches_from(kg, vg, cap)
    rows = [0, 63, 64, 1500, 2047, 2048, 2999]
    oo, ol = orc.attention_rows(synth.to_numpy_storage(q[:, :, :3000]), synth.to_numpy_storage(k[:, :, :3000]),
                                synth.to_numpy_storage(v[:, :, :3000]), rows, orc.Pattern(64, 4, 1))
    o1, l1 = pa.prefill_chunk(pat, ccnt, cidx, qg[:, :, :2048].contiguous(), kc, vc, 0)
    o2, l2 = pa.prefill_chunk(pat, ccnt, cidx, qg[:, :, 2048:3000].contiguous(), kc, vc, 2048)
    torch.cuda.synchronize()
    o = torch.cat([o1, o2], dim=2).double().cpu().numpy()
    l = torch.cat([l1, l2], dim=2).double().cpu().numpy()
    assert np.abs(o[:, :, rows] - oo).max() <= 2e-2 and np.abs(l[:, :, rows] - ol).max() <= 1e-3
    for t in (3000, 3001, 3135, 3199):
        od, ld = pa.decode(pat, qg[:, :, t].contiguous(), kc, vc, torch.tensor([t + 1], dtype=torch.int32).cuda())
        torch.cuda.synchronize()
        oo, ol = orc.attention_rows(synth.to_numpy_storage(q), synth.to_numpy_storage(k), synth.to_numpy_storage(v),
                                    [t], orc.Pattern(64, 4, 1))
        assert np.abs(od.double().cpu().numpy() - oo[:, :, 0]).max() <= 2e-2
        assert np.abs(ld.double().cpu().numpy() - ol[:, :, 0]).max() <= 1e-3
