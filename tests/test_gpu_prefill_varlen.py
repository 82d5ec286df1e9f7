"""GPU parity: powattn_prefill_varlen (a padded batch of sequences of different lengths) vs the oracle run on each
sequence alone, and vs powattn_prefill on each sequence alone (same kernel, same order of operations per work
item: bit-identical).  Bar: 2e-2 on the outputs, 1e-3 on the log-sum-exp."""
import numpy as np
import pytest
import torch

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa
from paper_2503_03588_amd import synth
from gpu_util import TOL_LSE, TOL_O, oracle_pattern

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,W,S,hq,hkv,d,npad,lens", [
    (64, 4, 1, 4, 2, 128, 2048, [2048, 1000, 64, 1]),
    (128, 4, 1, 8, 2, 128, 1536, [777, 1536, 0]),                 # an empty sequence is skipped
    (64, 2, 0, 2, 2, 64, 1024, [1024, 513]),
])
def test_padded_batch(B, W, S, hq, hkv, d, npad, lens):
    pat = pa.Pattern(B, W, S)
    batch = len(lens)
    q, k, v = synth.qkv(batch, hq, hkv, npad, d, "bf16", seed=71)
    cnt, idx, _ = pa.mask_build(pat, npad)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    o = torch.full_like(qd, 7.0)                                   # rows beyond a sequence must stay untouched
    lse = torch.full((batch, hq, npad), -3.0, dtype=torch.float32, device="cuda")
    pa.prefill_varlen(pat, cnt, idx, qd, kd, vd, lens, o=o, lse=lse)
    torch.cuda.synchronize()
    for b, n in enumerate(lens):
        assert torch.all(o[b, :, n:] == 7.0) and torch.all(lse[b, :, n:] == -3.0)
        if n == 0:
            continue
        qs, ks, vs = q[b:b + 1, :, :n].contiguous(), k[b:b + 1, :, :n].contiguous(), v[b:b + 1, :, :n].contiguous()
        o1, l1 = pa.prefill(pat, cnt, idx, qs.cuda(), ks.cuda(), vs.cuda())
        torch.cuda.synchronize()
        assert torch.equal(o[b, :, :n], o1[0]) and torch.equal(lse[b, :, :n], l1[0])
        oo, olse = orc.attention(synth.to_numpy_storage(qs), synth.to_numpy_storage(ks), synth.to_numpy_storage(vs),
                                 oracle_pattern(pat))
        assert np.abs(o[b:b + 1, :, :n].double().cpu().numpy() - oo).max() <= TOL_O["bf16"]
        assert np.abs(lse[b:b + 1, :, :n].double().cpu().numpy() - olse).max() <= TOL_LSE
