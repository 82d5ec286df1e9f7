"""GPU parity: powattn_prefill_varlen (a padded batch of sequences of different lengths, lengths in device
memory, one launch) vs the oracle run on each sequence alone, and vs powattn_prefill on each sequence alone (same
kernel, same order of operations per work item: bit-identical).  Bar: 2e-2 on the outputs, 1e-3 on the
log-sum-exp."""
import numpy as np
import pytest
import torch

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa
from paper_2503_03588_amd import synth
from gpu_util import TOL_LSE, TOL_O, oracle_pattern

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,W,S,flags,hq,hkv,d,npad,lens", [
    (64, 4, 1, pa.POWER, 4, 2, 128, 2048, [2048, 1000, 64, 1]),
    (128, 4, 1, pa.POWER, 8, 2, 128, 1536, [777, 1536, 0]),                 # an empty sequence is skipped
    (64, 2, 0, pa.POWER, 2, 2, 64, 1024, [1024, 513]),
    (64, 4, 1, pa.POWER, 4, 4, 128, 1024, [0, 0, 5, 1024, 0, 63, 64, 65, 1000, 0, 512, 0]),   # runs of empty sequences
    (64, 3, 1, pa.DENSE, 4, 2, 128, 1024, [1000, 1, 700]),                  # the implicit full causal list
    (64, 70, 1, pa.POWER, 2, 1, 64, 6400, [6400, 3000, 100]),               # rows of more than 63 blocks: not chained
    (128, 4, 1, pa.POWER, 6, 2, 128, 900, [900, 0, 130]),                   # three heads per KV head: two chunks, one half empty
])
def test_padded_batch(B, W, S, flags, hq, hkv, d, npad, lens):
    pat = pa.Pattern(B, W, S, flags)
    batch = len(lens)
    q, k, v = synth.qkv(batch, hq, hkv, npad, d, "bf16", seed=71)
    dense = bool(flags & pa.DENSE)
    cnt, idx = (None, None) if dense else pa.mask_build(pat, npad)[:2]
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    # the rows behind every sequence hold NaN in K and V: nothing of them may reach a result
    for b, n in enumerate(lens):
        kd[b, :, n:] = float("nan")
        vd[b, :, n:] = float("nan")
    o = torch.full_like(qd, 7.0)                                   # rows beyond a sequence must stay untouched
    lse = torch.full((batch, hq, npad), -3.0, dtype=torch.float32, device="cuda")
    pa.prefill_varlen(pat, cnt, idx, qd, kd, vd, torch.tensor(lens, dtype=torch.int32, device="cuda"), o=o, lse=lse)
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


def test_lengths_outside_the_padding_are_clamped_and_many_sequences_share_one_launch():
    # 300 short prompts in one launch (thousands of work items, most compute units pass over many items that do not
    # exist); a negative length counts as 0 and one beyond the padding as the padding
    pat = pa.Pattern(64, 4, 1)
    batch, hq, hkv, d, npad = 300, 4, 2, 128, 512
    rng = np.random.default_rng(73)
    lens = [int(x) for x in rng.integers(0, npad + 1, size=batch)]
    lens[0], lens[1], lens[2] = -5, npad + 1000, npad
    q, k, v = synth.qkv(batch, hq, hkv, npad, d, "bf16", seed=74)
    cnt, idx, _ = pa.mask_build(pat, npad)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    o = torch.full_like(qd, 7.0)
    lse = torch.full((batch, hq, npad), -3.0, dtype=torch.float32, device="cuda")
    pa.prefill_varlen(pat, cnt, idx, qd, kd, vd, torch.tensor(lens, dtype=torch.int32, device="cuda"), o=o, lse=lse)
    torch.cuda.synchronize()
    eff = [min(max(n, 0), npad) for n in lens]
    for b in list(range(6)) + [int(x) for x in rng.integers(6, batch, size=10)] + [batch - 1]:
        n = eff[b]
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
