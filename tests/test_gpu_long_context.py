"""GPU parity at a context of 1,048,576 tokens: tensors beyond 2^32 elements, so that every row and slab offset of
the kernels is exercised in 64 bits.  Inputs are drawn on the GPU (seeded); the oracle gets the sampled query rows
and the one KV head they read, taken from the far end of the tensors, where the offsets are largest.  Bars as for
the other parity tests: 2e-2 on the outputs, 1e-3 on the log-sum-exp."""
import numpy as np
import pytest
import torch

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa
from paper_2503_03588_amd import synth
from gpu_util import TOL_LSE, TOL_O, oracle_pattern

pytestmark = pytest.mark.gpu

N = 1 << 20


def test_prefill_at_a_million_tokens():
    pat = pa.Pattern(128, 4, 1)
    hq, hkv, d = 32, 8, 128                                  # Q and O: 2^32 elements each
    g = torch.Generator(device="cuda")
    g.manual_seed(101)
    q = torch.randn(1, hq, N, d, device="cuda", dtype=torch.bfloat16, generator=g)
    k = torch.randn(1, hkv, N, d, device="cuda", dtype=torch.bfloat16, generator=g)
    v = torch.randn(1, hkv, N, d, device="cuda", dtype=torch.bfloat16, generator=g)
    cnt, idx, max_k = pa.mask_build(pat, N)
    # the lists of a few query blocks against the oracle's token predicate (the row of a block's last token touches
    # every block the query block attends; the whole table at this length would take the oracle minutes)
    cn, ix = cnt.cpu().numpy(), idx.cpu().numpy()
    for i in (0, 1, 5, 4095, 4096, 8190, 8191):
        allowed = orc.token_mask_rows([(i + 1) * 128 - 1], N, oracle_pattern(pat))[0]
        blocks = np.unique(np.nonzero(allowed)[0] // 128)
        assert cn[i] == blocks.size and np.array_equal(ix[i, :cn[i]], blocks) and (ix[i, cn[i]:] == -1).all(), i
    o, lse = pa.prefill(pat, cnt, idx, q, k, v)
    torch.cuda.synchronize()
    rng = np.random.default_rng(102)
    rows = np.unique(np.concatenate([[0, 127, 128, N // 2 - 1, N // 2, N - 129, N - 128, N - 1], rng.integers(0, N, 8)]))
    rt = torch.from_numpy(rows).cuda()
    for kvh in (hkv - 1, 0):                                 # the last KV head's group (largest offsets), then the first
        hs = slice(kvh * (hq // hkv), (kvh + 1) * (hq // hkv))
        oo, ol = orc.attention_rows(synth.to_numpy_storage(q[:, hs][:, :, rt]), synth.to_numpy_storage(k[:, kvh:kvh + 1]),
                                    synth.to_numpy_storage(v[:, kvh:kvh + 1]), rows, oracle_pattern(pat),
                                    q_holds_rows_only=True)
        go = o[:, hs][:, :, rt].double().cpu().numpy()
        gl = lse[:, hs][:, :, rt].double().cpu().numpy()
        assert np.isfinite(go).all()
        assert np.abs(go - oo).max() <= TOL_O["bf16"], kvh
        assert np.abs(gl - ol).max() <= TOL_LSE, kvh


def test_decode_at_a_million_tokens():
    pat = pa.Pattern(64, 4, 1)
    batch, hq, hkv, d, cap = 16, 32, 8, 128, N + 64          # each cache: 1.7e10 elements
    g = torch.Generator(device="cuda")
    g.manual_seed(103)
    kc = torch.randn(batch, hkv, cap, d, device="cuda", dtype=torch.bfloat16, generator=g)
    vc = torch.randn(batch, hkv, cap, d, device="cuda", dtype=torch.bfloat16, generator=g)
    q = torch.randn(batch, hq, d, device="cuda", dtype=torch.bfloat16, generator=g)
    lens_list = [N, N - 1, N - 63, N - 64, 1000003, 777, 1, N] + [N - 5 * i for i in range(8)]
    lens = torch.tensor(lens_list, dtype=torch.int32).cuda()
    o, lse = pa.decode(pat, q, kc, vc, lens)
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all()
    for b, kvh in ((batch - 1, hkv - 1), (0, 0), (4, 3)):    # far end, near end, a shorter sequence
        hs = slice(kvh * (hq // hkv), (kvh + 1) * (hq // hkv))
        oo, ol = orc.decode(synth.to_numpy_storage(q[b:b + 1, hs]), synth.to_numpy_storage(kc[b:b + 1, kvh:kvh + 1]),
                            synth.to_numpy_storage(vc[b:b + 1, kvh:kvh + 1]), np.asarray([lens_list[b]]), oracle_pattern(pat))
        assert np.abs(o[b:b + 1, hs].double().cpu().numpy() - oo).max() <= TOL_O["bf16"], (b, kvh)
        assert np.abs(lse[b:b + 1, hs].double().cpu().numpy() - ol).max() <= TOL_LSE, (b, kvh)
