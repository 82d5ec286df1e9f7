"""GPU: powattn_decode_static (the entry point that allocates nothing: partial results in the library's own
static device buffer) against powattn_decode on a caller's workspace and against the oracle, on two calls in a
row, the second on a smaller input, so that the second call meets the first one's leftovers in the shared buffer.
Bars: bit-equal to powattn_decode (same kernels, same order of the sums); 2e-2 / 1e-3 against the oracle."""
import numpy as np
import pytest
import torch

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa
from paper_2503_03588_amd import synth
from gpu_util import TOL_LSE, TOL_O, oracle_pattern

pytestmark = pytest.mark.gpu


def _case(pat, batch, hq, hkv, cap, d, kv_len, seed):
    q, k, v = synth.decode_inputs(batch, hq, hkv, cap, d, "bf16", seed)
    lens = torch.tensor(kv_len, dtype=torch.int32)
    oo, olse = orc.decode(synth.to_numpy_storage(q), synth.to_numpy_storage(k), synth.to_numpy_storage(v),
                          np.asarray(kv_len), oracle_pattern(pat), None)
    return [t.cuda() for t in (q, k, v, lens)], oo, olse


def _check(pat, dev, oo, olse):
    q, k, v, lens = dev
    o_ref, lse_ref = pa.decode(pat, q, k, v, lens)                     # caller-workspace entry point
    o = torch.full_like(q, float("nan"))
    lse = torch.full((q.shape[0], q.shape[1]), float("nan"), dtype=torch.float32, device=q.device)
    pa.decode_static(pat, q, k, v, lens, o, lse)
    torch.cuda.synchronize()
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)
    assert np.abs(o.double().cpu().numpy() - oo).max() <= TOL_O["bf16"]
    assert np.abs(lse.double().cpu().numpy() - olse).max() <= TOL_LSE


def test_static_scratch_decode_two_calls_second_smaller():
    pat = pa.Pattern(64, 4, 1)
    big = _case(pat, 6, 8, 2, 8192, 128, [8192, 8191, 4097, 4096, 130, 1], seed=71)       # 5 workgroups per pair
    small = _case(pat, 2, 8, 2, 4096, 128, [4096, 2000], seed=72)                          # fewer pairs, other data
    _check(pat, *big)
    _check(pat, *small)
    _check(pat, *big)          # and back: the buffer now holds the smaller call's leftovers
    # another pattern and head_dim on the same buffer, 10 workgroups per pair
    pat2 = pa.Pattern(128, 4, 1)
    _check(pat2, *_case(pat2, 1, 4, 2, 16384, 64, [16384], seed=73))


def test_static_scratch_decode_large_batch_paths():
    # persistent workgroups + merge kernel on the static buffer (float partials), then the small fused case again
    pat = pa.Pattern(64, 4, 1)
    rng = np.random.default_rng(74)
    lens = [int(x) for x in rng.integers(1, 2049, size=288)]
    _check(pat, *_case(pat, 288, 8, 4, 2048, 128, lens, seed=75))
    _check(pat, *_case(pat, 2, 8, 2, 4096, 128, [4096, 2000], seed=72))


def test_static_scratch_refuses_sizes_beyond_its_maximum():
    pat = pa.Pattern(64, 4, 1)
    batch, hq, hkv, cap, d = 1024, 32, 8, 1 << 16, 128
    assert pa.decode_workspace_bytes(pat, batch, hq, hkv, d, cap) > (32 << 20)
    q = torch.zeros(batch, hq, d, dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros(1, dtype=torch.bfloat16, device="cuda")            # never read: the call is refused on the host
    lens = torch.ones(batch, dtype=torch.int32, device="cuda")
    import ctypes
    st = pa.lib().powattn_decode_static(ctypes.byref(pat.c()), q.data_ptr(), kv.data_ptr(), kv.data_ptr(),
                                        lens.data_ptr(), cap, q.data_ptr(), None, batch, hq, hkv, d, pa.BF16, 0.0, None)
    assert st == pa.WORKSPACE_TOO_SMALL
