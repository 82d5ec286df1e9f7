"""Helpers of the GPU parity tests: run the library and the oracle on the same seeded inputs."""
import numpy as np
import torch

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa
from paper_2503_03588_amd import synth

# bars from the benchmark spec: max abs error of the outputs 2e-2 for bf16 inputs, 1e-5 for fp32;
# log-sum-exp within 1e-3
TOL_O = {"bf16": 2e-2, "f32": 1e-5}
TOL_LSE = 1e-3


def oracle_pattern(pat: pa.Pattern) -> orc.Pattern:
    return orc.Pattern(pat.block, pat.window, pat.sink, power=bool(pat.flags & pa.POWER),
                       dense=bool(pat.flags & pa.DENSE))


def gpu_prefill(pat, q, k, v, scale=0.0, lists=None):
    """q, k, v: CPU tensors.  Returns (o, lse) as float64 NumPy arrays."""
    n = q.shape[2]
    if pat.flags & pa.DENSE:
        cnt = idx = None
    elif lists is None:
        cnt, idx, _ = pa.mask_build(pat, n)
    else:
        cnt, idx = lists
    o, lse = pa.prefill(pat, cnt, idx, q.cuda(), k.cuda(), v.cuda(), softmax_scale=scale)
    torch.cuda.synchronize()
    return o.double().cpu().numpy(), lse.double().cpu().numpy()


def check_prefill(pat, batch, hq, hkv, n, d, dtype, seed, rows=None, scale=0.0, std=1.0):
    """Element-by-element comparison (all rows, or the sampled `rows`) against the oracle.
    Returns (max abs error of o, max abs error of lse)."""
    q, k, v = synth.qkv(batch, hq, hkv, n, d, dtype, seed, std)
    return check_prefill_tensors(pat, q, k, v, dtype, rows, scale)


def check_prefill_tensors(pat, q, k, v, dtype, rows=None, scale=0.0):
    """The same comparison on given CPU tensors q [b,Hq,N,D], k, v [b,Hkv,N,D]."""
    go, glse = gpu_prefill(pat, q, k, v, scale)
    assert np.isfinite(go).all() and np.isfinite(glse).all()
    qs, ks, vs = (synth.to_numpy_storage(t) for t in (q, k, v))
    opat = oracle_pattern(pat)
    sc = None if scale <= 0 else scale
    if rows is None:
        oo, olse = orc.attention(qs, ks, vs, opat, sc)
    else:
        rows = np.asarray(sorted(set(int(r) for r in rows)))
        oo, olse = orc.attention_rows(qs, ks, vs, rows, opat, sc)
        go, glse = go[:, :, rows], glse[:, :, rows]
    err_o = float(np.abs(go - oo).max())
    err_lse = float(np.abs(glse - olse).max())
    assert err_o <= TOL_O[dtype], (err_o, TOL_O[dtype])
    assert err_lse <= TOL_LSE, err_lse
    return err_o, err_lse


def sample_rows(n, block, window, count, seed):
    """All rows of a few characteristic query blocks plus `count` seeded random rows."""
    nb = -(-n // block)
    blocks = sorted(set(b for b in (0, 1, window - 1, window, nb // 2, nb - 2, nb - 1) if 0 <= b < nb))
    rows = set()
    for b in blocks:
        rows.update(range(b * block, min((b + 1) * block, n)))
    rng = np.random.default_rng(seed)
    rows.update(int(r) for r in rng.integers(0, n, size=count))
    return sorted(rows)
