"""GPU parity: powattn_backward (dQ, dK, dV of Equation 1 under the block pattern) vs the oracle's float64
gradients on the same bf16 inputs.

Bars, per gradient tensor (the benchmark spec gives none for gradients; derived from the kernel's arithmetic):
  * max |got - ref| <= 8e-3 * max |ref|.  A stored gradient is bf16: rounding to nearest costs up to 2^-9 = 1.95e-3
    of the entry itself.  P and dS enter the second products (dV = P^T dO, dQ = dS K, dK = dS^T Q) rounded to bf16
    too: every term of those sums carries an independent relative error of up to 2^-9, i.e. a standard deviation of
    about 2^-9 / sqrt(3) = 1.1e-3 of the root-sum-square of the terms, which for the large entries is of the order
    of the entry; over the 1e5..1e7 entries of a tensor the worst of them sits 4-5 standard deviations out.  fp32
    accumulation and the fp32 log-sum-exp / Delta are far below that.  2e-3 + 5.5e-3, rounded up: 8e-3 of the
    largest entry.
  * ||got - ref||_2 / ||ref||_2 <= 4e-3: the same three roundings as root-mean-square figures (about 1.1e-3 each for
    uniform rounding errors, those inside the sums enlarged by cancellation between terms); unlike the max-norm
    bar this one is sensitive to errors in the many small entries.
Measured over the ~60 cases of this file and of the random shapes: max-norm 2.1e-3..6.5e-3 of the largest entry,
relative root-mean-square 1.8e-3..3.0e-3."""
import numpy as np
import pytest
import torch

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa
from paper_2503_03588_amd import synth
from gpu_util import oracle_pattern

pytestmark = pytest.mark.gpu
TOL_G_MAX = 8e-3     # of the largest entry of the tensor
TOL_G_RMS = 4e-3     # relative root-mean-square error of the tensor


TOL_G_ABS = 1e-5     # absolute floor: where a gradient vanishes (a single token: P = 1, dS = dP - Delta = 0) the fp32
                     # difference dP - Delta leaves ~2^-23 * |dO . v| ~ 1e-6, times scale * |k|


def check_grad(name, got, ref):
    """got, ref: float64 arrays of one gradient tensor (or a sample of it)."""
    assert np.isfinite(got).all(), name
    big = np.abs(ref).max()
    err = np.abs(got - ref).max()
    rms_err, rms_ref = float(np.sqrt(((got - ref) ** 2).mean())), float(np.sqrt((ref ** 2).mean()))
    print(f"  {name}: max abs err {err:.3e} = {err / max(big, 1e-30):.2e} of the largest entry {big:.3f}; "
          f"rms err {rms_err:.3e} = {rms_err / max(rms_ref, 1e-30):.2e} of the rms entry", flush=True)
    assert err <= TOL_G_MAX * big + TOL_G_ABS, (name, err, big)
    assert rms_err <= TOL_G_RMS * rms_ref + TOL_G_ABS, (name, rms_err, rms_ref)


def run_backward(pat, batch, hq, hkv, n, d, seed, scale=0.0):
    print(f"backward case B={pat.block} W={pat.window} S={pat.sink} flags={pat.flags} b={batch} hq={hq} hkv={hkv} "
          f"n={n} d={d}", flush=True)
    q, k, v = synth.qkv(batch, hq, hkv, n, d, "bf16", seed)
    do = synth.gaussian((batch, hq, n, d), "bf16", seed + 1000)
    cnt, idx, _ = pa.mask_build(pat, n)
    qd, kd, vd, dod = q.cuda(), k.cuda(), v.cuda(), do.cuda()
    o, lse = pa.prefill(pat, cnt, idx, qd, kd, vd, softmax_scale=scale)
    need = pa.backward_workspace_bytes(pat, batch, hq, hkv, n, d)
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")      # contents must not matter
    dq, dk, dv = pa.backward(pat, cnt, idx, qd, kd, vd, o, lse, dod, softmax_scale=scale, workspace=ws)
    torch.cuda.synchronize()
    rq, rk, rv = orc.attention_backward(synth.to_numpy_storage(q), synth.to_numpy_storage(k),
                                        synth.to_numpy_storage(v), synth.to_numpy_storage(do),
                                        oracle_pattern(pat), None if scale <= 0 else scale)
    for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        check_grad(name, got.double().cpu().numpy(), ref)


@pytest.mark.parametrize("B,W,S,flags,hq,hkv,n,d", [
    (64, 2, 1, pa.POWER, 4, 2, 1024, 128),
    (64, 4, 0, pa.POWER, 2, 2, 1000, 128),        # no sink, ragged tail, no GQA
    (128, 4, 1, pa.POWER, 8, 2, 2048, 128),       # the long-prefill block size, GQA 4
    (256, 5, 1, pa.POWER, 4, 1, 2048, 64),        # the paper's setting; head_dim 64
    (64, 3, 2, 0, 6, 2, 777, 128),                # sliding window + two sink blocks, GQA 3, ragged
    (64, 0, 1, pa.POWER, 2, 1, 1536, 64),         # W = 0
])
def test_gradients_match_oracle(B, W, S, flags, hq, hkv, n, d):
    run_backward(pa.Pattern(B, W, S, flags), 1, hq, hkv, n, d, seed=51)


def test_batch_and_scale():
    run_backward(pa.Pattern(64, 4, 1), 2, 4, 2, 1280, 128, seed=52, scale=0.07)


def test_sink_column_longer_than_one_part():
    # 40 query blocks attend the sink block: three parts add up in the fp32 buffer
    run_backward(pa.Pattern(64, 2, 1), 1, 2, 1, 2560, 128, seed=53)


def test_rows_outside_the_sink_blocks_are_reproducible():
    # only the sink blocks' rows of dK/dV are summed with atomics; everything else has a fixed order of operations
    pat = pa.Pattern(64, 4, 1)
    q, k, v = synth.qkv(1, 4, 2, 1536, 128, "bf16", seed=54)
    do = synth.gaussian((1, 4, 1536, 128), "bf16", 55)
    cnt, idx, _ = pa.mask_build(pat, 1536)
    qd, kd, vd, dod = q.cuda(), k.cuda(), v.cuda(), do.cuda()
    o, lse = pa.prefill(pat, cnt, idx, qd, kd, vd)
    a = pa.backward(pat, cnt, idx, qd, kd, vd, o, lse, dod)
    b = pa.backward(pat, cnt, idx, qd, kd, vd, o, lse, dod)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0])
    assert torch.equal(a[1][:, :, 64:], b[1][:, :, 64:]) and torch.equal(a[2][:, :, 64:], b[2][:, :, 64:])
    assert (a[1][:, :, :64].float() - b[1][:, :, :64].float()).abs().max().item() <= 1e-2      # last bits only



def test_prefill_configuration_size_on_sampled_rows_and_keys():
    # configuration 2 at its full size (batch 1, 32/8 heads, N = 32768, block 64, W = 4): the dense oracle does not
    # fit, so sampled query rows (dQ) and sampled keys outside the sink block (dK, dV) of two KV heads are checked
    # against the oracle's sampled form
    pat = pa.Pattern(64, 4, 1)
    hq, hkv, n, d = 32, 8, 32768, 128
    q, k, v = synth.qkv(1, hq, hkv, n, d, "bf16", seed=61)
    do = synth.gaussian((1, hq, n, d), "bf16", 62)
    cnt, idx, _ = pa.mask_build(pat, n)
    qd, kd, vd, dod = q.cuda(), k.cuda(), v.cuda(), do.cuda()
    o, lse = pa.prefill(pat, cnt, idx, qd, kd, vd)
    dq, dk, dv = pa.backward(pat, cnt, idx, qd, kd, vd, o, lse, dod)
    torch.cuda.synchronize()
    rng = np.random.default_rng(63)
    rows = np.unique(np.concatenate([[0, 63, 64, n - 1], rng.integers(0, n, 20)]))
    keys = np.unique(np.concatenate([[64, n - 1, n - 64], 64 * rng.integers(1, n // 64, 2)[:, None].repeat(3, 1).ravel()
                                     + rng.integers(0, 64, 6)]))
    opat = oracle_pattern(pat)
    for kvh in (0, 7):
        hs = slice(4 * kvh, 4 * kvh + 4)
        rq, rk, rv = orc.backward_sample(synth.to_numpy_storage(q[:, hs]), synth.to_numpy_storage(k[:, kvh:kvh + 1]),
                                         synth.to_numpy_storage(v[:, kvh:kvh + 1]), synth.to_numpy_storage(do[:, hs]),
                                         rows, keys, opat)
        got = (dq[:, hs][:, :, rows].double().cpu().numpy(), dk[:, kvh:kvh + 1][:, :, keys].double().cpu().numpy(),
               dv[:, kvh:kvh + 1][:, :, keys].double().cpu().numpy())
        for name, g, ref in zip(("dq", "dk", "dv"), got, (rq, rk, rv)):
            check_grad(f"kv head {kvh} {name}", g, ref)


def test_long_prefill_configuration_size_with_a_row_sparse_upstream_gradient():
    # configuration 3 at its full size (batch 1, 32/8 heads, N = 131072, block 128, W = 4, S = 1): what the bench
    # times as `backward_128k`, i.e. the split-wavefront dK/dV kernel with the sink block's column cut into 64 parts
    # that add up in fp32.  The dense oracle is out of reach and so is the sampled one for sink keys (every query
    # attends them).  Instead dO is zero outside 200 query rows that are spread over all 64 parts: then only those rows
    # contribute to dK and dV (a row with dO = 0 has dS = 0), and the oracle's row-sparse form gives dK and dV of
    # EVERY key: the sink block's rows, the diagonal and window blocks of the sampled rows and their power-of-two
    # blocks, and exact zeros everywhere else; dQ is checked on the sampled rows and must be zero on the others.
    pat = pa.Pattern(128, 4, 1)
    hq, hkv, n, d = 32, 8, 131072, 128
    print("backward at N=131072 B=128 32/8 heads, row-sparse dO", flush=True)
    q, k, v = synth.qkv(1, hq, hkv, n, d, "bf16", seed=2)
    rng = np.random.default_rng(64)
    rows = np.unique(np.concatenate([[0, 127, 128, n - 1], 2048 * np.arange(64) + rng.integers(0, 2048, 64),
                                     rng.integers(0, n, 140)]))
    do_rows = synth.gaussian((1, hq, rows.size, d), "bf16", 65)
    do = torch.zeros((1, hq, n, d), dtype=torch.bfloat16)
    do[:, :, torch.from_numpy(rows)] = do_rows
    cnt, idx, _ = pa.mask_build(pat, n)
    qd, kd, vd, dod = q.cuda(), k.cuda(), v.cuda(), do.cuda()
    o, lse = pa.prefill(pat, cnt, idx, qd, kd, vd)
    dq, dk, dv = pa.backward(pat, cnt, idx, qd, kd, vd, o, lse, dod)
    torch.cuda.synchronize()
    opat = oracle_pattern(pat)
    others = np.setdiff1d(np.arange(n), rows)
    for kvh in (0, 7):
        hs = slice(4 * kvh, 4 * kvh + 4)
        rq, rk, rv = orc.attention_backward_rows(synth.to_numpy_storage(q[:, hs]), synth.to_numpy_storage(k[:, kvh:kvh + 1]),
                                                 synth.to_numpy_storage(v[:, kvh:kvh + 1]),
                                                 synth.to_numpy_storage(do_rows[:, hs]), rows, opat)
        gq = dq[:, hs].double().cpu().numpy()
        gk, gv = dk[:, kvh:kvh + 1].double().cpu().numpy(), dv[:, kvh:kvh + 1].double().cpu().numpy()
        check_grad(f"kv head {kvh} dq (sampled rows)", gq[:, :, rows], rq)
        assert (gq[:, :, others] == 0).all()
        check_grad(f"kv head {kvh} dk (all keys)", gk, rk)
        check_grad(f"kv head {kvh} dv (all keys)", gv, rv)
        check_grad(f"kv head {kvh} dk (sink block)", gk[:, :, :128], rk[:, :, :128])
        check_grad(f"kv head {kvh} dv (sink block)", gv[:, :, :128], rv[:, :, :128])
        # keys that no sampled row attends get exactly nothing
        untouched = (rk == 0).all(axis=-1) & (rv == 0).all(axis=-1)
        assert untouched.sum() > 1000
        assert (gk[untouched] == 0).all() and (gv[untouched] == 0).all()


@pytest.mark.parametrize("B,W,S,flags,hq,hkv,n,d", [
    (64, 4, 1, pa.POWER, 2, 1, 1, 128),           # a single token
    (64, 4, 1, pa.POWER, 2, 2, 65, 64),           # one token into the second block
    (64, 2, 8, pa.POWER, 2, 1, 300, 128),         # more sink blocks than blocks: every column is whole
    (64, 40, 0, pa.POWER, 4, 1, 1100, 128),       # the window covers the whole sequence (full causal attention)
    (128, 1, 1, 0, 16, 1, 700, 64),               # GQA 16, window of the diagonal block only
    (256, 2, 1, pa.POWER, 1, 1, 2100, 128),       # one head, block 256, ragged
])
def test_degenerate_shapes(B, W, S, flags, hq, hkv, n, d):
    run_backward(pa.Pattern(B, W, S, flags), 1, hq, hkv, n, d, seed=57)
