"""Pins for the oracle's gradients (CPU only).

attention_backward is checked against things that do not share its formula: central finite differences of the
oracle's own forward pass (a different function, itself pinned elsewhere), torch's autograd through a library
softmax with the mask applied (float64), invariants (no gradient reaches unattended keys; rows of dS sum to
zero, so adding a constant to all attended keys' logits changes nothing), and planted mistakes.
"""
import math

import numpy as np
import pytest
import torch

from oracle import powattn_oracle as orc
from oracle.powattn_oracle import Pattern


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _loss(q, k, v, do, pat, scale):
    o, _ = orc.attention(q, k, v, pat, scale)
    return float((o * do).sum())


@pytest.mark.parametrize("B,W,S,power,hq,hkv", [(4, 2, 1, True, 2, 1), (3, 1, 0, True, 2, 2), (4, 3, 1, False, 4, 2)])
def test_against_finite_differences_of_the_forward_pass(B, W, S, power, hq, hkv):
    batch, n, d = 1, 22, 5
    q, k, v = _rand((batch, hq, n, d), 1), _rand((batch, hkv, n, d), 2), _rand((batch, hkv, n, d), 3)
    do = _rand((batch, hq, n, d), 4)
    pat = Pattern(B, W, S, power=power)
    scale = 0.37
    dq, dk, dv = orc.attention_backward(q, k, v, do, pat, scale)
    rng = np.random.default_rng(5)
    eps = 1e-6
    for name, x, gx in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for _ in range(25):
            idx = tuple(int(rng.integers(0, s)) for s in x.shape)
            old = x[idx]
            x[idx] = old + eps
            lp = _loss(q, k, v, do, pat, scale)
            x[idx] = old - eps
            lm = _loss(q, k, v, do, pat, scale)
            x[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - gx[idx]) < 1e-7 * max(1.0, abs(fd)), (name, idx, fd, gx[idx])


@pytest.mark.parametrize("B,W,S,power,hq,hkv", [(8, 2, 1, True, 4, 2), (8, 3, 0, True, 3, 1), (16, 2, 1, False, 2, 2)])
def test_against_autograd_through_a_library_softmax(B, W, S, power, hq, hkv):
    batch, n, d = 2, 100, 8
    q, k, v = _rand((batch, hq, n, d), 6), _rand((batch, hkv, n, d), 7), _rand((batch, hkv, n, d), 8)
    do = _rand((batch, hq, n, d), 9)
    pat = Pattern(B, W, S, power=power)
    dq, dk, dv = orc.attention_backward(q, k, v, do, pat)
    tq, tk, tv = (torch.from_numpy(x).clone().requires_grad_(True) for x in (q, k, v))
    g = hq // hkv
    mask = torch.from_numpy(orc.token_mask(n, pat))
    s = (tq @ tk.repeat_interleave(g, dim=1).transpose(-1, -2)) / math.sqrt(d)
    p = torch.softmax(s.masked_fill(~mask, float("-inf")), dim=-1)
    o = p @ tv.repeat_interleave(g, dim=1)
    (o * torch.from_numpy(do)).sum().backward()
    assert np.abs(dq - tq.grad.numpy()).max() < 1e-12
    assert np.abs(dk - tk.grad.numpy()).max() < 1e-12
    assert np.abs(dv - tv.grad.numpy()).max() < 1e-12


def test_no_gradient_reaches_keys_nobody_attends_to():
    # with S = 0 and W = 1 the last block's keys are only seen by the last block's queries: zero dO there
    # and those keys get no gradient at all
    batch, hq, hkv, n, d, B = 1, 2, 1, 64, 4, 8
    q, k, v = _rand((batch, hq, n, d), 10), _rand((batch, hkv, n, d), 11), _rand((batch, hkv, n, d), 12)
    do = _rand((batch, hq, n, d), 13)
    do[:, :, n - B:] = 0.0
    dq, dk, dv = orc.attention_backward(q, k, v, do, Pattern(B, 1, 0))
    assert np.all(dk[:, :, n - B:] == 0.0) and np.all(dv[:, :, n - B:] == 0.0)
    assert np.all(dq[:, :, n - B:] == 0.0)
    assert np.abs(dk[:, :, : n - B]).max() > 0


def test_gradients_are_linear_in_do_and_dv_needs_no_softmax_derivative():
    batch, hq, hkv, n, d = 1, 2, 2, 40, 4
    q, k, v = _rand((batch, hq, n, d), 14), _rand((batch, hkv, n, d), 15), _rand((batch, hkv, n, d), 16)
    do1, do2 = _rand((batch, hq, n, d), 17), _rand((batch, hq, n, d), 18)
    pat = Pattern(8, 2, 1)
    a = orc.attention_backward(q, k, v, do1, pat)
    b = orc.attention_backward(q, k, v, do2, pat)
    c = orc.attention_backward(q, k, v, 2.0 * do1 - 3.0 * do2, pat)
    for x, y, z in zip(a, b, c):
        assert np.abs(2.0 * x - 3.0 * y - z).max() < 1e-12
    # dV_j = sum_i P_ij dO_i: with dO = e_c on one query row only, dV's column c is that row of P
    do = np.zeros((batch, hq, n, d)); do[0, 1, 33, 2] = 1.0
    _, _, dv = orc.attention_backward(q, k, v, do, pat)
    allowed = orc.token_mask(n, pat)[33]
    s = np.where(allowed, (q[0, 1, 33] @ k[0, 1].T) / math.sqrt(d), -np.inf)
    prob = np.exp(s - s.max()); prob /= prob.sum()
    assert np.abs(dv[0, 1, :, 2] - prob).max() < 1e-14
    assert np.all(dv[0, 0] == 0.0)


def test_column_lists_are_the_transposed_row_lists():
    for n, pat in ((1000, Pattern(16, 3, 1)), (512, Pattern(8, 0, 0)), (777, Pattern(16, 2, 2, power=False))):
        cnt, idx, _ = orc.block_lists(n, pat)
        cols = orc.column_lists(n, pat)
        nb = cnt.shape[0]
        back = [[] for _ in range(nb)]
        for i in range(nb):
            for j in idx[i, : cnt[i]]:
                back[j].append(i)
        for j in range(nb):
            assert cols[j].tolist() == back[j]


def test_planted_mistakes_in_the_backward_are_caught(monkeypatch):
    batch, hq, hkv, n, d = 1, 2, 1, 24, 4
    q, k, v = _rand((batch, hq, n, d), 19), _rand((batch, hkv, n, d), 20), _rand((batch, hkv, n, d), 21)
    do = _rand((batch, hq, n, d), 22)
    pat = Pattern(4, 2, 1)
    good = orc.attention_backward(q, k, v, do, pat, 0.5)

    def fd_check(grads):
        eps, rng = 1e-6, np.random.default_rng(23)
        for x, gx in zip((q, k, v), grads):
            for _ in range(12):
                idx = tuple(int(rng.integers(0, s)) for s in x.shape)
                old = x[idx]
                x[idx] = old + eps; lp = _loss(q, k, v, do, pat, 0.5)
                x[idx] = old - eps; lm = _loss(q, k, v, do, pat, 0.5)
                x[idx] = old
                if abs((lp - lm) / (2 * eps) - gx[idx]) > 1e-6:
                    return False
        return True

    assert fd_check(good)
    dq, dk, dv = good
    assert not fd_check((dq / 0.5, dk, dv))                  # dropped scale
    assert not fd_check((dq, dk.copy()[:, :, ::-1], dv))     # transposed / reversed operand
    assert not fd_check((dq, dk, dv * (1 + 1e-3)))           # slightly wrong dV


def test_sampled_form_equals_the_dense_form():
    batch, hq, hkv, n, d = 2, 4, 2, 150, 8
    q, k, v = _rand((batch, hq, n, d), 24), _rand((batch, hkv, n, d), 25), _rand((batch, hkv, n, d), 26)
    do = _rand((batch, hq, n, d), 27)
    for pat in (Pattern(8, 2, 1), Pattern(16, 3, 0), Pattern(8, 2, 2, power=False)):
        dq, dk, dv = orc.attention_backward(q, k, v, do, pat, 0.3)
        rows = np.array([0, 7, 8, 64, 100, 149])
        keys = np.array([0, 3, 8, 15, 16, 77, 148, 149])
        sq, sk, sv = orc.backward_sample(q, k, v, do, rows, keys, pat, 0.3)
        assert np.abs(sq - dq[:, :, rows]).max() < 1e-12
        assert np.abs(sk - dk[:, :, keys]).max() < 1e-12
        assert np.abs(sv - dv[:, :, keys]).max() < 1e-12



def test_row_sparse_form_equals_the_dense_form_with_do_zero_elsewhere():
    # attention_backward_rows is pinned to attention_backward (itself pinned by finite differences and autograd):
    # with dO zero outside the sampled rows the dense form must give the same dK, dV for EVERY key and the same
    # dQ on the rows, and exactly zero dQ elsewhere; and autograd through a library softmax agrees as well
    batch, hq, hkv, n, d = 2, 4, 2, 150, 8
    q, k, v = _rand((batch, hq, n, d), 34), _rand((batch, hkv, n, d), 35), _rand((batch, hkv, n, d), 36)
    rows = np.array([0, 7, 8, 63, 64, 100, 149])
    do = np.zeros((batch, hq, n, d))
    do[:, :, rows] = _rand((batch, hq, rows.size, d), 37)
    for pat in (Pattern(8, 2, 1), Pattern(16, 3, 0), Pattern(8, 2, 2, power=False)):
        dq, dk, dv = orc.attention_backward(q, k, v, do, pat, 0.3)
        rq, rk, rv = orc.attention_backward_rows(q, k, v, do[:, :, rows], rows, pat, 0.3)
        assert np.abs(rq - dq[:, :, rows]).max() < 1e-12
        assert np.abs(rk - dk).max() < 1e-12 and np.abs(rv - dv).max() < 1e-12
        others = np.setdiff1d(np.arange(n), rows)
        assert (dq[:, :, others] == 0).all()
    pat = Pattern(8, 2, 1)
    tq, tk, tv = (torch.from_numpy(x).clone().requires_grad_(True) for x in (q, k, v))
    mask = torch.from_numpy(orc.token_mask(n, pat))
    s = (tq @ tk.repeat_interleave(2, dim=1).transpose(-1, -2)) / math.sqrt(d)
    o = torch.softmax(s.masked_fill(~mask, float("-inf")), dim=-1) @ tv.repeat_interleave(2, dim=1)
    (o * torch.from_numpy(do)).sum().backward()
    rq, rk, rv = orc.attention_backward_rows(q, k, v, do[:, :, rows], rows, pat)
    assert np.abs(rq - tq.grad.numpy()[:, :, rows]).max() < 1e-12
    assert np.abs(rk - tk.grad.numpy()).max() < 1e-12 and np.abs(rv - tv.grad.numpy()).max() < 1e-12
