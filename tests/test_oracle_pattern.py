"""Pins for the oracle's mask predicate, block lists and reachability (CPU only).

Each test checks oracle/powattn_oracle.py against something other than itself:
values the paper prints (tests/golden), Theorem B.1, brute force written with a
different formulation (pure-Python loops, popcount through bin()), or invariants
of the pattern.
"""
import math
import os

import numpy as np
import pytest

from oracle import powattn_oracle as orc
from oracle.powattn_oracle import Pattern

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _data_lines(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def _popcount(x):
    return bin(x).count("1")


def brute_pair(q, kv, B, W, S, power=True, dense=False):
    """Independent statement of the pattern: causal and (near, or block distance
    with a single set bit / zero, or inside the first S blocks)."""
    if kv > q:
        return False
    if dense:
        return True
    d = q // B - kv // B
    if d < W:
        return True
    if kv // B < S:
        return True
    return power and _popcount(d) <= 1


def brute_block_list(i, W, S, power=True):
    """Block-level definition A(i) written as a set union."""
    a = set(j for j in range(i + 1) if i - j < W)
    a |= set(j for j in range(min(S, i + 1)))
    if power:
        a.add(i)
        k = 1
        while k <= i:
            a.add(i - k)
            k *= 2
    return sorted(a)


@pytest.mark.parametrize("B", [1, 2, 4, 16])
@pytest.mark.parametrize("W,S,power", [(1, 0, True), (2, 1, True), (3, 2, True), (5, 1, True),
                                       (0, 0, True), (3, 1, False), (1, 0, False)])
def test_predicate_matches_brute_force(B, W, S, power):
    n = 37 * B if B <= 4 else 200
    pat = Pattern(block=B, window=W, sink=S, power=power)
    M = orc.token_mask(n, pat)
    for q in range(n):
        for kv in range(n):
            assert bool(M[q, kv]) == brute_pair(q, kv, B, W, S, power), (q, kv)


def test_dense_is_lower_triangle():
    M = orc.token_mask(50, Pattern(block=4, window=1, dense=True))
    assert np.array_equal(M, np.tril(np.ones((50, 50), dtype=bool)))


@pytest.mark.parametrize("n,B", [(96, 4), (101, 4), (130, 16), (64, 1), (7, 16)])
@pytest.mark.parametrize("W,S,power", [(2, 1, True), (4, 0, True), (3, 2, False)])
def test_block_mask_shortcut_equals_exhaustive(n, B, W, S, power):
    pat = Pattern(block=B, window=W, sink=S, power=power)
    assert np.array_equal(orc.block_mask(n, pat), orc.block_mask(n, pat, exhaustive=True))


@pytest.mark.parametrize("nb,W,S,power", [(16, 2, 1, True), (16, 2, 0, True), (100, 4, 1, True),
                                          (77, 1, 0, True), (64, 9, 1, False), (33, 3, 3, True)])
def test_block_lists_match_set_definition(nb, W, S, power):
    B = 2
    pat = Pattern(block=B, window=W, sink=S, power=power)
    cnt, idx, max_k = orc.block_lists(nb * B, pat)
    assert idx.shape == (nb, max_k)
    for i in range(nb):
        want = brute_block_list(i, W, S, power)
        assert cnt[i] == len(want)
        assert idx[i, : cnt[i]].tolist() == want
        assert (idx[i, cnt[i]:] == -1).all()
    assert max_k == max(len(brute_block_list(i, W, S, power)) for i in range(nb))


def test_ragged_tail_block_lists():
    # 10 full blocks of 8 tokens + 3 tokens: 11 blocks, last one partial.
    pat = Pattern(block=8, window=2, sink=1)
    cnt, idx, _ = orc.block_lists(83, pat)
    assert cnt.shape == (11,)
    assert idx[10, : cnt[10]].tolist() == brute_block_list(10, 2, 1)


# ---- values the paper prints -------------------------------------------------
def test_paper_budget_five_plus_one_plus_four():
    (n, B, W, S, extra, total), = [[int(x) for x in ln] for ln in _data_lines("power_budget_32k.txt")]
    pat = Pattern(block=B, window=W, sink=S)
    cnt, idx, _ = orc.block_lists(n, pat)
    nb = n // B
    row = idx[nb - 1, : cnt[nb - 1]].tolist()
    assert len(row) == total
    in_window = [j for j in row if nb - 1 - j < W]
    in_sink = [j for j in row if j < S and j not in in_window]
    rest = [j for j in row if j not in in_window and j not in in_sink]
    assert (len(in_window), len(in_sink), len(rest)) == (W, S, extra)
    assert all(_popcount(nb - 1 - j) == 1 for j in rest)
    # the distances of those four: the powers of two at or beyond the window
    assert sorted(nb - 1 - j for j in rest) == [8, 16, 32, 64]


def test_paper_sliding_window_B1_and_accuracy():
    (nb, W, S), b1, (num, den) = [[int(x) for x in ln] for ln in _data_lines("sliding_window_B1.txt")]
    pat = Pattern(block=256, window=W, sink=S, power=False)
    bm = orc.block_mask(nb * 256, pat)
    sets = orc.reach_sets_from(bm, nb - 1, 1)
    assert (sets[0] + 1).tolist() == b1          # paper is 1-indexed
    assert (len(sets[0]), nb) == (num, den)
    assert abs(len(sets[0]) / nb - 0.078125) < 1e-12


def test_paper_full_coverage_within_six_layers():
    (nb, W, S, layers), = [[int(x) for x in ln] for ln in _data_lines("coverage_layers.txt")]
    B = 256
    power = orc.block_mask(nb * B, Pattern(block=B, window=W, sink=S))
    sets = orc.reach_sets_from(power, nb - 1, layers)
    sizes = [len(s) for s in sets]
    assert sizes[-1] == nb and sizes[-2] < nb          # covered at exactly `layers`
    assert sizes[0] == 10
    assert all(a < b for a, b in zip(sizes, sizes[1:]))
    # every query block, not only the last one
    depth = orc.reach_depth(power)
    low = np.tril(np.ones((nb, nb), dtype=bool))
    assert depth[low].min() == 0 and depth[low].max() <= layers
    assert (depth[~low] == -1).all()                   # nothing flows backwards
    # sliding window with the same 10-block budget does not get there (linear growth)
    sw = orc.block_mask(nb * B, Pattern(block=B, window=9, sink=1, power=False))
    sizes_sw = [len(s) for s in orc.reach_sets_from(sw, nb - 1, layers)]
    assert sizes_sw == [10 + 8 * k for k in range(layers)]
    assert sizes_sw[-1] < nb


# ---- Theorem B.1 ---------------------------------------------------------------
@pytest.mark.parametrize("n", [16, 37, 128, 512])
def test_theorem_b1_degree_and_distance(n):
    pat = Pattern(block=1, window=1, sink=0)      # pure edge set i - j = 2^k (plus the self edge)
    adj = orc.token_mask(n, pat)
    logn = math.ceil(math.log2(n))
    out_deg = adj.sum(axis=1) - 1
    assert out_deg.max() <= logn
    depth = orc.reach_depth(adj)
    for i in range(n):
        for j in range(i + 1):
            # shortest path = number of ones in the binary form of i - j
            assert depth[i, j] == _popcount(i - j)
    assert depth.max() <= logn
    if n & (n - 1) == 0:
        assert depth.max() == logn


def test_reach_depth_on_a_chain_and_unreachable():
    # 0 <- 1 <- 2 <- 3 chain: depth = index difference; forward pairs unreachable
    adj = np.eye(4, dtype=bool)
    for i in range(1, 4):
        adj[i, i - 1] = True
    depth = orc.reach_depth(adj)
    for i in range(4):
        for j in range(4):
            assert depth[i, j] == (i - j if j <= i else -1)


# ---- invariants at the benchmark configurations --------------------------------
CONFIGS = [  # (seq_len, B, W, pairs S=1, pairs S=0, max_k S=1, max_k S=0, depth S=1, depth S=0)
    (1024, 64, 2, 76, 65, 6, 5, 3, 4),
    (32768, 64, 4, 5619, 5118, 12, 11, 8, 8),
    (131072, 128, 4, 12274, 11262, 13, 12, 9, 9),
    (65536, 64, 4, 12274, 11262, 13, 12, 9, 9),
]


@pytest.mark.parametrize("cfg", CONFIGS)
def test_config_counts_and_invariants(cfg):
    n, B, W, pairs1, pairs0, mk1, mk0, dep1, dep0 = cfg
    nb = n // B
    for S, pairs, mk, dep in ((1, pairs1, mk1, dep1), (0, pairs0, mk0, dep0)):
        pat = Pattern(block=B, window=W, sink=S)
        cnt, idx, max_k = orc.block_lists(n, pat)
        # independent count by the set definition
        assert int(cnt.sum()) == sum(len(brute_block_list(i, W, S)) for i in range(nb)) == pairs
        assert max_k == mk
        bound = W + S + max(0, int(math.floor(math.log2(nb - 1))) - int(math.ceil(math.log2(W))) + 1)
        assert max_k <= bound
        for i in range(nb):
            row = idx[i, : cnt[i]]
            assert (np.diff(row) > 0).all()                       # ascending, unique
            assert row[-1] == i and row[0] >= 0                   # causal, diagonal present
            assert set(range(max(0, i - W + 1), i + 1)) <= set(row.tolist())   # window complete
            for j in row:
                assert i - j < W or j < S or _popcount(i - j) == 1
        # multi-layer coverage (Section 3.1, Appendix A, Theorem B.1): the worst pair needs `dep` layers, which
        # stays within ceil(log2 nb) and far below the 28 layers of the layer-stack configuration
        depth = orc.reach_depth(orc.block_mask(n, pat))
        assert depth.max() == dep
        assert dep <= math.ceil(math.log2(nb)) <= 28
        # the library-facing work count equals the set-union count
        assert orc.attended_pairs(n, pat) == pairs


@pytest.mark.parametrize("n,B,W,S,power", [(96, 4, 2, 1, True), (101, 4, 3, 0, True), (130, 16, 2, 2, False),
                                           (64, 1, 1, 0, True), (7, 16, 4, 1, True)])
def test_attended_pairs_counts_nonempty_blocks_of_the_token_mask(n, B, W, S, power):
    # brute force on small sequences: count block pairs holding at least one attended token pair, one token
    # pair at a time with the independent predicate above (also with a ragged last block)
    pat = Pattern(block=B, window=W, sink=S, power=power)
    nb = -(-n // B)
    want = sum(any(brute_pair(q, kv, B, W, S, power)
                   for q in range(i * B, min((i + 1) * B, n)) for kv in range(j * B, min((j + 1) * B, n)))
               for i in range(nb) for j in range(nb))
    assert orc.attended_pairs(n, pat) == want
    assert orc.attended_pairs(n, Pattern(block=B, window=W, dense=True)) == nb * (nb + 1) // 2


def test_decode_row_of_config_four():
    # 65536-token cache, 64-token blocks, W=4, S=1: the query sits in block 1023
    pat = Pattern(block=64, window=4, sink=1)
    row = orc.token_mask_rows([65535], 65536, pat)[0]
    blocks = np.flatnonzero(row.reshape(1024, 64).any(axis=1)).tolist()
    assert blocks == brute_block_list(1023, 4, 1)
    assert blocks == [0, 511, 767, 895, 959, 991, 1007, 1015, 1019, 1020, 1021, 1022, 1023]
    assert int(row.sum()) == 13 * 64      # every listed block fully visible to the last token


# ---- planted mistakes must be caught by the pins above ------------------------
def test_pins_catch_planted_mistakes(monkeypatch):
    """Break the oracle's predicate in plausible ways (on the CPU) and check
    that the paper-derived pins notice."""
    good = orc.attended

    def no_sink(q, kv, pat):
        return good(q, kv, Pattern(pat.block, pat.window, 0, pat.power, pat.dense))

    def window_inclusive(q, kv, pat):   # blk <= W instead of blk < W
        return good(q, kv, Pattern(pat.block, pat.window + 1, pat.sink, pat.power, pat.dense))

    def token_distance(q, kv, pat):     # power of two in tokens, not blocks
        q = np.asarray(q, dtype=np.int64)
        kv = np.asarray(kv, dtype=np.int64)
        d = q - kv
        base = good(q, kv, Pattern(pat.block, pat.window, pat.sink, False, pat.dense))
        return base | ((q >= kv) & ((d & (d - 1)) == 0))

    def any_pin_fails():
        pins = (test_paper_budget_five_plus_one_plus_four,
                test_paper_sliding_window_B1_and_accuracy,
                test_paper_full_coverage_within_six_layers,
                lambda: test_theorem_b1_degree_and_distance(37),
                lambda: test_predicate_matches_brute_force(4, 2, 1, True))
        for pin in pins:
            try:
                pin()
            except AssertionError:
                return True
        return False

    for bad in (no_sink, window_inclusive, token_distance):
        monkeypatch.setattr(orc, "attended", bad)
        assert any_pin_fails(), bad.__name__
        monkeypatch.setattr(orc, "attended", good)
    assert not any_pin_fails()
