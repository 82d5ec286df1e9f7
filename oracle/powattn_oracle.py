"""CPU float64 oracle for PowerAttention's forward pass and its gradients.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain definition that the GPU library is checked
against.  It is imported by the tests, by the smoke check and by the bench's
CPU-baseline leg, and by nothing on the product path.  It shares no code with
the HIP kernels and imports nothing from the GPU package; inputs come in as
NumPy arrays (float32/float64, or uint16 holding bfloat16 bit patterns).

What it follows:
  * the mask predicate of Algorithm 1 (Section 3.3), evaluated per token pair;
  * Equation 1 (Section 3.1): softmax attention restricted to the attended set,
    logits scaled by 1/sqrt(d_k);
  * the receptive-field / DAG-reachability view of Section 3.1 and Appendix A
    (the sets B_k of blocks reachable in at most k steps);
  * decoding with the same pattern as prefilling (Section 4.1).

Everything is float64.  Nothing here is blocked, fused or reordered: the
attention is a dense N x N score matrix with -inf where the predicate is false.
Every function is pinned by tests/test_oracle_*.py against values the paper
prints, closed forms, library routines and brute force; none is unpinned.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Pattern:
    """Hyper-parameters of the static pattern (Algorithm 1's B and W, plus the
    sink width, which Algorithm 1 and the setting of Section 4.1 fix at one block).

    block  : B, tokens per block
    window : W, block distances 0..W-1 are attended
    sink   : S, the first S key blocks are always attended (paper: 1)
    power  : attend block distances that are powers of two (off = sliding
             window + sink, the first baseline of Section 4.1)
    dense  : full causal attention, A_i = {j <= i} (Section 3.1)
    """
    block: int
    window: int
    sink: int = 1
    power: bool = True
    dense: bool = False


# --------------------------------------------------------------------------
# Algorithm 1: the mask predicate
# --------------------------------------------------------------------------
def attended(q_idx, kv_idx, pat: Pattern):
    """The attended set of Algorithm 1, for integer arrays q_idx and kv_idx that broadcast together.

    With d = floor(q/B) - floor(kv/B) the block distance, the set is
        causal  and  ( window  or  power  or  sink )
    where causal = {kv <= q}, window = {d < W}, sink = {key inside the first S
    blocks} and power = {d is zero or a power of two}, i.e. the binary form of
    d has at most one digit set (counted directly here: a non-causal pair has
    d < 0 at worst and is excluded by the causal term whatever the other terms
    say, so d is clipped at zero before counting).
    """
    q_idx = np.asarray(q_idx, dtype=np.int64)
    kv_idx = np.asarray(kv_idx, dtype=np.int64)
    causal = kv_idx <= q_idx
    if pat.dense:
        return causal
    q_blk, kv_blk = q_idx // pat.block, kv_idx // pat.block
    d = q_blk - kv_blk
    members = (d < pat.window) | (kv_blk < pat.sink)
    if pat.power:
        members = members | (np.bitwise_count(np.maximum(d, 0)) <= 1)
    return causal & members


def token_mask(seq_len: int, pat: Pattern):
    """The full seq_len x seq_len boolean mask M[q, kv] (small seq_len only)."""
    q = np.arange(seq_len, dtype=np.int64)[:, None]
    kv = np.arange(seq_len, dtype=np.int64)[None, :]
    return attended(q, kv, pat)


def token_mask_rows(rows, kv_len: int, pat: Pattern):
    """Rows `rows` of the mask against keys 0..kv_len-1."""
    q = np.asarray(rows, dtype=np.int64)[:, None]
    kv = np.arange(kv_len, dtype=np.int64)[None, :]
    return attended(q, kv, pat)


def n_blocks(seq_len: int, pat: Pattern) -> int:
    return -(-seq_len // pat.block)


def block_mask(seq_len: int, pat: Pattern, exhaustive: bool = False):
    """nb x nb boolean matrix: block (i, j) is set when some token of query
    block i attends some token of key block j.

    exhaustive=True reduces the full token mask (O(N^2), small N only).
    Otherwise only the last token of each query block is evaluated against all
    keys: inside one query block the window/power/sink terms of Algorithm 1
    depend on the query through floor(q/B) alone, and the causal term q >= kv
    only grows with q, so the block's last token attends a superset of what any
    other token of the block attends.  Tests check the two agree.
    """
    B = pat.block
    nb = n_blocks(seq_len, pat)
    if exhaustive:
        M = token_mask(seq_len, pat)
        pad = nb * B - seq_len
        M = np.pad(M, ((0, pad), (0, pad)))
        return M.reshape(nb, B, nb, B).any(axis=(1, 3))
    last = np.minimum((np.arange(nb, dtype=np.int64) + 1) * B, seq_len) - 1
    out = np.zeros((nb, nb), dtype=bool)
    pad = nb * B - seq_len
    for i in range(nb):
        row = token_mask_rows([last[i]], seq_len, pat)[0]
        row = np.pad(row, (0, pad))
        out[i] = row.reshape(nb, B).any(axis=1)
    return out


def block_lists(seq_len: int, pat: Pattern, exhaustive: bool = False):
    """Per query block, the ascending list of attended key blocks.

    Returns (kv_cnt[nb] int32, kv_idx[nb, max_k] int32 padded with -1, max_k)
    where max_k is the longest list.
    """
    bm = block_mask(seq_len, pat, exhaustive=exhaustive)
    nb = bm.shape[0]
    cnt = bm.sum(axis=1).astype(np.int32)
    max_k = int(cnt.max()) if nb else 0
    idx = np.full((nb, max_k), -1, dtype=np.int32)
    for i in range(nb):
        js = np.flatnonzero(bm[i])
        idx[i, : js.size] = js
    return cnt, idx, max_k


# --------------------------------------------------------------------------
# Section 3.1 / Appendix A: receptive field as reachability in the DAG
# --------------------------------------------------------------------------
def reach_depth(adj):
    """adj[i, j] = node i attends node j (one layer).  Returns an int matrix
    depth[i, j] = the least number of layers after which information of j can
    have arrived at i (0 on the diagonal, -1 when j is never reachable).

    R_0 = I, R_k = R_{k-1} or (R_{k-1} . adj) over the boolean semiring.
    """
    adj = np.asarray(adj, dtype=bool)
    n = adj.shape[0]
    depth = np.full((n, n), -1, dtype=np.int64)
    reach = np.eye(n, dtype=bool)
    depth[reach] = 0
    k = 0
    while True:
        k += 1
        step = (reach.astype(np.float64) @ adj.astype(np.float64)) > 0
        new = step & ~reach
        if not new.any():
            return depth
        depth[new] = k
        reach |= new


def reach_sets_from(adj, start: int, max_steps: int):
    """Appendix A's B_k for k = 1..max_steps: the nodes reachable from `start`
    in at most k steps (the start node itself belongs to every B_k because the
    diagonal block is always attended)."""
    adj = np.asarray(adj, dtype=bool)
    cur = np.zeros(adj.shape[0], dtype=bool)
    cur[start] = True
    out = []
    for _ in range(max_steps):
        cur = cur | adj[cur].any(axis=0)
        out.append(np.flatnonzero(cur))
    return out


# --------------------------------------------------------------------------
# Equation 1: masked softmax attention
# --------------------------------------------------------------------------
def widen(x):
    """Stored tensor -> float64.  uint16 arrays are bfloat16 bit patterns."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


def _softmax_rows(s, allowed, v):
    """s: [R, L] scaled logits, allowed: [R, L] bool, v: [L, D].
    Returns o[R, D] and lse[R] = ln sum_j exp(s_j) over the attended j."""
    s = np.where(allowed, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    p = np.exp(s - m)
    l = p.sum(axis=1, keepdims=True)
    o = (p @ v) / l
    lse = (m + np.log(l))[:, 0]
    return o, lse


def attention_rows(q, k, v, rows, pat: Pattern, scale=None, q_holds_rows_only=False):
    """Equation 1 for the query positions `rows` only.

    q: [batch, Hq, N, D]; k, v: [batch, Hkv, N, D]; query head h reads KV head
    h // (Hq // Hkv).  Returns o[batch, Hq, len(rows), D], lse[batch, Hq, len(rows)].
    With q_holds_rows_only, q is [batch, Hq, len(rows), D] and already holds just
    the queries at positions `rows` (saves widening a long Q for a few rows).
    """
    q, k, v = widen(q), widen(k), widen(v)
    batch, hq, _, d = q.shape
    n = k.shape[2]
    hkv = k.shape[1]
    g = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    rows = np.asarray(rows, dtype=np.int64)
    allowed = token_mask_rows(rows, n, pat)
    o = np.empty((batch, hq, rows.size, d), dtype=np.float64)
    lse = np.empty((batch, hq, rows.size), dtype=np.float64)
    for b in range(batch):
        for h in range(hq):
            qr = q[b, h] if q_holds_rows_only else q[b, h, rows]
            s = scale * (qr @ k[b, h // g].T)
            o[b, h], lse[b, h] = _softmax_rows(s, allowed, v[b, h // g])
    return o, lse


def attention(q, k, v, pat: Pattern, scale=None):
    """Equation 1 for every query position (dense N x N mask)."""
    n = np.asarray(q).shape[2]
    return attention_rows(q, k, v, np.arange(n), pat, scale)


def decode(q, k_cache, v_cache, kv_len, pat: Pattern, scale=None):
    """One decoding step with the prefill pattern (Section 4.1).

    q: [batch, Hq, D], the query of the newest token; k_cache, v_cache:
    [batch, Hkv, capacity, D] already holding that token's key and value;
    kv_len[b] = number of valid cache positions, so the query sits at position
    kv_len[b] - 1.  Returns o[batch, Hq, D], lse[batch, Hq].
    """
    q, k_cache, v_cache = widen(q), widen(k_cache), widen(v_cache)
    batch, hq, d = q.shape
    hkv = k_cache.shape[1]
    g = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    o = np.empty((batch, hq, d), dtype=np.float64)
    lse = np.empty((batch, hq), dtype=np.float64)
    for b in range(batch):
        length = int(kv_len[b])
        t = length - 1
        allowed = token_mask_rows([t], length, pat)
        for h in range(hq):
            s = scale * (q[b, h][None, :] @ k_cache[b, h // g, :length].T)
            ob, lb = _softmax_rows(s, allowed, v_cache[b, h // g, :length])
            o[b, h], lse[b, h] = ob[0], lb[0]
    return o, lse


# --------------------------------------------------------------------------
# Gradients of Equation 1 (the paper trains with the sparse pattern in place,
# Section 4.1; the gradient of a softmax-weighted sum is textbook calculus)
# --------------------------------------------------------------------------
def attention_backward(q, k, v, do, pat: Pattern, scale=None):
    """Gradients of L = sum(o * do) with o from `attention` (Equation 1).

    With P the row-wise softmax of the masked, scaled logits S = scale * q k^T:
      dV = P^T dO,  dP = dO V^T,  dS = P * (dP - rowsum(P * dP)),
      dQ = scale * dS K,  dK = scale * dS^T Q.
    KV head g receives the sum over the query heads of its group.
    Returns dq [batch, Hq, N, D], dk, dv [batch, Hkv, N, D] in float64.
    """
    q, k, v, do = widen(q), widen(k), widen(v), widen(do)
    batch, hq, n, d = q.shape
    hkv = k.shape[1]
    g = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    allowed = token_mask(n, pat)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for b in range(batch):
        for h in range(hq):
            kh, vh = k[b, h // g], v[b, h // g]
            s = np.where(allowed, scale * (q[b, h] @ kh.T), -np.inf)
            p = np.exp(s - s.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            dp = do[b, h] @ vh.T
            ds = p * (dp - (p * dp).sum(axis=1, keepdims=True))
            dq[b, h] = scale * (ds @ kh)
            dk[b, h // g] += scale * (ds.T @ q[b, h])
            dv[b, h // g] += p.T @ do[b, h]
    return dq, dk, dv


def backward_sample(q, k, v, do, rows, keys, pat: Pattern, scale=None):
    """The same gradients for a sample only, for sequences too long for the dense N x N form:
    dq at the query positions `rows`, dk and dv at the key positions `keys`.

    dq_i needs row i of P and dP only.  dk_j and dv_j sum over the queries i that attend j; for each of them
    p_ij = exp(s_ij - lse_i) with lse_i from `attention_rows` and Delta_i = sum_d do_id o_id.
    Returns dq [batch, Hq, len(rows), D], dk, dv [batch, Hkv, len(keys), D].
    """
    q, k, v, do = widen(q), widen(k), widen(v), widen(do)
    batch, hq, n, d = q.shape
    hkv = k.shape[1]
    g = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    rows = np.asarray(rows, dtype=np.int64)
    keys = np.asarray(keys, dtype=np.int64)
    dq = np.zeros((batch, hq, rows.size, d))
    dk = np.zeros((batch, hkv, keys.size, d))
    dv = np.zeros((batch, hkv, keys.size, d))
    allowed_rows = token_mask_rows(rows, n, pat)
    # every query that attends at least one sampled key
    allq = np.arange(n, dtype=np.int64)
    att_qk = attended(allq[:, None], keys[None, :], pat)            # [N, len(keys)]
    qs = np.nonzero(att_qk.any(axis=1))[0]
    att_qk = att_qk[qs]
    for b in range(batch):
        for h in range(hq):
            kh, vh = k[b, h // g], v[b, h // g]
            s = np.where(allowed_rows, scale * (q[b, h, rows] @ kh.T), -np.inf)
            p = np.exp(s - s.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            dp = do[b, h, rows] @ vh.T
            ds = p * (dp - (p * dp).sum(axis=1, keepdims=True))
            dq[b, h] = scale * (ds @ kh)
            if keys.size:
                o_q, lse_q = attention_rows(q[b:b + 1, h:h + 1], kh[None, None], vh[None, None], qs, pat, scale)
                delta = (do[b, h, qs] * o_q[0, 0]).sum(axis=1, keepdims=True)
                sk = scale * (q[b, h, qs] @ kh[keys].T)
                pk = np.where(att_qk, np.exp(sk - lse_q[0, 0][:, None]), 0.0)
                dsk = pk * (do[b, h, qs] @ vh[keys].T - delta)
                dk[b, h // g] += scale * (dsk.T @ q[b, h, qs])
                dv[b, h // g] += pk.T @ do[b, h, qs]
    return dq, dk, dv


def attention_backward_rows(q, k, v, do_rows, rows, pat: Pattern, scale=None):
    """The gradients of `attention_backward` for an upstream gradient dO that is zero outside the query
    positions `rows` (do_rows: [batch, Hq, len(rows), D] holds its rows there).

    A query row with dO = 0 has dP = 0 and rowsum(P * dP) = 0, hence dS = 0: it contributes nothing to dQ, dK
    or dV.  So the sums over queries in dK = scale * dS^T Q and dV = P^T dO run over `rows` only, and each of
    those rows is the dense, masked row of Equation 1 against all keys, exactly as in `attention_backward`.
    That keeps sequences far too long for the N x N form within reach, for every key at once (the sink
    blocks' keys included, which every later query attends).
    Returns dq [batch, Hq, len(rows), D] (the other rows of dQ are zero), dk, dv [batch, Hkv, N, D].
    """
    q, k, v, do_rows = widen(q), widen(k), widen(v), widen(do_rows)
    batch, hq, n, d = q.shape
    hkv = k.shape[1]
    g = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    rows = np.asarray(rows, dtype=np.int64)
    allowed = token_mask_rows(rows, n, pat)
    dq = np.zeros((batch, hq, rows.size, d))
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for b in range(batch):
        for h in range(hq):
            kh, vh = k[b, h // g], v[b, h // g]
            qr = q[b, h, rows]
            s = np.where(allowed, scale * (qr @ kh.T), -np.inf)
            p = np.exp(s - s.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            dp = do_rows[b, h] @ vh.T
            ds = p * (dp - (p * dp).sum(axis=1, keepdims=True))
            dq[b, h] = scale * (ds @ kh)
            dk[b, h // g] += scale * (ds.T @ qr)
            dv[b, h // g] += p.T @ do_rows[b, h]
    return dq, dk, dv


def column_lists(seq_len: int, pat: Pattern):
    """For every key block j, the query blocks that attend it, ascending (the columns of the block mask)."""
    bm = block_mask(seq_len, pat)
    return [np.nonzero(bm[:, j])[0].astype(np.int64) for j in range(bm.shape[1])]


# --------------------------------------------------------------------------
# Work count: the bench's CPU-baseline leg checks the library's own count of
# attended block pairs (the basis of its FLOP figure) against this one
# --------------------------------------------------------------------------
def attended_pairs(seq_len: int, pat: Pattern) -> int:
    """Number of (query block, key block) pairs with at least one attended token pair."""
    return int(block_mask(seq_len, pat).sum())
