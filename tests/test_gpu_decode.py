"""GPU parity: powattn_decode (split-K over the attended blocks) vs the oracle.
Bar: max abs error 2e-2 on the outputs (bf16), 1e-3 on the log-sum-exp."""
import numpy as np
import pytest
import torch

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa
from paper_2503_03588_amd import synth
from gpu_util import TOL_LSE, TOL_O, oracle_pattern

pytestmark = pytest.mark.gpu


def run_decode(pat, batch, hq, hkv, cap, d, kv_len, seed, scale=0.0, calls=1):
    q, k, v = synth.decode_inputs(batch, hq, hkv, cap, d, "bf16", seed)
    lens = torch.tensor(kv_len, dtype=torch.int32)
    ws = pa.decode_workspace(pat, batch, hq, hkv, d, cap)
    ws.fill_(0xFF)                  # the library must not rely on the workspace's contents (0xFF.. = NaN)
    qd, kd, vd, ld = q.cuda(), k.cuda(), v.cuda(), lens.cuda()
    for c in range(calls):          # the workspace is reused: counters must come back to zero, and
        if c < calls - 1:           # partials of an earlier call with other data must not leak into this one
            pa.decode(pat, -qd, vd, kd, ld, softmax_scale=scale, workspace=ws)
        o, lse = pa.decode(pat, qd, kd, vd, ld, softmax_scale=scale, workspace=ws)
    torch.cuda.synchronize()
    go, glse = o.double().cpu().numpy(), lse.double().cpu().numpy()
    assert np.isfinite(go).all() and np.isfinite(glse).all()
    oo, olse = orc.decode(synth.to_numpy_storage(q), synth.to_numpy_storage(k), synth.to_numpy_storage(v),
                          np.asarray(kv_len), oracle_pattern(pat), None if scale <= 0 else scale)
    err_o, err_l = np.abs(go - oo).max(), np.abs(glse - olse).max()
    assert err_o <= TOL_O["bf16"], err_o
    assert err_l <= TOL_LSE, err_l
    return qd, kd, vd, ld, go, glse


@pytest.mark.parametrize("B,W,S,hq,hkv,d,cap,kv_len", [
    (64, 4, 1, 8, 2, 128, 4096, [4096, 4095, 1, 64, 65, 2049, 3000, 100]),
    (64, 4, 0, 4, 1, 128, 2048, [2048, 1025]),
    (128, 4, 1, 8, 2, 128, 4096, [4096, 129, 128, 127]),          # two 64-token chunks per block
    (256, 5, 1, 4, 2, 64, 8192, [8192, 5000, 300]),               # paper's block size; head_dim 64
    (64, 2, 1, 7, 1, 128, 3000, [3000, 2999, 777]),               # GQA 7: two heads per wavefront; ragged capacity
    (64, 4, 1, 16, 1, 128, 1024, [1000]),                         # GQA 16
    (64, 3, 1, 2, 2, 128, 2048, [2048, 1]),                       # no GQA
    (64, 0, 0, 4, 2, 128, 4096, [4096, 4033]),                    # W = 0
    (192, 3, 1, 4, 2, 128, 2304, [2304, 1000, 193, 192]),         # a block size that is no power of two: three chunks per block
    (512, 2, 1, 4, 1, 128, 4096, [4096, 513]),                    # eight chunks per block
    (1024, 2, 1, 2, 1, 64, 4096, [4096, 3000]),                   # the largest block
])
def test_shapes_and_lengths(B, W, S, hq, hkv, d, cap, kv_len):
    run_decode(pa.Pattern(B, W, S), len(kv_len), hq, hkv, cap, d, kv_len, seed=31, calls=2)


def test_sliding_window_flag_and_scale():
    run_decode(pa.Pattern(64, 5, 1, flags=0), 2, 4, 2, 2048, 128, [2048, 900], seed=32, scale=0.11)


@pytest.mark.parametrize("B,hq,hkv,d,cap,kv_len", [
    (64, 8, 2, 128, 8192, [8192, 8191, 4097, 65, 1]),      # up to 128 chunks per (sequence, KV head)
    (128, 4, 1, 64, 16384, [16384, 9000]),                   # up to 256 chunks
])
def test_window_over_the_whole_cache_is_full_attention(B, hq, hkv, d, cap, kv_len):
    # a sliding window of as many blocks as the cache has attends every key: the dense decode step that bench.py
    # times beside the sparse one
    run_decode(pa.Pattern(B, cap // B + 1, 0, flags=0), len(kv_len), hq, hkv, cap, d, kv_len, seed=34, calls=2)


def test_peaked_scores():
    # softmax scale 1 on N(0,1) inputs: logits with a standard deviation of ~11, nearly one-hot rows; 25 chunks per
    # row, so a wavefront meets larger and larger maxima over its passes and the workgroups' partials differ widely
    run_decode(pa.Pattern(64, 20, 1), 3, 8, 2, 4096, 128, [4096, 3000, 70], seed=34, scale=1.0)


def test_config4_shape_reduced_batch():
    # config 4 (batch 16, 32/8 heads, 65536-token cache) at batch 2 so the oracle and the upload stay small
    run_decode(pa.Pattern(64, 4, 1), 2, 32, 8, 65536, 128, [65536, 65535], seed=3)


def test_context_of_131072_tokens():
    # the metric's context length: 14 attended blocks per row (one more power-of-two distance than at 65536)
    run_decode(pa.Pattern(64, 4, 1), 2, 32, 8, 131072, 128, [131072, 131071 - 64], seed=4)


def test_decode_replayed_from_a_hip_graph():
    # The call keeps no per-call state on the host (the generation numbers of the merge live in the workspace), so
    # a captured launch can be replayed: capture one decode step per entry point, replay each several times with
    # eager calls on the same inputs and changed inputs in between, and compare every replay with the eager result.
    pat = pa.Pattern(64, 4, 1)
    batch, hq, hkv, cap, d = 4, 8, 2, 8192, 128
    q, k, v = synth.decode_inputs(batch, hq, hkv, cap, d, "bf16", 91)
    q2 = synth.decode_inputs(batch, hq, hkv, cap, d, "bf16", 92)[0]
    lens = torch.tensor([8192, 5000, 4097, 130], dtype=torch.int32).cuda()
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    ws = pa.decode_workspace(pat, batch, hq, hkv, d, cap)
    ref1, rl1 = pa.decode(pat, qd, kd, vd, lens)
    ref2, rl2 = pa.decode(pat, q2.cuda(), kd, vd, lens)
    torch.cuda.synchronize()
    ref1, rl1, ref2, rl2 = ref1.clone(), rl1.clone(), ref2.clone(), rl2.clone()
    qs = qd.clone()                                    # static input of the graphs
    o_g = torch.empty_like(qd); l_g = torch.empty((batch, hq), dtype=torch.float32, device="cuda")
    o_s = torch.empty_like(qd); l_s = torch.empty((batch, hq), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm up on the capture stream (one-time launch set-up)
        pa.decode(pat, qs, kd, vd, lens, o=o_g, lse=l_g, workspace=ws, stream=side)
        pa.decode_static(pat, qs, kd, vd, lens, o_s, l_s, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g1, g2 = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(g1):
        pa.decode(pat, qs, kd, vd, lens, o=o_g, lse=l_g, workspace=ws)
    with torch.cuda.graph(g2):
        pa.decode_static(pat, qs, kd, vd, lens, o_s, l_s)
    for rep in range(6):
        src, want, want_l = (qd, ref1, rl1) if rep % 2 == 0 else (q2.cuda(), ref2, rl2)
        qs.copy_(src)
        o_g.fill_(float("nan")); o_s.fill_(float("nan"))
        g1.replay()
        torch.cuda.synchronize()
        assert torch.equal(o_g, want) and torch.equal(l_g, want_l), rep
        # eager work of the program between the replays, on the same workspace and on the library's own buffer
        e, _ = pa.decode(pat, src, kd, vd, lens, workspace=ws)
        assert torch.equal(e, want)
        g2.replay()
        torch.cuda.synchronize()
        assert torch.equal(o_s, want) and torch.equal(l_s, want_l), rep


def test_decode_equals_prefill_row():
    pat = pa.Pattern(64, 4, 1)
    n, hq, hkv, d = 2048, 8, 2, 128
    q, k, v = synth.qkv(1, hq, hkv, n, d, "bf16", seed=33)
    cnt, idx, _ = pa.mask_build(pat, n)
    o, lse = pa.prefill(pat, cnt, idx, q.cuda(), k.cuda(), v.cuda())
    for t in (2047, 1984, 1000, 63, 0):
        od, ld = pa.decode(pat, q[:, :, t].contiguous().cuda(), k.cuda(), v.cuda(),
                           torch.tensor([t + 1], dtype=torch.int32).cuda())
        torch.cuda.synchronize()
        assert (od.float() - o[:, :, t].float()).abs().max().item() <= 2e-2
        assert (ld - lse[:, :, t]).abs().max().item() <= 1e-3


def test_out_of_range_lengths_are_clamped():
    pat = pa.Pattern(64, 4, 1)
    qd, kd, vd, _, go, glse = run_decode(pat, 2, 4, 2, 1024, 128, [1024, 1], seed=34)
    bad = torch.tensor([5000, -3], dtype=torch.int32).cuda()      # clamped to [1, capacity]
    o, lse = pa.decode(pat, qd, kd, vd, bad)
    torch.cuda.synchronize()
    assert np.array_equal(o.double().cpu().numpy(), go)


def test_full_size_config4():
    # batch 16, 32 q / 8 kv heads, 65536-token caches; random draws happen on the GPU to keep the upload
    # small, and the oracle sees the same bits copied back (only the attended blocks matter).
    pat = pa.Pattern(64, 4, 1)
    batch, hq, hkv, cap, d = 16, 32, 8, 65536, 128
    g = torch.Generator(device="cuda"); g.manual_seed(3)
    k = torch.randn(batch, hkv, cap, d, device="cuda", dtype=torch.bfloat16, generator=g)
    v = torch.randn(batch, hkv, cap, d, device="cuda", dtype=torch.bfloat16, generator=g)
    q = torch.randn(batch, hq, d, device="cuda", dtype=torch.bfloat16, generator=g)
    lens = torch.full((batch,), cap, dtype=torch.int32, device="cuda")
    lens[1] = cap - 37
    o, lse = pa.decode(pat, q, k, v, lens)
    torch.cuda.synchronize()
    for b in (0, 1, 15):
        oo, ol = orc.decode(synth.to_numpy_storage(q[b:b + 1]), synth.to_numpy_storage(k[b:b + 1]),
                            synth.to_numpy_storage(v[b:b + 1]), [int(lens[b])], orc.Pattern(64, 4, 1))
        assert np.abs(o[b:b + 1].double().cpu().numpy() - oo).max() <= 2e-2
        assert np.abs(lse[b:b + 1].double().cpu().numpy() - ol).max() <= 1e-3


def test_many_sequences():
    # 4160 (sequence, KV head) pairs of two workgroups each; sequences are checked at both ends and in the middle
    pat = pa.Pattern(64, 4, 1)
    batch, hq, hkv, cap, d = 520, 8, 8, 4096, 128
    g = torch.Generator(device="cuda"); g.manual_seed(35)
    k = torch.randn(batch, hkv, cap, d, device="cuda", dtype=torch.bfloat16, generator=g)
    v = torch.randn(batch, hkv, cap, d, device="cuda", dtype=torch.bfloat16, generator=g)
    q = torch.randn(batch, hq, d, device="cuda", dtype=torch.bfloat16, generator=g)
    lens = torch.full((batch,), cap, dtype=torch.int32, device="cuda")
    lens[7] = cap - 100
    o, lse = pa.decode(pat, q, k, v, lens)
    torch.cuda.synchronize()
    for b in (0, 7, 300, 519):
        oo, ol = orc.decode(synth.to_numpy_storage(q[b:b + 1]), synth.to_numpy_storage(k[b:b + 1]),
                            synth.to_numpy_storage(v[b:b + 1]), [int(lens[b])], orc.Pattern(64, 4, 1))
        assert np.abs(o[b:b + 1].double().cpu().numpy() - oo).max() <= 2e-2
        assert np.abs(lse[b:b + 1].double().cpu().numpy() - ol).max() <= 1e-3


def test_back_to_back_calls_on_one_workspace():
    # a call must not take the partials that the call before left in the workspace for its own (they carry the
    # previous generation number): alternate two different inputs many times and compare with fresh results
    pat = pa.Pattern(64, 4, 1)
    batch, hq, hkv, cap, d = 4, 8, 2, 8192, 128
    qa, ka, va = synth.decode_inputs(batch, hq, hkv, cap, d, "bf16", 36)
    qb, kb, vb = synth.decode_inputs(batch, hq, hkv, cap, d, "bf16", 37)
    lens = torch.tensor([8192, 8000, 4097, 64], dtype=torch.int32).cuda()
    A = [t.cuda() for t in (qa, ka, va)]
    Bt = [t.cuda() for t in (qb, kb, vb)]
    ws = pa.decode_workspace(pat, batch, hq, hkv, d, cap)
    ref_a = pa.decode(pat, *A, lens)[0].clone()
    ref_b = pa.decode(pat, *Bt, lens)[0].clone()
    torch.cuda.synchronize()
    for i in range(40):
        o, _ = pa.decode(pat, *(A if i % 2 == 0 else Bt), lens, workspace=ws)
        assert torch.equal(o, ref_a if i % 2 == 0 else ref_b), i


def test_many_calls_in_flight_on_several_streams():
    # 96 calls on four streams, each call with a workspace of its own (calls that may overlap must not share
    # one; beyond that the library sets no limit on calls in flight): every output equals the one computed alone,
    # which is checked against the oracle.
    pat = pa.Pattern(64, 4, 1)
    batch, hq, hkv, cap, d = 3, 8, 2, 8192, 128
    cases = []
    for seed, lens in ((81, [8192, 5000, 64]), (82, [8191, 4097, 1]), (83, [6000, 8192, 129])):
        q, k, v = synth.decode_inputs(batch, hq, hkv, cap, d, "bf16", seed)
        oo, olse = orc.decode(synth.to_numpy_storage(q), synth.to_numpy_storage(k), synth.to_numpy_storage(v),
                              np.asarray(lens), oracle_pattern(pat), None)
        dev = [t.cuda() for t in (q, k, v, torch.tensor(lens, dtype=torch.int32))]
        o, lse = pa.decode(pat, *dev)
        torch.cuda.synchronize()
        assert np.abs(o.double().cpu().numpy() - oo).max() <= TOL_O["bf16"]
        assert np.abs(lse.double().cpu().numpy() - olse).max() <= TOL_LSE
        cases.append((dev, o.clone(), lse.clone()))
    streams = [torch.cuda.Stream() for _ in range(4)]
    n_calls = 96
    wss = [pa.decode_workspace(pat, batch, hq, hkv, d, cap) for _ in range(n_calls)]
    for i, w in enumerate(wss):
        w.fill_(i & 0xFF)               # whatever a fresh allocation may hold
    torch.cuda.synchronize()
    outs = []
    for i in range(n_calls):
        dev, _, _ = cases[i % 3]
        st = streams[i % 4]
        with torch.cuda.stream(st):
            outs.append(pa.decode(pat, *dev, workspace=wss[i], stream=st))
    torch.cuda.synchronize()
    for i, (o, lse) in enumerate(outs):
        _, ro, rl = cases[i % 3]
        assert torch.equal(o, ro) and torch.equal(lse, rl), i


def test_more_splits_than_the_workgroups_merge_among_themselves():
    # one sequence and a long row: with 21 and 75 workgroups per (sequence, KV head) the partials are left as plain
    # numbers for the merge kernel; with 10 the workgroups merge among themselves in two rounds of loads
    for B, W, cap in ((64, 40, 8192), (64, 150, 16384)):
        run_decode(pa.Pattern(B, W, 1), 1, 4, 1, cap, 128, [cap], seed=84, calls=2)
    run_decode(pa.Pattern(128, 4, 1), 1, 8, 2, 16384, 128, [16384], seed=85, calls=3)


@pytest.mark.parametrize("B,W,S,hq,hkv,d,cap,batch", [
    (64, 4, 1, 8, 4, 128, 2048, 288),      # 288 x 4 x 2 splits = 2304 work items on 256 compute units
    (128, 4, 1, 8, 2, 64, 4096, 200),      # two chunks per block, head_dim 64, three splits
    (64, 3, 2, 4, 4, 128, 1024, 300),      # one query head per KV head
    (64, 4, 1, 8, 4, 128, 512, 300),       # rows of at most 8 chunks: one split, outputs written without a merge kernel
    (64, 4, 1, 32, 2, 128, 1536, 260),     # 16 query heads per KV head: the largest LDS footprint
    (64, 20, 1, 8, 4, 128, 4096, 300),     # rows of up to 26 chunks: a (sequence, KV head) pair is walked in four passes
    (256, 5, 1, 4, 4, 64, 8192, 270),      # the paper's block size: four chunks per block, up to 40 chunks, five passes
    (256, 6, 1, 4, 2, 64, 8192, 120),      # 240 pairs (fewer than compute units) of five splits: 1200 one-pass items + merge kernel
])
def test_large_batches_on_persistent_workgroups(B, W, S, hq, hkv, d, cap, batch):
    # With at least four work items (sequence, KV head, split) per compute unit the library streams the items through
    # persistent workgroups (the next chunk's loads are issued before the current item is merged, lengths and pages
    # are read ahead): with at least one (sequence, KV head) pair per compute unit a pair is one item walked in
    # passes of eight chunks and the outputs come out of the same kernel; with fewer pairs the splits stay and a
    # second kernel merges them.  Every sequence is checked, with lengths at both ends, around block boundaries and
    # at random.
    pat = pa.Pattern(B, W, S)
    rng = np.random.default_rng(61)
    kv_len = rng.integers(1, cap + 1, size=batch)
    kv_len[:8] = [1, 2, B - 1, B, B + 1, cap, cap - 1, 2 * B]
    kv_len = [int(x) for x in kv_len]
    q, k, v = synth.decode_inputs(batch, hq, hkv, cap, d, "bf16", seed=62)
    lens = torch.tensor(kv_len, dtype=torch.int32).cuda()
    ws = pa.decode_workspace(pat, batch, hq, hkv, d, cap)
    ws.fill_(0xFF)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    o, lse = pa.decode(pat, qd, kd, vd, lens, workspace=ws)
    o2, lse2 = pa.decode(pat, qd, kd, vd, lens, workspace=ws)          # same workspace again: same result
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(lse, lse2)
    go, glse = o.double().cpu().numpy(), lse.double().cpu().numpy()
    assert np.isfinite(go).all() and np.isfinite(glse).all()
    oo, olse = orc.decode(synth.to_numpy_storage(q), synth.to_numpy_storage(k), synth.to_numpy_storage(v),
                          np.asarray(kv_len), oracle_pattern(pat), None)
    assert np.abs(go - oo).max() <= TOL_O["bf16"]
    assert np.abs(glse - olse).max() <= TOL_LSE
    # the same sequences eight at a time take the one-workgroup-per-item kernel: same numbers up to the order
    # in which the splits are merged
    for b0 in (0, 8, batch - 8):
        ob, lb = pa.decode(pat, qd[b0:b0 + 8].contiguous(), kd[b0:b0 + 8].contiguous(), vd[b0:b0 + 8].contiguous(),
                           lens[b0:b0 + 8].contiguous())
        assert (ob.float() - o[b0:b0 + 8].float()).abs().max().item() <= 1e-2
        assert (lb - lse[b0:b0 + 8]).abs().max().item() <= 1e-5
