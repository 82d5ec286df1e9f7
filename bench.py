#!/usr/bin/env python3
"""Benchmark of the PowerAttention hot path on one MI355X.

One "step" = one pass of the method's path over one batch of synthetic input:
  block-index generation (powattn_mask_build)
  + sparse prefill at 128K context (configuration 3: batch 1, 32 query / 8 KV heads,
    head_dim 128, seq 131072, block 128, window 4, sink 1, bf16 N(0,1))
  + one decode step (configuration 4: batch 16, 32/8 heads, 65536-token bf16 caches,
    block 64, window 4, sink 1), rotating over several distinct caches so the reads come from HBM.
The in-library dense causal kernel (the comparison leg) and the CPU oracle are timed outside
the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-dense] [--no-sustained]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E peak

# HBM traffic of one prefill launch at the default workload, from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs scaled by a copy kernel of known size (profiles/prefill_bf16_128k_pmc.md).
# read 4.33 GB + written 1.09 GB per launch.
PREFILL_TRAFFIC_BYTES = 5.43e9
# The same for one decode launch at the default workload (profiles/decode_b16_64k_pmc.md):
# read 55.5 MB (the partials that the merging workgroups read back included) + written 0.79 MB.
DECODE_TRAFFIC_BYTES = 56.3e6


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-sustained", action="store_true")
    ap.add_argument("--dense-iters", type=int, default=2)
    ap.add_argument("--decode-caches", type=int, default=6)
    ap.add_argument("--cpu-rows", type=int, default=512)
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one elementwise copy of 1 GiB (reads 1 GiB, writes 1 GiB): the reference "
                         "dispatch for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2503_03588_amd import binding as pa
    from paper_2503_03588_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"

    # ---------------- workload ----------------
    P = dict(batch=1, hq=32, hkv=8, n=131072, d=128, B=128, W=4, S=1, seed=2)          # configuration 3
    # configuration 4: 65536 tokens in every cache.  The caches are allocated with room for one more block
    # (generation appends): with a capacity of exactly 2^16 tokens the slabs of the 128 (sequence, KV head) pairs
    # lie 16 MB apart and every pair's attended blocks fall on the same HBM channels and banks (measured: 18.7 us
    # per step instead of 15.8).
    Dc = dict(batch=16, hq=32, hkv=8, len=65536, cap=65536 + 64, d=128, B=64, W=4, S=1, seed=3)
    pat_p = pa.Pattern(P["B"], P["W"], P["S"])
    pat_d = pa.Pattern(Dc["B"], Dc["W"], Dc["S"])

    q, k, v = synth.qkv(P["batch"], P["hq"], P["hkv"], P["n"], P["d"], "bf16", P["seed"])
    qg, kg, vg = q.to(dev), k.to(dev), v.to(dev)
    og = torch.empty_like(qg)
    lseg = torch.empty((P["batch"], P["hq"], P["n"]), dtype=torch.float32, device=dev)
    nb = pa.num_blocks(pat_p, P["n"])
    mk = pa.max_k(pat_p, P["n"])
    cnt = torch.empty((nb,), dtype=torch.int32, device=dev)
    idx = torch.empty((nb, mk), dtype=torch.int32, device=dev)

    gen = torch.Generator(device=dev)
    gen.manual_seed(Dc["seed"])
    # all caches in one allocation each for K and V, so that the same memory can also be addressed as a pool of pages
    kall = torch.randn(args.decode_caches, Dc["batch"], Dc["hkv"], Dc["cap"], Dc["d"], device=dev,
                       dtype=torch.bfloat16, generator=gen)
    vall = torch.randn(args.decode_caches, Dc["batch"], Dc["hkv"], Dc["cap"], Dc["d"], device=dev,
                       dtype=torch.bfloat16, generator=gen)
    caches = [(kall[c], vall[c]) for c in range(args.decode_caches)]
    qd = torch.randn(Dc["batch"], Dc["hq"], Dc["d"], device=dev, dtype=torch.bfloat16, generator=gen)
    lens = torch.full((Dc["batch"],), Dc["len"], dtype=torch.int32, device=dev)
    od = torch.empty_like(qd)
    lsed = torch.empty((Dc["batch"], Dc["hq"]), dtype=torch.float32, device=dev)
    ws = pa.decode_workspace(pat_d, Dc["batch"], Dc["hq"], Dc["hkv"], Dc["d"], Dc["cap"])

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(s, marks=None):
        pa.mask_build(pat_p, P["n"], kv_cnt=cnt, kv_idx=idx)
        if marks is not None:
            marks[0].record()
        pa.prefill(pat_p, cnt, idx, qg, kg, vg, o=og, lse=lseg)
        if marks is not None:
            marks[1].record()
        kc, vc = caches[s % len(caches)]
        pa.decode(pat_d, qd, kc, vc, lens, o=od, lse=lsed, workspace=ws)
        if marks is not None:
            marks[2].record()

    if args.calib_copy:
        src = torch.ones((1 << 28,), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    for s in range(args.warmup):
        step(s)
    torch.cuda.synchronize()
    marks = [(ev(), ev(), ev()) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(s, marks[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    prefill_ms = sum(m[0].elapsed_time(m[1]) for m in marks) / args.steps
    decode_in_step_us = sum(m[1].elapsed_time(m[2]) for m in marks) / args.steps * 1e3

    # Decode as it runs in generation: step after step, each on another cache so that every read is cold.
    # (Inside the step above the decode launch follows a 3 ms prefill and an event record; that figure is
    # reported too, as in_step_us.)
    dec_iters = 20 * len(caches)
    for s in range(2 * len(caches)):
        pa.decode(pat_d, qd, *caches[s % len(caches)], lens, o=od, lse=lsed, workspace=ws)
    torch.cuda.synchronize()
    d0, d1 = ev(), ev()
    d0.record()
    for s in range(dec_iters):
        pa.decode(pat_d, qd, *caches[s % len(caches)], lens, o=od, lse=lsed, workspace=ws)
    d1.record()
    torch.cuda.synchronize()
    decode_us = d0.elapsed_time(d1) * 1e3 / dec_iters

    # The same step over a paged cache (powattn_decode_paged): the caches' memory read as a pool of pages of one
    # block each, every sequence's blocks on random pages of the whole pool (26 GB: cold), several tables in
    # rotation.  Then larger batches on the same pool: the fixed costs of a step (launch, the look-ups that
    # depend on one another, the slowest wavefront) are spread over more bytes.
    kpool = kall.view(-1, Dc["hkv"], Dc["B"], Dc["d"])
    vpool = vall.view(-1, Dc["hkv"], Dc["B"], Dc["d"])
    n_pages, stride = kpool.shape[0], Dc["cap"] // Dc["B"]
    n_row = len(pa.row_host(pat_d, (Dc["len"] - 1) // Dc["B"]))
    paged = []
    for batch in (Dc["batch"], 64, 256):
        tables = [torch.randint(0, n_pages, (batch, stride), dtype=torch.int32, device=dev, generator=gen)
                  for _ in range(4)]
        qb = torch.randn(batch, Dc["hq"], Dc["d"], device=dev, dtype=torch.bfloat16, generator=gen)
        lb = torch.full((batch,), Dc["len"], dtype=torch.int32, device=dev)
        ob = torch.empty_like(qb)
        lseb = torch.empty((batch, Dc["hq"]), dtype=torch.float32, device=dev)
        wsb = pa.decode_workspace(pat_d, batch, Dc["hq"], Dc["hkv"], Dc["d"], Dc["cap"])
        iters = 80
        for s in range(8):
            pa.decode_paged(pat_d, qb, kpool, vpool, tables[s % 4], lb, o=ob, lse=lseb, workspace=wsb)
        torch.cuda.synchronize()
        p0, p1 = ev(), ev()
        p0.record()
        for s in range(iters):
            pa.decode_paged(pat_d, qb, kpool, vpool, tables[s % 4], lb, o=ob, lse=lseb, workspace=wsb)
        p1.record()
        torch.cuda.synchronize()
        us = p0.elapsed_time(p1) * 1e3 / iters
        nbytes = n_row * Dc["B"] * Dc["d"] * 2 * 2 * Dc["hkv"] * batch
        paged.append({"batch": batch, "us_per_step": round(us, 2), "tokens_per_s": round(batch / (us * 1e-6), 1),
                      "GB/s": round(nbytes / (us * 1e-6) / 1e9, 1),
                      "frac_of_hbm_peak": round(nbytes / (us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)})
        del tables, qb, lb, ob, lseb, wsb

    pairs = int(cnt.sum().item())
    f_block = 4.0 * P["B"] * P["B"] * P["d"] * P["hq"] * P["batch"] * pairs      # attended blocks, diagonal whole
    value = f_block / (ms_per_step * 1e-3) / 1e12
    prefill_tflops = f_block / (prefill_ms * 1e-3) / 1e12

    row = pa.row_host(pat_d, (Dc["len"] - 1) // Dc["B"])
    decode_bytes = len(row) * Dc["B"] * Dc["d"] * 2 * 2 * Dc["hkv"] * Dc["batch"]   # attended K and V tokens
    decode_gbs = decode_bytes / (decode_us * 1e-6) / 1e9

    # ---------------- the clock and the power the prefill kernel sustains (outside the timed region) ----------------
    # The kernel runs back to back for about two seconds while rocm-smi / amd-smi (child processes that only read
    # the driver's counters) are polled: the chip holds its package power limit under this kernel and the shader
    # clock settles well below the 2.4 GHz that the published peak assumes.  Best effort: null where a tool or a
    # field is missing.
    sustained = None
    if not args.no_sustained:
        import re
        import subprocess
        import threading

        def tool(cmd):
            try:
                return subprocess.run(cmd, capture_output=True, text=True, timeout=10).stdout
            except Exception:
                return ""

        samples = {"sclk": [], "power": []}
        stop = threading.Event()

        def poll():
            while not stop.is_set():
                m = re.search(r"sclk clock level[^\n]*\((\d+)Mhz\)", tool(["rocm-smi", "--showclocks"]))
                if m:
                    samples["sclk"].append(int(m.group(1)))
                m = re.search(r"SOCKET_POWER:\s*(\d+)\s*W", tool(["amd-smi", "metric", "-p"]))
                if m:
                    samples["power"].append(int(m.group(1)))
                stop.wait(0.2)

        m = re.search(r"Max Graphics Package Power \(W\):\s*([0-9.]+)", tool(["rocm-smi", "-M"]))
        cap_w = float(m.group(1)) if m else None
        n_loop = max(50, int(2000.0 / max(prefill_ms, 0.1)))
        for _ in range(20):
            pa.prefill(pat_p, cnt, idx, qg, kg, vg, o=og, lse=lseg)
        torch.cuda.synchronize()
        th = threading.Thread(target=poll, daemon=True)
        s0, s1 = ev(), ev()
        th.start()
        time.sleep(0.05)
        s0.record()
        for _ in range(n_loop):
            pa.prefill(pat_p, cnt, idx, qg, kg, vg, o=og, lse=lseg)
        s1.record()
        torch.cuda.synchronize()
        stop.set()
        th.join(timeout=15)
        sus_ms = s0.elapsed_time(s1) / n_loop
        # the first sample may predate the loop, the last may follow it: take the median
        med = lambda xs: sorted(xs)[len(xs) // 2] if xs else None
        sustained = {"launches": n_loop, "ms_per_prefill": round(sus_ms, 4),
                     "tflops": round(f_block / (sus_ms * 1e-3) / 1e12, 1),
                     "sclk_mhz_median": med(samples["sclk"]), "sclk_mhz_nominal": 2400,
                     "socket_power_w_median": med(samples["power"]), "package_power_cap_w": cap_w,
                     "samples": len(samples["sclk"])}
        if sustained["sclk_mhz_median"]:
            # the same matrix-core peak scaled to the clock the kernel is given (context; `roofline` keeps the nominal one)
            peak_at_clock = PEAK_MFMA_BF16_TFLOPS * sustained["sclk_mhz_median"] / 2400.0
            sustained["frac_of_peak_at_sustained_clock"] = round(sustained["tflops"] / peak_at_clock, 4)

    # ---------------- dense causal baseline of the same library (outside the timed region) ----------------
    dense = None
    if not args.no_dense:
        pat_dense = pa.Pattern(P["B"], P["W"], P["S"], flags=pa.DENSE)
        o2 = torch.empty_like(qg)
        pa.prefill(pat_dense, None, None, qg, kg, vg, o=o2, want_lse=False)
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(args.dense_iters):
            pa.prefill(pat_dense, None, None, qg, kg, vg, o=o2, want_lse=False)
        e1.record()
        torch.cuda.synchronize()
        dense_ms = e0.elapsed_time(e1) / args.dense_iters
        f_dense = 4.0 * P["d"] * P["hq"] * P["batch"] * (P["n"] * (P["n"] + 1) / 2)
        dense = {"ms": round(dense_ms, 3), "tflops_causal": round(f_dense / (dense_ms * 1e-3) / 1e12, 1),
                 "speedup_sparse_vs_dense": round(dense_ms / prefill_ms, 2),
                 "block_pair_ratio": round((nb * (nb + 1) / 2) / pairs, 2)}
        del o2

    # ---------------- the paper's own setting (Section 4.1: 256-token blocks, 5-block window, sink) over the
    # context lengths of its kernel experiment (Section 4.4 / Figure 3b: 16K-128K): sparse and dense kernel
    # times and their ratio, next to the ratio of attended block pairs; outside the timed region -------------
    sweep = None
    if not args.no_dense:
        sweep = []
        pat_s = pa.Pattern(256, 5, 1)
        pat_sd = pa.Pattern(256, 5, 1, flags=pa.DENSE)
        for n_ctx in (16384, 32768, 65536, 131072):
            qs, ks_, vs_ = qg[:, :, :n_ctx].contiguous(), kg[:, :, :n_ctx].contiguous(), vg[:, :, :n_ctx].contiguous()
            os_ = torch.empty_like(qs)
            c_s, i_s, _ = pa.mask_build(pat_s, n_ctx)

            def timed(fn, iters):
                fn()
                torch.cuda.synchronize()
                a, b = ev(), ev()
                a.record()
                for _ in range(iters):
                    fn()
                b.record()
                torch.cuda.synchronize()
                return a.elapsed_time(b) / iters
            ms_s = timed(lambda: pa.prefill(pat_s, c_s, i_s, qs, ks_, vs_, o=os_, want_lse=False), 5)
            ms_d = timed(lambda: pa.prefill(pat_sd, None, None, qs, ks_, vs_, o=os_, want_lse=False),
                         3 if n_ctx < 131072 else 1)
            nbs = n_ctx // 256
            sweep.append({"n": n_ctx, "sparse_ms": round(ms_s, 4), "dense_ms": round(ms_d, 3),
                          "dense_over_sparse": round(ms_d / ms_s, 2),
                          "block_pair_ratio": round((nbs * (nbs + 1) / 2) / int(c_s.sum().item()), 2)})
            del qs, ks_, vs_, os_

    # ---------------- layer stack (configuration 5): 28 successive sparse-attention layers, 28 query /
    # 4 KV heads, 64K context, block 64, fresh random Q/K/V per layer (no projection weights exist, so the layers
    # are not chained); per-layer kernel time.  Second pass: the hybrid schedule of Section 4.3, in which 2 of
    # every 7 layers keep full attention.  Outside the timed region. ----------------
    # ---------------- gradients (powattn_backward) at the 128K workload: dQ, dK, dV from dO.  FLOPs as the five
    # products of the definition (S, dP, dV, dQ, dK) over the attended block pairs: 2.5 x the forward count; the
    # kernels compute S and dP twice (once per pass), which is not counted. ----------------
    backward = None
    if not args.no_dense:
        dog = torch.randn(qg.shape, device=dev, dtype=torch.bfloat16, generator=gen)
        dqg, dkg, dvg = torch.empty_like(qg), torch.empty_like(kg), torch.empty_like(vg)
        wsb = torch.empty((pa.backward_workspace_bytes(pat_p, P["batch"], P["hq"], P["hkv"], P["n"], P["d"]),),
                          dtype=torch.uint8, device=dev)
        pa.backward(pat_p, cnt, idx, qg, kg, vg, og, lseg, dog, dq=dqg, dk=dkg, dv=dvg, workspace=wsb)
        torch.cuda.synchronize()
        b0, b1 = ev(), ev()
        b0.record()
        for _ in range(3):
            pa.backward(pat_p, cnt, idx, qg, kg, vg, og, lseg, dog, dq=dqg, dk=dkg, dv=dvg, workspace=wsb)
        b1.record()
        torch.cuda.synchronize()
        bms = b0.elapsed_time(b1) / 3
        backward = {"ms": round(bms, 3), "tflops_5_products": round(2.5 * f_block / (bms * 1e-3) / 1e12, 1),
                    "over_forward": round(bms / prefill_ms, 2)}
        del dog, dqg, dkg, dvg, wsb

    stack = None
    if not args.no_dense:
        Ls = dict(layers=28, hq=28, hkv=4, n=65536, d=128, B=64, W=4, S=1)
        pat_l = pa.Pattern(Ls["B"], Ls["W"], Ls["S"])
        pat_ld = pa.Pattern(Ls["B"], Ls["W"], Ls["S"], flags=pa.DENSE)
        c_l, i_l, _ = pa.mask_build(pat_l, Ls["n"])
        gl = torch.Generator(device=dev)
        layers_in = []
        for l in range(Ls["layers"]):
            gl.manual_seed(4000 + l)
            layers_in.append((torch.randn(1, Ls["hq"], Ls["n"], Ls["d"], device=dev, dtype=torch.bfloat16, generator=gl),
                              torch.randn(1, Ls["hkv"], Ls["n"], Ls["d"], device=dev, dtype=torch.bfloat16, generator=gl),
                              torch.randn(1, Ls["hkv"], Ls["n"], Ls["d"], device=dev, dtype=torch.bfloat16, generator=gl)))
        ol = torch.empty_like(layers_in[0][0])

        def run_stack(dense_layers):
            a, b = ev(), ev()
            a.record()
            for l, (ql, kl, vl) in enumerate(layers_in):
                if l in dense_layers:
                    pa.prefill(pat_ld, None, None, ql, kl, vl, o=ol, want_lse=False)
                else:
                    pa.prefill(pat_l, c_l, i_l, ql, kl, vl, o=ol, want_lse=False)
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b)
        run_stack(set())
        ms_sparse = run_stack(set())
        hybrid = {l for l in range(Ls["layers"]) if l % 7 in (0, 3)}          # 2 full-attention layers per 7
        ms_hybrid = run_stack(hybrid)
        ms_full = run_stack(set(range(Ls["layers"])))
        pairs_l = int(c_l.sum().item())
        f_layer = 4.0 * Ls["B"] * Ls["B"] * Ls["d"] * Ls["hq"] * pairs_l
        stack = {"layers": Ls["layers"], "workload": "28q/4kv heads, N=65536, D=128, block 64, W=4, S=1, bf16",
                 "sparse_ms_per_layer": round(ms_sparse / Ls["layers"], 4),
                 "sparse_tflops": round(f_layer * Ls["layers"] / (ms_sparse * 1e-3) / 1e12, 1),
                 "hybrid_2_dense_per_7_ms_total": round(ms_hybrid, 2), "sparse_ms_total": round(ms_sparse, 2),
                 "all_dense_ms_total": round(ms_full, 2)}
        del layers_in, ol

    # ---------------- CPU oracle on a bounded row sample (also the bench's own parity check) ----------------
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import powattn_oracle as orc
        rng = np.random.default_rng(12345)
        rows = sorted(set(rng.integers(0, P["n"], size=args.cpu_rows - 64).tolist())
                      | set(range(P["n"] - 64, P["n"])))
        rows_t = torch.tensor(rows, dtype=torch.long)
        q_rows = synth.to_numpy_storage(q[:, :, rows_t])
        ks, vs = synth.to_numpy_storage(k), synth.to_numpy_storage(v)
        c0 = time.perf_counter()
        oo, olse = orc.attention_rows(q_rows, ks, vs, rows, orc.Pattern(P["B"], P["W"], P["S"]),
                                      q_holds_rows_only=True)
        c1 = time.perf_counter()
        cores = len(os.sched_getaffinity(0))
        if os.environ.get("OMP_NUM_THREADS", "").isdigit():
            cores = min(cores, int(os.environ["OMP_NUM_THREADS"]))
        cpu_tflops = f_block * (len(rows) / P["n"]) / (c1 - c0) / 1e12
        cpu = {"value": cpu_tflops, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
               "sample": f"{len(rows)} query rows (seeded random + the last 64) x all 32 heads of the 128K workload, "
                         f"each against all 131072 keys in float64; {c1 - c0:.1f} s; FLOPs credited as for the GPU "
                         f"(attended blocks only, scaled by rows/N)"}
        go = og[:, :, rows_t.to(dev)].double().cpu().numpy()
        gl = lseg[:, :, rows_t.to(dev)].double().cpu().numpy()
        parity = {"prefill_rows_checked": len(rows) * P["hq"],
                  "max_abs_err_o": float(np.abs(go - oo).max()), "max_abs_err_lse": float(np.abs(gl - olse).max())}

    out = {
        "metric": "sparse-attn prefill effective TFLOP/s (attended blocks only) at 128K",
        "value": round(value, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "step = mask_build + sparse prefill (b1, 32q/8kv heads, N=131072, D=128, block 128, "
                               "W=4, S=1, bf16) + one decode step (b16, 32q/8kv, 65536-token bf16 caches of capacity 65600, "
                               "block 64, W=4, S=1, cold: rotating over %d caches)" % len(caches),
                   "attended_block_pairs": pairs, "flops_per_step": f_block},
        "roofline": {"bound": "mfma", "kernel": "pa_prefill_bf16_kernel", "achieved": round(prefill_tflops, 2),
                     "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(prefill_tflops / PEAK_MFMA_BF16_TFLOPS, 4),
                     "avg_launch_ms": round(prefill_ms, 4), "traffic": PREFILL_TRAFFIC_BYTES},
        "cpu_baseline": cpu,
        "decode": {"tokens_per_s": round(Dc["batch"] / (decode_us * 1e-6), 1), "us_per_step": round(decode_us, 2),
                   "in_step_us": round(decode_in_step_us, 2), "steps_timed": dec_iters,
                   "roofline": {"bound": "hbm", "kernel": "pa_decode_kernel (+ merge)", "achieved": round(decode_gbs, 1),
                                "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(decode_gbs / PEAK_HBM_GBS, 4),
                                "bytes_per_step": decode_bytes, "traffic": DECODE_TRAFFIC_BYTES},
                   "paged_cache_by_batch": paged},
        "dense_baseline": dense,
        "paper_setting_b256_w5_s1": sweep,
        "layer_stack": stack,
        "backward_128k": backward,
        "prefill_sustained": sustained,
        "parity": parity,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
