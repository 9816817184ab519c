#!/usr/bin/env python3
"""Benchmark of the fused parallel-pattern attention forward path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-variants] [--no-cpu]

A step is one forward pass of the whole operator (scoring, modification,
online row normalization, aggregation: one kernel launch) over one batch of
seeded synthetic inputs already resident in HBM.  Prints ONE JSON line.
FLOP convention: 2 * (D_qk + D_v) per visible (query, key) pair.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6  # MI355X dense bf16 MFMA: 256 CU x 2.4 GHz x 4096 flop/clk/CU



def measured_traffic(workload_name):
    """HBM bytes per launch (fetch + write) of the forward kernel on this workload, as `bench.py --profile
    --workload NAME` measured them (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by the same counter's reading
    for a 1 GiB device copy): read from the tracked summary profiles/attn_fwd_<workload>.txt.  None where no summary
    with that measurement exists."""
    from paper_2502_15349_amd.rocprof_harness import read_traffic
    t = read_traffic(os.path.join(ROOT, "profiles", f"attn_fwd_{workload_name}.txt"), "attn_fwd_kernel")
    return None if t is None else t[0] + t[1]



def time_gpu(A, torch, w, Q, K, V, steps, warmup, settle_s=0.4, out_bf16=False):
    """Returns (wall ms per step, mean step ms by HIP events, output, launch info)."""
    O = torch.empty((w.B, w.H_q, w.L_q, w.D_v), dtype=torch.bfloat16 if out_bf16 else torch.float32, device=Q.device)
    h = A.ae_attn_create(B=w.B, H_q=w.H_q, H_kv=w.H_kv, L_q=w.L_q, L_k=w.L_k, D_qk=w.D_qk, D_v=w.D_v,
                         scale=w.scale_value, score_mod=w.score_mod, bias=w.bias, gamma=w.gamma(),
                         norm=w.norm, mask=w.mask, out_dtype="bf16" if out_bf16 else "f32", window=w.window)
    info = A.ae_attn_query(h)
    stream = torch.cuda.current_stream()
    args = (h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), stream.cuda_stream)
    fwd = A.ae_attn_forward
    try:
        # The GPU reaches its working clock only after ~0.1-0.3 s of sustained load and a
        # step lasts a fraction of a millisecond: spin the same call until the clock has
        # settled (not counted as warmup steps), then do the W warmup steps.
        t_settle = time.perf_counter()
        while time.perf_counter() - t_settle < settle_s:
            for _ in range(20):
                fwd(*args)
            torch.cuda.synchronize()
        for _ in range(warmup):
            fwd(*args)
        torch.cuda.synchronize()
        # One pair of events around the K launches, recorded on the stream the kernel is
        # launched on: launches queue back to back, so elapsed / K is the kernel's mean
        # duration (launch gaps included) without an event between every two kernels.
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record(stream)
        for _ in range(steps):
            fwd(*args)
        ev1.record(stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        ker_ms = ev0.elapsed_time(ev1) / steps
    finally:
        A.ae_attn_destroy(h)
    return wall_ms, ker_ms, O, info


def parity_sample(w, Q, K, V, O, n_rows=48, scaled=False):
    """Re-assert parity on sampled rows of one head before reporting.  scaled: errors of
    each row divided by max(1, max |oracle row|), for variants whose outputs are not O(1)."""
    from oracle import attention_head
    rng = np.random.default_rng(7)
    b, h = int(rng.integers(w.B)), int(rng.integers(w.H_q))
    g = w.H_q // w.H_kv
    rows = np.unique(np.concatenate([[0, w.L_q - 1], rng.integers(0, w.L_q, n_rows)])).astype(np.int64)
    gam = w.gamma()
    ref = attention_head(Q[b, h].cpu(), K[b, h // g].cpu(), V[b, h // g].cpu(), scale=w.scale_value,
                         score_mod=w.score_mod, bias=w.bias, gamma_h=None if gam is None else gam[h],
                         norm=w.norm, mask=w.oracle_mask(), rows=rows)
    got = O[b, h].cpu().double().numpy()[rows]
    err = np.abs(got - ref)
    if scaled:
        err = err / np.maximum(1.0, np.abs(ref).max(axis=1, keepdims=True))
    return {"max_abs": float(err.max()), "mean_abs": float(err.mean()), "rows": int(len(rows)), "head": [b, h]}


def cpu_baseline(w, Q, K, V, budget_s=15.0):
    """The fp64 oracle as it stands, timed on the host cores on a bounded
    sample of the same workload: whole heads, full S materialised."""
    import torch
    from oracle import attention_head
    cores = len(os.sched_getaffinity(0))
    torch.set_num_threads(cores)
    g = w.H_q // w.H_kv
    gam = w.gamma()
    done, t0 = 0, time.perf_counter()
    heads = [(b, h) for b in range(w.B) for h in range(w.H_q)]
    for (b, h) in heads:
        attention_head(Q[b, h], K[b, h // g], V[b, h // g], scale=w.scale_value, score_mod=w.score_mod,
                       bias=w.bias, gamma_h=None if gam is None else gam[h], norm=w.norm, mask=w.oracle_mask())
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    flop_per_head = w.mfma_flop() / (w.B * w.H_q)
    return {"value": flop_per_head * done / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{done} of {len(heads)} (batch, head) slices of {w.name}, every query row, "
                      f"full L_q x L_k scores in fp64, {dt:.1f} s; rate counted on the same "
                      f"visible-pair flop as the GPU figure"}


def calib_mfma(A, torch, seconds):
    """Sustained rate of the pure-MFMA calibration kernel (two waves per SIMD on every CU),
    reported per half second so that the settling of the clock is visible."""
    wgs, iters = 256, 20000
    sink = torch.empty(wgs * 512, dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream()
    rates, t0 = [], time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        flop = A.ae_calib_mfma_bf16(sink.data_ptr(), sink.numel() * 4, wgs, iters, stream.cuda_stream)
        b.record(stream)
        torch.cuda.synchronize()
        rates.append((time.perf_counter() - t0, flop / (a.elapsed_time(b) * 1e-3) / 1e12))
    tail = [r for t, r in rates if t > seconds / 2] or [r for _, r in rates]
    return {"calib": "pure bf16 MFMA, operands in registers, 2 waves per SIMD", "seconds": seconds,
            "tflops_first": round(rates[0][1], 1), "tflops_sustained": round(float(np.mean(tail)), 1),
            "nominal_peak": PEAK_BF16_TFLOPS}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c5_mla_causal_softmax",
                    help="benchmark configuration of the contract line (default: the largest single-GPU one)")
    ap.add_argument("--profile", action="store_true",
                    help="instead of running the benchmark in this process, run it under rocprofv3 in child processes "
                         "(kernel trace, FETCH_SIZE, WRITE_SIZE, their 1 GiB copy calibration, SQ counters) and write a "
                         "summary with per-kernel durations, MFMA busy fraction, HBM bytes and GB/s; combines with "
                         "--workload, --backward / --recurrent (and --only)")
    ap.add_argument("--profile-dir", default=os.path.join(ROOT, "gpurun_out", "profiles"),
                    help="where --profile writes <name>.txt (and the raw rocprofv3 output, under <name>_raw/)")
    ap.add_argument("--no-variants", action="store_true", help="skip the per-variant table (other configs)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--table2", action="store_true",
                    help="time the parallel-pattern rows of the paper's Table 2 (batch 1/8, sequence 2k/4k/8k) and print them")
    ap.add_argument("--decode", action="store_true",
                    help="time the paper's decoding row (Table 2: one query row, 16 heads, 192/128) with and without "
                         "split keys and print GB/s against the HBM peak")
    ap.add_argument("--backward", action="store_true",
                    help="time the backward pass (ae_attn_backward: dQ, dK, dV) on the softmax / sigmoid benchmark "
                         "shapes and print TFLOP/s against the bf16 MFMA peak")
    ap.add_argument("--bias-tensor", action="store_true",
                    help="time the forward pass with an additive bias tensor (score_mod bias_tensor) beside the same shape "
                         "without one")
    ap.add_argument("--recurrent", action="store_true",
                    help="time the recurrent pattern (chunk-parallel retention, ae_recurrent_forward) per chunk size, beside "
                         "the parallel form of the same sum; prints one JSON object with a row per shape")
    ap.add_argument("--gated", action="store_true",
                    help="time the recurrent pattern with per-token gates (ae_gated_forward; with --backward: ae_gated_backward; gated retention, Mamba2 SSM, "
                         "retention with a constant decay) on Table 2's recurrent shapes; GB/s against the HBM peak")
    ap.add_argument("--only", default="", help="with --backward: only the shapes whose name contains this")
    ap.add_argument("--calib-copy", type=int, default=0, metavar="MiB",
                    help="instead of the benchmark, run a plain device-to-device copy of this many MiB "
                         "(reference reading for the FETCH_SIZE / WRITE_SIZE counters under rocprofv3)")
    ap.add_argument("--calib-mfma", type=float, default=0.0, metavar="SECONDS",
                    help="instead of the benchmark, run the library's pure-MFMA kernel for this long and print "
                         "the bf16 TFLOP/s the matrix pipes sustain under the board's power limit")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    if a.profile:
        # No GPU call is made in this process: every pass is a child process under rocprofv3.
        from paper_2502_15349_amd.rocprof_harness import profile
        if a.gated and a.backward:
            child, name = ["--gated", "--backward", "--only", a.only], f"gated_recurrent_bwd_{a.only or 'all'}"
            trace_args, pmc_args = ("--steps", "10"), ("--steps", "2")
        elif a.backward:
            child, name = ["--backward", "--only", a.only], f"attn_bwd_{a.only or 'all'}"
            trace_args = pmc_args = ()
        elif a.gated:
            child, name = ["--gated", "--only", a.only], f"gated_recurrent_{a.only or 'all'}"
            trace_args, pmc_args = ("--steps", "20"), ("--steps", "3")
        elif a.recurrent:
            child, name = ["--recurrent", "--only", a.only], f"recurrent_{a.only or 'all'}"
            trace_args, pmc_args = ("--steps", "20"), ("--steps", "3")
        else:
            child, name = ["--workload", a.workload, "--no-variants", "--no-cpu"], f"attn_fwd_{a.workload}"
            trace_args, pmc_args = ("--steps", str(a.steps), "--warmup", str(a.warmup)), ("--steps", "3", "--warmup", "1")
        profile(os.path.abspath(__file__), child, a.profile_dir, name, trace_args=trace_args, pmc_args=pmc_args)
        return

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    from paper_2502_15349_amd import ae_attn as A
    from paper_2502_15349_amd.workloads import CONFIGS, make_inputs

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if a.calib_copy:
        n = a.calib_copy << 20
        src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calib_copy_bytes": n, "reads": n, "writes": n}))
        return
    if a.calib_mfma > 0:
        print(json.dumps(calib_mfma(A, torch, a.calib_mfma)))
        return
    if a.decode:
        # Decoding is bound by reading K and V once: bytes / time against the 8 TB/s HBM peak.
        from paper_2502_15349_amd.workloads import Workload
        rows = []
        for batch in (1, 8):
            for seq in (2048, 4096, 8192):
                w = Workload(f"t2_decode_dsv2_lite_b{batch}_s{seq}", 200 + len(rows), batch, 16, 16, 1, seq, 192, 128, mask="causal")
                Qc, Kc, Vc = make_inputs(w)
                Q, K, V = Qc.to(dev), Kc.to(dev), Vc.to(dev)
                res = {}
                for splits in (0, 2, 4, 8, 16, 32, 64, -1):   # -1: the library's own choice
                    O = torch.empty((w.B, w.H_q, w.L_q, w.D_v), dtype=torch.float32, device=dev)
                    h = A.ae_attn_create(B=w.B, H_q=w.H_q, H_kv=w.H_kv, L_q=w.L_q, L_k=w.L_k, D_qk=w.D_qk, D_v=w.D_v,
                                         scale=w.scale_value, mask=w.mask, kv_splits=splits)
                    need = A.ae_attn_workspace_bytes(h)
                    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
                    st = torch.cuda.current_stream()
                    args = (h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), 0, ws.data_ptr(), ws.numel(), st.cuda_stream)
                    for _ in range(200):
                        A.ae_attn_forward_split(*args)
                    torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(st)
                    for _ in range(200):
                        A.ae_attn_forward_split(*args)
                    e1.record(st)
                    torch.cuda.synchronize()
                    ms = e0.elapsed_time(e1) / 200
                    par = parity_sample(w, Q, K, V, O, n_rows=1)["max_abs"]
                    if splits == -1:
                        # The same launches replayed from a HIP graph (the library allocates nothing and clears
                        # nothing, so it can be captured): 50 calls per graph, 4 replays timed, every replay's
                        # output compared with the eager one.
                        side = torch.cuda.Stream()
                        gargs = args[:-1] + (side.cuda_stream,)
                        eager = O.clone()
                        graph = torch.cuda.CUDAGraph()
                        side.wait_stream(st)
                        with torch.cuda.graph(graph, stream=side):
                            for _ in range(50):
                                A.ae_attn_forward_split(*gargs)
                        torch.cuda.synchronize()
                        graph.replay()
                        torch.cuda.synchronize()
                        same = bool(torch.equal(O, eager))
                        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        for _ in range(4):
                            O.zero_()
                            graph.replay()
                            torch.cuda.synchronize()
                            same = same and bool(torch.equal(O, eager))
                        g0.record(st)
                        for _ in range(4):
                            graph.replay()
                        g1.record(st)
                        torch.cuda.synchronize()
                        graph_ms = g0.elapsed_time(g1) / 200
                        del graph
                    A.ae_attn_destroy(h)
                    res[splits] = (ms, par)
                byts = w.compulsory_bytes()
                t0, p0 = res[0]
                s1 = min((k for k in res if k > 0), key=lambda k: res[k][0])   # the fastest split count of the sweep
                t1, p1 = res[s1]
                sweep = {("auto" if k < 0 else str(k)): round(v[0], 5) for k, v in sorted(res.items())}
                rows.append({"workload": w.name, "B": batch, "L_k": seq, "bytes": byts, "unsplit_ms": round(t0, 5),
                             "kv_splits": s1, "split_ms": round(t1, 5), "auto_ms": round(res[-1][0], 5),
                             "auto_graph_ms": round(graph_ms, 5), "graph_replays_equal_eager": same,
                             "auto_graph_GBps": round(byts / graph_ms / 1e6, 1), "split_GBps": round(byts / t1 / 1e6, 1),
                             "frac_of_hbm_peak": round(byts / t1 / 1e6 / 8000.0, 4), "parity_max_abs": max(v[1] for v in res.values()),
                             "ms_by_kv_splits": sweep})
                print(f"# {w.name:34s} unsplit {t0:8.4f} ms | {s1:3d} splits {t1:8.4f} ms  {byts / t1 / 1e6:8.1f} GB/s "
                      f"({100 * byts / t1 / 1e6 / 8000.0:4.1f} % of 8 TB/s)  max_abs {max(v[1] for v in res.values()):.2e}  "
                      f"auto from a HIP graph {graph_ms:7.4f} ms {byts / graph_ms / 1e6:7.1f} GB/s (replays equal eager: {same})  sweep {sweep}",
                      file=sys.stderr, flush=True)
        print(json.dumps({"decode": rows, "bound": "hbm", "peak_GBps": 8000.0, "dtype": "bf16", "data": "synthetic"}))
        return
    if a.backward and not a.gated:
        # Not the contract line.  Algorithmic work of the backward pass: five contractions per visible (query, key)
        # pair (S, dP, dV, dK, dQ) = 2 * (3 D_qk + 2 D_v) flop; the key-side and the query-side kernel each recompute
        # S and dP, so the MFMAs they issue amount to 2 * (4 D_qk + 3 D_v) flop per pair.
        from oracle import attention_backward
        from paper_2502_15349_amd.workloads import C2, C3, C4, C5, Workload, make_grad, table2_workloads
        rows = []
        # the benchmark configurations with a backward pass, one unmasked shape, and the paper's Table 2 shapes at
        # batch 8 x 8k (softmax at three head-dim pairs, sigmoid, ReLU)
        shapes = [C2, C3, C4, C5, Workload("t2_softmax_b8_h32_s8192_noncausal", 150, 8, 32, 32, 8192, 8192, 128, 128)]
        shapes += [w for w in table2_workloads() if w.B == 8 and w.L_q == 8192 and w.L_q == w.L_k and w.D_qk <= 192]  # (256/512 has no backward pass)
        for w in shapes:
            if a.only not in w.name:
                continue
            Qc, Kc, Vc = make_inputs(w)
            dOc = make_grad(w)
            Q, K, V, dO = Qc.to(dev), Kc.to(dev), Vc.to(dev), dOc.to(dev)
            has_stat = w.norm in ("softmax", "abssum", "abs_of_sum")
            stats = torch.empty((w.B, w.H_q, w.L_q), dtype=torch.float32, device=dev) if has_stat else None
            O = A.run_workload(w, Q, K, V, stats=stats)
            h = A.ae_attn_create(B=w.B, H_q=w.H_q, H_kv=w.H_kv, L_q=w.L_q, L_k=w.L_k, D_qk=w.D_qk, D_v=w.D_v,
                                 scale=w.scale_value, score_mod=w.score_mod, bias=w.bias, gamma=w.gamma(), norm=w.norm,
                                 mask=w.mask)
            dQ = torch.empty(Q.shape, dtype=torch.float32, device=dev)
            dK = torch.empty(K.shape, dtype=torch.float32, device=dev)
            dV = torch.empty(V.shape, dtype=torch.float32, device=dev)
            ws = torch.empty(max(A.ae_attn_backward_workspace_bytes(h), 16), dtype=torch.uint8, device=dev)
            st = torch.cuda.current_stream()
            args = (h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(),
                    0 if stats is None else stats.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), ws.data_ptr(),
                    ws.numel(), st.cuda_stream)
            t_end = time.perf_counter() + 0.3
            while time.perf_counter() < t_end:
                A.ae_attn_backward(*args)
                torch.cuda.synchronize()
            n = 10
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            for _ in range(n):
                A.ae_attn_backward(*args)
            e1.record(st)
            torch.cuda.synchronize()
            A.ae_attn_destroy(h)
            ms = e0.elapsed_time(e1) / n
            pairs = w.visible_pairs_per_head() * w.B * w.H_q
            alg, issued = 2 * (3 * w.D_qk + 2 * w.D_v) * pairs, 2 * (4 * w.D_qk + 3 * w.D_v) * pairs
            par = None
            if w.L_q <= 4096:   # one (batch, k/v head) group against the oracle
                b, hk, g = w.B - 1, w.H_kv // 2, w.H_q // w.H_kv
                hs = slice(hk * g, hk * g + g)
                ref = attention_backward(Qc[b:b + 1, hs], Kc[b:b + 1, hk:hk + 1], Vc[b:b + 1, hk:hk + 1], dOc[b:b + 1, hs],
                                         scale=w.scale_value, score_mod=w.score_mod, bias=w.bias,
                                         gamma=None if w.gamma() is None else w.gamma()[hs], norm=w.norm, mask=w.mask)
                got = (dQ[b:b + 1, hs], dK[b:b + 1, hk:hk + 1], dV[b:b + 1, hk:hk + 1])
                par = {}
                for name, x, r in zip(("dQ", "dK", "dV"), got, ref):
                    rs = np.maximum(np.abs(r).max(axis=-1, keepdims=True), 1.0)
                    err = np.abs(x.cpu().double().numpy() - r) / rs
                    par[name] = {"max_abs_scaled": float(err.max()), "mean_abs_scaled": float(err.mean())}
            tf = alg / (ms * 1e-3) / 1e12
            rows.append({"workload": w.name, "backward_ms": round(ms, 4), "tflops": round(tf, 1),
                         "frac_of_peak": round(tf / PEAK_BF16_TFLOPS, 4),
                         "issued_mfma_tflops": round(issued / (ms * 1e-3) / 1e12, 1), "flop": alg, "parity": par})
            print(f"# {w.name:40s} backward {ms:9.4f} ms {tf:8.1f} TFLOP/s ({100 * tf / PEAK_BF16_TFLOPS:4.1f} % of peak; "
                  f"MFMAs issued: {issued / (ms * 1e-3) / 1e12:7.1f} TFLOP/s)  parity {par}", file=sys.stderr, flush=True)
            del Q, K, V, dO, O, dQ, dK, dV
        print(json.dumps({"backward": rows, "unit": "TFLOP/s", "peak": PEAK_BF16_TFLOPS, "dtype": "bf16", "data": "synthetic"}))
        return
    if a.bias_tensor:
        # Not the contract line.  The bias tensor [1, H_q, L_q, L_k] (bf16, shared over the batch) is read once per
        # batch element: B * H_q * visible pairs * 2 bytes on top of Q, K, V, O.
        from oracle import attention_head
        from paper_2502_15349_amd.workloads import C2, Workload, make_bias_tensor
        rows = []
        for base in (C2, Workload("softmax_b8_h32_s4096_causal", 160, 8, 32, 32, 4096, 4096, 128, 128, mask="causal"),
                     Workload("softmax_b8_h32_s4096", 161, 8, 32, 32, 4096, 4096, 128, 128)):
            w = base.scaled(score_mod="bias_tensor")
            Qc, Kc, Vc = make_inputs(w)
            Q, K, V = Qc.to(dev), Kc.to(dev), Vc.to(dev)
            bt = make_bias_tensor(w, per_batch=False)
            btd = bt.to(dev)
            O = torch.empty((w.B, w.H_q, w.L_q, w.D_v), dtype=torch.float32, device=dev)
            res = {}
            for name, ww in (("plain", base), ("bias_tensor", w)):
                h = A.ae_attn_create(B=w.B, H_q=w.H_q, H_kv=w.H_kv, L_q=w.L_q, L_k=w.L_k, D_qk=w.D_qk, D_v=w.D_v,
                                     scale=w.scale_value, score_mod=ww.score_mod, mask=w.mask,
                                     bias_stride=(0, btd.stride(1), btd.stride(2)))
                st = torch.cuda.current_stream()

                def call():
                    if name == "plain":
                        A.ae_attn_forward(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), st.cuda_stream)
                    else:
                        A.ae_attn_forward_bias(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), btd.data_ptr(), O.data_ptr(), 0,
                                               st.cuda_stream)
                t_end = time.perf_counter() + 0.3
                while time.perf_counter() < t_end:
                    call()
                    torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(st)
                for _ in range(20):
                    call()
                e1.record(st)
                torch.cuda.synchronize()
                A.ae_attn_destroy(h)
                res[name] = e0.elapsed_time(e1) / 20
            # parity of the bias run on sampled rows of one head
            b, hq = w.B - 1, w.H_q // 2
            rows_s = np.linspace(0, w.L_q - 1, 24).astype(np.int64)
            ref = attention_head(Qc[b, hq], Kc[b, hq // (w.H_q // w.H_kv)], Vc[b, hq // (w.H_q // w.H_kv)], scale=w.scale_value,
                                 score_mod="bias_tensor", mask=w.mask, rows=rows_s, bias_t=bt[0, hq])
            err = float(np.abs(O[b, hq].cpu().double().numpy()[rows_s] - ref).max())
            # the backward pass of the same two problems (dQ, dK, dV; the bias gets no gradient)
            from paper_2502_15349_amd.workloads import make_grad
            dO = make_grad(w).to(dev)
            stats = torch.empty((w.B, w.H_q, w.L_q), dtype=torch.float32, device=dev)
            grads = [torch.empty(x.shape, dtype=torch.float32, device=dev) for x in (Q, K, V)]
            bres = {}
            dB = torch.zeros((w.B, w.H_q, w.L_q, w.L_k), dtype=torch.bfloat16, device=dev)   # the bias gradient, zero-filled once
            for name, ww in (("plain", base), ("bias_tensor", w), ("bias_tensor_dbias", w)):
                A.run_workload(ww, Q, K, V, out=O, stats=stats, bias_tensor=None if name == "plain" else btd)
                h = A.ae_attn_create(B=w.B, H_q=w.H_q, H_kv=w.H_kv, L_q=w.L_q, L_k=w.L_k, D_qk=w.D_qk, D_v=w.D_v,
                                     scale=w.scale_value, score_mod=ww.score_mod, mask=w.mask,
                                     bias_stride=(0, btd.stride(1), btd.stride(2)))
                ws = torch.empty(A.ae_attn_backward_workspace_bytes(h), dtype=torch.uint8, device=dev)
                st = torch.cuda.current_stream()
                tail = (O.data_ptr(), dO.data_ptr(), stats.data_ptr(), grads[0].data_ptr(), grads[1].data_ptr(), grads[2].data_ptr(),
                        ws.data_ptr(), ws.numel(), st.cuda_stream)

                def bcall():
                    if name == "plain":
                        A.ae_attn_backward(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), *tail)
                    elif name == "bias_tensor":
                        A.ae_attn_backward_bias(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), btd.data_ptr(), *tail[:6], 0, 0, *tail[6:])
                    else:
                        A.ae_attn_backward_bias(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), btd.data_ptr(), *tail[:6], dB.data_ptr(), w.L_k,
                                                *tail[6:])
                for _ in range(3):
                    bcall()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(st)
                for _ in range(10):
                    bcall()
                e1.record(st)
                torch.cuda.synchronize()
                A.ae_attn_destroy(h)
                bres[name] = e0.elapsed_time(e1) / 10
            bflop = 2 * (3 * w.D_qk + 2 * w.D_v) * w.visible_pairs_per_head() * w.B * w.H_q
            flop = w.mfma_flop()
            bias_bytes = 2 * w.visible_pairs_per_head() * w.B * w.H_q
            rows.append({"workload": w.name, "plain_ms": round(res["plain"], 4), "bias_tensor_ms": round(res["bias_tensor"], 4),
                         "plain_tflops": round(flop / res["plain"] / 1e9, 1), "bias_tensor_tflops": round(flop / res["bias_tensor"] / 1e9, 1),
                         "bias_GBps": round(bias_bytes / res["bias_tensor"] / 1e6, 1), "parity_max_abs": err,
                         "backward_plain_ms": round(bres["plain"], 4), "backward_bias_tensor_ms": round(bres["bias_tensor"], 4),
                         "backward_bias_tensor_tflops": round(bflop / bres["bias_tensor"] / 1e9, 1),
                         "backward_with_dbias_ms": round(bres["bias_tensor_dbias"], 4)})
            print(f"# {w.name:32s} plain {res['plain']:8.4f} ms {flop / res['plain'] / 1e9:7.1f} TFLOP/s | bias tensor "
                  f"{res['bias_tensor']:8.4f} ms {flop / res['bias_tensor'] / 1e9:7.1f} TFLOP/s ({100 * flop / res['bias_tensor'] / 1e9 / PEAK_BF16_TFLOPS:4.1f} % "
                  f"of peak), bias read at {bias_bytes / res['bias_tensor'] / 1e6:7.1f} GB/s  max_abs {err:.2e} | backward plain "
                  f"{bres['plain']:8.4f} ms, bias tensor {bres['bias_tensor']:8.4f} ms {bflop / bres['bias_tensor'] / 1e9:7.1f} TFLOP/s, "
                  f"with dBias {bres['bias_tensor_dbias']:8.4f} ms",
                  file=sys.stderr, flush=True)
            del Q, K, V, O, btd, dO, grads, dB
        print(json.dumps({"bias_tensor": rows, "unit": "TFLOP/s", "peak": PEAK_BF16_TFLOPS, "dtype": "bf16", "data": "synthetic"}))
        return
    if a.recurrent:
        # Not the contract line.  Retention with a per-head decay as a recurrence: 4 D_qk D_v flop per token (state
        # update and read-out, as the token-by-token definition does them) over 2 (2 D_qk + D_v) + 4 D_v compulsory
        # bytes: about 50 flop per byte at 128/128, far under the chip's 300, so the recurrence is priced against HBM.
        import math
        from oracle.retention_recurrent_oracle import retention_recurrent_head
        from paper_2502_15349_amd.workloads import Workload
        rows = []
        shapes = [("retention_b8_h32_s2048_d128", 8, 32, 2048, 128), ("retention_b8_h32_s8192_d128", 8, 32, 8192, 128),
                  ("retention_b1_h32_s32768_d128", 1, 32, 32768, 128), ("retention_b8_h16_s8192_d64", 8, 16, 8192, 64)]
        for name, B, H, L, D in shapes:
            if a.only and a.only not in name:
                continue
            w = Workload(name, 300 + len(rows), B, H, H, L, L, D, D, score_mod="head_decay", norm="none", mask="causal")
            Qc, Kc, Vc = make_inputs(w)
            Q, K, V = Qc.to(dev), Kc.to(dev), Vc.to(dev)
            gam = [1.0 - 2.0 ** (-5 - (i % 8)) for i in range(H)]   # RetNet's per-head rates, cycled
            scale = 1.0 / math.sqrt(D)
            O = torch.empty((B, H, L, D), dtype=torch.float32, device=dev)
            st = torch.cuda.current_stream()

            def timed(fn, n):
                import time
                t_settle = time.perf_counter()   # (0.2 s of the same call first: the board's clock under this load settles)
                while time.perf_counter() - t_settle < 0.2:
                    for _ in range(3):
                        fn()
                    torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(st)
                for _ in range(n):
                    fn()
                e1.record(st)
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / n
            t_par = timed(lambda: A.attention_forward(Q, K, V, scale=scale, score_mod="head_decay", gamma=gam, norm="none",
                                                      mask="causal", out=O), max(2, a.steps // 4))
            row = {"workload": name, "B": B, "H": H, "L": L, "D_qk": D, "D_v": D, "parallel_form_ms": round(t_par, 4)}
            byts = B * H * L * (2 * (2 * D + D) + 4 * D)
            flop = 4.0 * D * D * B * H * L
            best = None
            for chunk in (64, 128, 256):
                h = A.ae_recurrent_create(B=B, H=H, L=L, D_qk=D, D_v=D, chunk=chunk, scale=scale, gamma=gam)
                ws = torch.empty(max(A.ae_recurrent_workspace_bytes(h), 256), dtype=torch.uint8, device=dev)
                t = timed(lambda: A.ae_recurrent_forward(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), ws.data_ptr(),
                                                         ws.numel(), st.cuda_stream), a.steps)
                if chunk == 256:   # parity of what the last timed call left in O: one head against the oracle
                    b_s, h_s = B - 1, H // 2
                    ref = retention_recurrent_head(Qc[b_s, h_s].float().numpy(), Kc[b_s, h_s].float().numpy(), Vc[b_s, h_s].float().numpy(),
                                                   scale=scale, gamma_h=gam[h_s])
                    got = O[b_s, h_s].cpu().double().numpy()
                    err = float((np.abs(got - ref) / np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1.0)).max())
                A.ae_recurrent_destroy(h)
                row[f"chunk{chunk}_ms"] = round(t, 4)
                if best is None or t < best[1]:
                    best = (chunk, t)
                del ws
            # the same with bf16 output (chunk 256): 2 instead of 4 bytes per output element
            h = A.ae_recurrent_create(B=B, H=H, L=L, D_qk=D, D_v=D, chunk=256, scale=scale, gamma=gam, out_dtype="bf16")
            ws = torch.empty(A.ae_recurrent_workspace_bytes(h), dtype=torch.uint8, device=dev)
            O16 = torch.empty((B, H, L, D), dtype=torch.bfloat16, device=dev)
            row["chunk256_bf16_out_ms"] = round(timed(lambda: A.ae_recurrent_forward(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O16.data_ptr(),
                                                                                      ws.data_ptr(), ws.numel(), st.cuda_stream), a.steps), 4)
            A.ae_recurrent_destroy(h)
            del ws, O16
            row.update({"best_chunk": best[0], "ms": round(best[1], 4), "tokens_per_s": round(B * L / best[1] * 1e3, 1),
                        "GBps": round(byts / best[1] / 1e6, 1), "frac_of_hbm_peak": round(byts / best[1] / 1e6 / 8000.0, 4),
                        "recurrence_tflops": round(flop / best[1] / 1e9, 1), "speedup_vs_parallel_form": round(t_par / best[1], 2),
                        "parity_max_abs": err})
            rows.append(row)
            print(f"# {name:32s} parallel form {t_par:8.4f} ms | chunks 64/128/256: {row['chunk64_ms']:8.4f} {row['chunk128_ms']:8.4f} "
                  f"{row['chunk256_ms']:8.4f} ms | best {best[1]:8.4f} ms = {byts / best[1] / 1e6:7.1f} GB/s "
                  f"({100 * byts / best[1] / 1e6 / 8000.0:4.1f} % of HBM peak), {t_par / best[1]:5.2f}x the parallel form, max_abs {err:.2e}"
                  f" | bf16 out {row['chunk256_bf16_out_ms']:8.4f} ms",
                  file=sys.stderr, flush=True)
            del Q, K, V, O
        # One decoding step on the carried state (ae_recurrent_step): the state is read and written once,
        # 8 bytes per element, which is all the traffic there is.
        steps_rows = []
        for name, B, H, D in (("retention_step_b8_h32_d128", 8, 32, 128), ("retention_step_b64_h32_d128", 64, 32, 128),
                              ("retention_step_b64_h16_d64", 64, 16, 64)):
            if a.only and a.only not in name:
                continue
            g = torch.Generator(device="cpu")
            g.manual_seed(400 + len(steps_rows))
            q, k, v = (torch.randn((B, H, D), generator=g).to(torch.bfloat16).to(dev) for _ in range(3))
            state = torch.zeros((B, H, D, D), dtype=torch.float32, device=dev)
            o = torch.empty((B, H, D), dtype=torch.float32, device=dev)
            h = A.ae_recurrent_create(B=B, H=H, L=1, D_qk=D, D_v=D, chunk=64, scale=1.0 / math.sqrt(D),
                                      gamma=[1.0 - 2.0 ** (-5 - (i % 8)) for i in range(H)])
            st = torch.cuda.current_stream()
            n = 200
            for _ in range(10):
                A.ae_recurrent_step(h, q.data_ptr(), k.data_ptr(), v.data_ptr(), state.data_ptr(), o.data_ptr(), st.cuda_stream)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            for _ in range(n):
                A.ae_recurrent_step(h, q.data_ptr(), k.data_ptr(), v.data_ptr(), state.data_ptr(), o.data_ptr(), st.cuda_stream)
            e1.record(st)
            torch.cuda.synchronize()
            A.ae_recurrent_destroy(h)
            ms = e0.elapsed_time(e1) / n
            byts = 8 * B * H * D * D
            steps_rows.append({"workload": name, "us_per_step": round(ms * 1e3, 2), "tokens_per_s": round(B / ms * 1e3, 1),
                               "GBps": round(byts / ms / 1e6, 1), "frac_of_hbm_peak": round(byts / ms / 1e6 / 8000.0, 4)})
            print(f"# {name:32s} {ms * 1e3:8.2f} us per step = {byts / ms / 1e6:7.1f} GB/s ({100 * byts / ms / 1e6 / 8000.0:4.1f} % of HBM peak)",
                  file=sys.stderr, flush=True)
        print(json.dumps({"recurrent": rows, "recurrent_step": steps_rows, "bound": "hbm", "peak_GBps": 8000.0, "dtype": "bf16",
                          "data": "synthetic"}))
        return
    if a.gated:
        # Not the contract line.  One pass over Q, K, V, the gates and O: compulsory bytes 2 (2 D_qk / g + D_v) + 4 D_v + 8
        # per token and value head (g value heads share a q/k head) against 8 TB/s.
        import math
        from oracle.gated_recurrent_oracle import gated_recurrent_head
        from paper_2502_15349_amd.workloads import Workload, make_gates
        shapes = [  # name, B, H, H_qk, L, D_qk, D_v, gates
            ("gated_retention_b8_h32_s8192_d128", 8, 32, 32, 8192, 128, 128, "gated_retention"),
            ("retention_const_b8_h32_s8192_d128", 8, 32, 32, 8192, 128, 128, "const"),
            ("gated_retention_rfa_b8_h16_s8192_d64", 8, 16, 16, 8192, 64, 64, "gated_retention"),
            ("mamba2_ssm_b8_h80_s8192_128_64", 8, 80, 1, 8192, 128, 64, "mamba2"),
            ("mamba2_ssm_b1_h80_s8192_128_64", 1, 80, 1, 8192, 128, 64, "mamba2"),
            ("gated_retention_b1_h32_s32768_d128", 1, 32, 32, 32768, 128, 128, "gated_retention"),
        ]
        rows = []
        for name, B, H, Hqk, L, Dq, Dv, kind in shapes:
            if a.only and a.only not in name:
                continue
            cid = 500 + len(rows)
            Qc, Kc, _ = make_inputs(Workload("q", cid, B, Hqk, Hqk, L, L, Dq, Dq))
            _, _, Vc = make_inputs(Workload("v", cid, B, H, H, L, L, Dv, Dv))
            if kind == "const":
                gam = torch.tensor([1.0 - 2.0 ** (-5 - (i % 8)) for i in range(H)], dtype=torch.float32)
                lac, kgc = torch.log(gam).view(1, H, 1).expand(B, H, L).contiguous(), None
            else:
                lac, kgc = make_gates(B, H, L, 1000 * cid + 5, kind)
            Q, K, V, la = Qc.to(dev), Kc.to(dev), Vc.to(dev), lac.to(dev)
            kg = None if kgc is None else kgc.to(dev)
            scale = 1.0 / math.sqrt(Dq)
            O = torch.empty((B, H, L, Dv), dtype=torch.float32, device=dev)
            h = A.ae_gated_create(B=B, H=H, H_qk=Hqk, L=L, D_qk=Dq, D_v=Dv, scale=scale)
            st = torch.cuda.current_stream()
            args = (h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), la.data_ptr(), 0 if kg is None else kg.data_ptr(), 0, O.data_ptr(), 0,
                    st.cuda_stream)
            # --gated times the forward pass, --gated --backward the backward pass: one kind of launch per run, so that a
            # profile of the run speaks of one of them
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

            def timed(call, n_warm):
                # (the same call for 0.3 s first: the clock the board holds under this load has to settle, as for the
                # contract line)
                import time
                t_settle = time.perf_counter()
                while time.perf_counter() - t_settle < 0.3:
                    for _ in range(max(n_warm, 4)):
                        call()
                    torch.cuda.synchronize()
                e0.record(st)
                for _ in range(a.steps):
                    call()
                e1.record(st)
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / a.steps

            ngate = 2 if kg is not None else 1
            row = {"workload": name, "B": B, "H": H, "H_qk": Hqk, "L": L, "D_qk": Dq, "D_v": Dv}
            if not a.backward:
                ms = timed(lambda: A.ae_gated_forward(*args), 3)
                b_s, h_s = B - 1, H // 2
                g_s = h_s // (H // Hqk)
                ref = gated_recurrent_head(Qc[b_s, g_s].float().numpy(), Kc[b_s, g_s].float().numpy(), Vc[b_s, h_s].float().numpy(),
                                           lac[b_s, h_s].numpy(), None if kgc is None else kgc[b_s, h_s].numpy(), scale=scale)
                got = O[b_s, h_s].cpu().double().numpy()
                err = float((np.abs(got - ref) / np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1.0)).max())
                # compulsory bytes: Q, K, V and the gates read once, O (fp32) written once
                byts = B * L * (2 * 2 * Dq * Hqk + H * (2 * Dv + 4 * Dv + 4 * ngate))
                flop = 4.0 * Dq * Dv * B * H * L
                row.update({"ms": round(ms, 4), "tokens_per_s": round(B * L / ms * 1e3, 1), "GBps": round(byts / ms / 1e6, 1),
                            "frac_of_hbm_peak": round(byts / ms / 1e6 / 8000.0, 4), "recurrence_tflops": round(flop / ms / 1e9, 1),
                            "compulsory_bytes": byts, "parity_max_abs": err})
                print(f"# {name:40s} {ms:8.4f} ms = {byts / ms / 1e6:7.1f} GB/s ({100 * byts / ms / 1e6 / 8000.0:4.1f} % of HBM peak), "
                      f"{flop / ms / 1e9:6.1f} TFLOP/s of recurrence, max_abs {err:.2e}", file=sys.stderr, flush=True)
                # few heads, long sequence: the same call with the walks cut into segments (ae_gated_forward_segmented)
                nfw = A.ae_gated_workspace_bytes(h)
                if nfw:
                    fws = torch.empty(nfw, dtype=torch.uint8, device=dev)
                    O2 = torch.empty_like(O)
                    sargs = args[:7] + (O2.data_ptr(), 0, fws.data_ptr(), nfw, st.cuda_stream)
                    seg_ms = timed(lambda: A.ae_gated_forward_segmented(*sargs), 3)
                    seg_diff = float((O2 - O).abs().max())
                    del fws, O2
                    row.update({"segmented_ms": round(seg_ms, 4), "segmented_GBps": round(byts / seg_ms / 1e6, 1),
                                "segmented_max_diff_to_single_walk": seg_diff})
                    print(f"#   {'cut into segments':38s} {seg_ms:8.4f} ms = {byts / seg_ms / 1e6:7.1f} GB/s "
                          f"({100 * byts / seg_ms / 1e6 / 8000.0:4.1f} % of HBM peak), max difference to the single walk {seg_diff:.2e}",
                          file=sys.stderr, flush=True)
            else:
                # ae_gated_backward: dQ, dK, dV, dlog_decay, dkey_gate; compulsory bytes: Q, K, V, dO and the gates read
                # once, the gradients (fp32) written once
                from paper_2502_15349_amd.workloads import make_grad
                dO = make_grad(Workload("v", cid, B, H, H, L, L, Dv, Dv)).to(dev)
                f32 = dict(dtype=torch.float32, device=dev)
                dQ, dK, dV = torch.empty(Q.shape, **f32), torch.empty(K.shape, **f32), torch.empty(V.shape, **f32)
                dla = torch.empty((B, H, L), **f32)
                dkg = None if kg is None else torch.empty((B, H, L), **f32)
                nws = A.ae_gated_backward_workspace_bytes(h)
                ws = torch.empty(nws, dtype=torch.uint8, device=dev)
                bargs = (h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), la.data_ptr(), 0 if kg is None else kg.data_ptr(), dO.data_ptr(),
                         dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), dla.data_ptr(), 0 if dkg is None else dkg.data_ptr(), ws.data_ptr(),
                         nws, st.cuda_stream)
                bwd_ms = timed(lambda: A.ae_gated_backward(*bargs), 2)
                bwd_byts = B * L * (Hqk * Dq * (2 * 2 + 2 * 4) + H * Dv * (2 + 2 + 4) + H * 8 * ngate)
                row.update({"backward_ms": round(bwd_ms, 4), "backward_GBps": round(bwd_byts / bwd_ms / 1e6, 1),
                            "backward_frac_of_hbm_peak": round(bwd_byts / bwd_ms / 1e6 / 8000.0, 4),
                            "backward_compulsory_bytes": bwd_byts, "workspace_bytes": nws})
                print(f"# {name:40s} backward {bwd_ms:8.4f} ms = {bwd_byts / bwd_ms / 1e6:7.1f} GB/s "
                      f"({100 * bwd_byts / bwd_ms / 1e6 / 8000.0:4.1f} % of HBM peak)", file=sys.stderr, flush=True)
                del dO, dQ, dK, dV, dla, dkg, ws
            rows.append(row)
            A.ae_gated_destroy(h)
            del Q, K, V, O, la, kg
        print(json.dumps({"gated_recurrent": rows, "bound": "hbm", "peak_GBps": 8000.0, "dtype": "bf16", "data": "synthetic"}))
        return
    if a.table2:
        # Not the contract line: the paper's own microbenchmark grid, one row per shape.
        from paper_2502_15349_amd.workloads import table2_workloads
        rows = []
        for w in table2_workloads():
            Qc, Kc, Vc = make_inputs(w)
            Q, K, V = Qc.to(dev), Kc.to(dev), Vc.to(dev)
            _, ker_ms, O, info = time_gpu(A, torch, w, Q, K, V, 20, 3, settle_s=0.3)
            par = parity_sample(w, Q, K, V, O, n_rows=16, scaled=True)
            tf = w.mfma_flop() / (ker_ms * 1e-3) / 1e12
            rows.append({"workload": w.name, "B": w.B, "H": w.H_q, "L": w.L_q, "D_qk": w.D_qk, "D_v": w.D_v,
                         "norm": w.norm, "score_mod": w.score_mod, "mask": w.mask, "kernel_ms": round(ker_ms, 4),
                         "tflops": round(tf, 1), "frac_of_peak": round(tf / PEAK_BF16_TFLOPS, 4),
                         "parity_max_abs_scaled": par["max_abs"], "kernel": info["kernel"]})
            print(f"# {w.name:40s} {ker_ms:9.4f} ms {tf:8.1f} TFLOP/s {100 * tf / PEAK_BF16_TFLOPS:5.1f} %  "
                  f"max_abs(scaled) {par['max_abs']:.2e}", file=sys.stderr, flush=True)
            del Q, K, V, O
        print(json.dumps({"table2": rows, "unit": "TFLOP/s", "peak": PEAK_BF16_TFLOPS, "dtype": "bf16", "data": "synthetic"}))
        return
    w = CONFIGS[a.workload]
    Qc, Kc, Vc = make_inputs(w)
    Q, K, V = Qc.to(dev), Kc.to(dev), Vc.to(dev)
    torch.cuda.synchronize()
    wall_ms, ker_ms, O, info = time_gpu(A, torch, w, Q, K, V, a.steps, a.warmup)
    par = parity_sample(w, Q, K, V, O)
    flop = w.mfma_flop()
    value = flop / (wall_ms * 1e-3) / 1e12
    achieved = flop / (ker_ms * 1e-3) / 1e12

    out = {
        "metric": "fwd attention TFLOP/s (and fraction of MI355X dense bf16 MFMA peak in roofline.frac)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(wall_ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H_q": w.H_q, "H_kv": w.H_kv, "L_q": w.L_q, "L_k": w.L_k,
                   "D_qk": w.D_qk, "D_v": w.D_v, "score_mod": w.score_mod, "norm": w.norm, "mask": w.mask,
                   "out": "fp32", "entry": "ae_attn_forward",
                   "kernel": info["kernel"], "block_m": info["block_m"], "block_n": info["block_n"],
                   "grid": info["grid_size"], "threads": info["block_threads"], "lds_bytes": info["lds_bytes"]},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": measured_traffic(w.name),
                     "kernel_ms": round(ker_ms, 5), "flop_per_launch": flop,
                     "compulsory_bytes": w.compulsory_bytes(),
                     },
        "parity": par,
    }

    if not a.no_variants:
        variants = {}
        for name, wv in CONFIGS.items():
            if name == w.name:
                variants[name] = {"tflops": round(achieved, 2), "frac_of_peak": round(achieved / PEAK_BF16_TFLOPS, 4),
                                  "kernel_ms": round(ker_ms, 5)}
                continue
            del Q, K, V, O
            torch.cuda.empty_cache()
            q, k, v = make_inputs(wv)
            Q, K, V = q.to(dev), k.to(dev), v.to(dev)
            steps = max(5, min(a.steps, 20))
            _, kms, O, _ = time_gpu(A, torch, wv, Q, K, V, steps, min(a.warmup, 5))
            pv = parity_sample(wv, Q, K, V, O)
            tf = wv.mfma_flop() / (kms * 1e-3) / 1e12
            variants[name] = {"tflops": round(tf, 2), "frac_of_peak": round(tf / PEAK_BF16_TFLOPS, 4),
                              "kernel_ms": round(kms, 5), "parity_max_abs": pv["max_abs"]}
        # the same workload storing bf16 instead of fp32 (half the output bytes)
        del Q, K, V, O
        torch.cuda.empty_cache()
        Q, K, V = Qc.to(dev), Kc.to(dev), Vc.to(dev)
        _, kms, Ob, _ = time_gpu(A, torch, w, Q, K, V, max(5, min(a.steps, 20)), min(a.warmup, 5), out_bf16=True)
        pv = parity_sample(w, Q, K, V, Ob.float())
        tf = flop / (kms * 1e-3) / 1e12
        variants[w.name + "_bf16_out"] = {"tflops": round(tf, 2), "frac_of_peak": round(tf / PEAK_BF16_TFLOPS, 4),
                                          "kernel_ms": round(kms, 5), "parity_max_abs": pv["max_abs"]}
        # the backward pass of the same workload (ae_attn_backward: delta, key-side and query-side kernel), timed the same
        # way; algorithmic flop = 2 (3 D_qk + 2 D_v) per visible pair.  `bench.py --backward` has the other shapes.
        from paper_2502_15349_amd.workloads import make_grad
        stats = torch.empty((w.B, w.H_q, w.L_q), dtype=torch.float32, device=dev)
        Of = A.run_workload(w, Q, K, V, stats=stats)
        dO = make_grad(w).to(dev)
        hb = A.ae_attn_create(B=w.B, H_q=w.H_q, H_kv=w.H_kv, L_q=w.L_q, L_k=w.L_k, D_qk=w.D_qk, D_v=w.D_v, scale=w.scale_value,
                              score_mod=w.score_mod, bias=w.bias, gamma=w.gamma(), norm=w.norm, mask=w.mask)
        grads = [torch.empty(x.shape, dtype=torch.float32, device=dev) for x in (Q, K, V)]
        wsb = torch.empty(max(A.ae_attn_backward_workspace_bytes(hb), 16), dtype=torch.uint8, device=dev)
        st = torch.cuda.current_stream()
        bargs = (hb, Q.data_ptr(), K.data_ptr(), V.data_ptr(), Of.data_ptr(), dO.data_ptr(), stats.data_ptr(), grads[0].data_ptr(),
                 grads[1].data_ptr(), grads[2].data_ptr(), wsb.data_ptr(), wsb.numel(), st.cuda_stream)
        t_end = time.perf_counter() + 0.3
        while time.perf_counter() < t_end:
            A.ae_attn_backward(*bargs)
            torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(20):
            A.ae_attn_backward(*bargs)
        e1.record(st)
        torch.cuda.synchronize()
        A.ae_attn_destroy(hb)
        bms = e0.elapsed_time(e1) / 20
        btf = 2 * (3 * w.D_qk + 2 * w.D_v) * w.visible_pairs_per_head() * w.B * w.H_q / (bms * 1e-3) / 1e12
        variants[w.name + "_backward"] = {"tflops": round(btf, 2), "frac_of_peak": round(btf / PEAK_BF16_TFLOPS, 4),
                                         "ms": round(bms, 5)}
        del grads, dO, Of, wsb
        # the recurrent pattern (ae_recurrent_forward, chunks of 256) on 8 x 32 heads x 8192 tokens, 128/128, priced
        # against HBM: compulsory bytes (Q, K, V once, O once) / time.  `bench.py --recurrent` has the other shapes.
        import math
        from paper_2502_15349_amd.workloads import Workload
        wr = Workload("retention_b8_h32_s8192_d128", 301, 8, 32, 32, 8192, 8192, 128, 128, score_mod="head_decay", norm="none", mask="causal")
        Qr, Kr, Vr = (x.to(dev) for x in make_inputs(wr))
        Or = torch.empty((wr.B, wr.H_q, wr.L_q, wr.D_v), dtype=torch.float32, device=dev)
        hr = A.ae_recurrent_create(B=wr.B, H=wr.H_q, L=wr.L_q, D_qk=128, D_v=128, chunk=256, scale=1.0 / math.sqrt(128),
                                   gamma=[1.0 - 2.0 ** (-5 - (i % 8)) for i in range(wr.H_q)])
        wsr = torch.empty(A.ae_recurrent_workspace_bytes(hr), dtype=torch.uint8, device=dev)
        rargs = (hr, Qr.data_ptr(), Kr.data_ptr(), Vr.data_ptr(), Or.data_ptr(), wsr.data_ptr(), wsr.numel(), st.cuda_stream)
        t_settle = time.perf_counter()   # (the board's clock under this load settles, as for the contract line)
        while time.perf_counter() - t_settle < 0.2:
            for _ in range(3):
                A.ae_recurrent_forward(*rargs)
            torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(20):
            A.ae_recurrent_forward(*rargs)
        e1.record(st)
        torch.cuda.synchronize()
        A.ae_recurrent_destroy(hr)
        rms = e0.elapsed_time(e1) / 20
        rbytes = wr.B * wr.H_q * wr.L_q * (2 * (2 * 128 + 128) + 4 * 128)
        variants[wr.name + "_recurrent"] = {"ms": round(rms, 5), "GBps": round(rbytes / rms / 1e6, 1),
                                            "frac_of_hbm_peak": round(rbytes / rms / 1e6 / 8000.0, 4),
                                            "tokens_per_s": round(wr.B * wr.L_q / rms * 1e3, 1)}
        del Qr, Kr, Vr, Or, wsr
        # the same shape with per-token gates (gated retention: ae_gated_forward, ae_gated_backward); `bench.py --gated`
        # and `--gated --backward` have the other shapes (Mamba2, batch 1)
        from paper_2502_15349_amd.workloads import make_gates, make_grad
        wg = Workload("gated_retention_b8_h32_s8192_d128", 500, 8, 32, 32, 8192, 8192, 128, 128)
        Qg, Kg, Vg = (x.to(dev) for x in make_inputs(wg))
        lag = make_gates(wg.B, wg.H_q, wg.L_q, 500005, "gated_retention")[0].to(dev)
        dOg = make_grad(wg).to(dev)
        f32 = dict(dtype=torch.float32, device=dev)
        Og, dQg, dKg, dVg = (torch.empty(Qg.shape, **f32) for _ in range(4))
        dlag = torch.empty(lag.shape, **f32)
        hg = A.ae_gated_create(B=wg.B, H=wg.H_q, L=wg.L_q, D_qk=128, D_v=128, scale=1.0 / math.sqrt(128))
        nwg = A.ae_gated_backward_workspace_bytes(hg)
        wsg = torch.empty(nwg, dtype=torch.uint8, device=dev)
        fargs = (hg, Qg.data_ptr(), Kg.data_ptr(), Vg.data_ptr(), lag.data_ptr(), 0, 0, Og.data_ptr(), 0, st.cuda_stream)
        bargs = (hg, Qg.data_ptr(), Kg.data_ptr(), Vg.data_ptr(), lag.data_ptr(), 0, dOg.data_ptr(), dQg.data_ptr(), dKg.data_ptr(),
                 dVg.data_ptr(), dlag.data_ptr(), 0, wsg.data_ptr(), nwg, st.cuda_stream)
        for call, cargs, tag, byts in ((A.ae_gated_forward, fargs, "", wg.B * wg.H_q * wg.L_q * (2 * 3 * 128 + 4 * 128 + 4)),
                                       (A.ae_gated_backward, bargs, "_backward", wg.B * wg.H_q * wg.L_q * (2 * 4 * 128 + 4 * 3 * 128 + 8))):
            t_settle = time.perf_counter()
            while time.perf_counter() - t_settle < 0.2:
                for _ in range(2):
                    call(*cargs)
                torch.cuda.synchronize()
            e0.record(st)
            for _ in range(10):
                call(*cargs)
            e1.record(st)
            torch.cuda.synchronize()
            gms = e0.elapsed_time(e1) / 10
            variants[wg.name + tag] = {"ms": round(gms, 5), "GBps": round(byts / gms / 1e6, 1),
                                       "frac_of_hbm_peak": round(byts / gms / 1e6 / 8000.0, 4),
                                       "tokens_per_s": round(wg.B * wg.L_q / gms * 1e3, 1)}
        A.ae_gated_destroy(hg)
        del Qg, Kg, Vg, lag, dOg, Og, dQg, dKg, dVg, dlag, wsg
        out["variants"] = variants

    # What the matrix pipes sustain on this board with nothing else in the way: the library's
    # pure-MFMA kernel, run after the timed work so that it does not disturb it.  Context for frac:
    # the ceiling the board's power limit leaves of the nominal peak.
    cal = calib_mfma(A, torch, 2.0)
    out["roofline"]["mfma_sustained_tflops"] = cal["tflops_sustained"]
    out["roofline"]["frac_of_sustained"] = round(achieved / cal["tflops_sustained"], 4)

    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, Qc, Kc, Vc)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
