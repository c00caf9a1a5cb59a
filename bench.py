#!/usr/bin/env python3
"""Benchmark of the Kunlun attention hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic batch of the headline workload
(BASELINE.json config "Large GDPA forward": B=1024, H=8, d=128, Nq=64, jagged log-normal
history lengths):
    kunlun_gdpa_fwd  (GELU score function, scale 1/tau)       Nq seed/context queries over the history
    kunlun_gdpa_bwd  (dQ, dK, dV of the same call)
    kunlun_swa_fwd   (window = previous 256 tokens)           self-attention over the same histories
Inputs are resident in HBM before the timed region; the scheduler kernels are inside it.

Prints ONE JSON line.  `value` = the metric: algorithmic TFLOP/s of GDPA forward + backward (their
flops over their time inside the timed steps, HIP events on the launch stream); `value_whole_step`
adds the sliding-window call (flops of all three over `ms_per_step`); `breakdown` gives each call
alone (TFLOP/s, % of the bf16 MFMA peak, achieved GB/s, % of the HBM roofline); `roofline`
describes the call that takes the longest; `cpu_baseline` is the CPU oracle timed on a bounded
sample of the same batch.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK = 2.5e15   # MI355X dense bf16, FLOP/s
HBM_PEAK = 8.0e12         # B/s
WORKLOAD = "cfg4"
WINDOW = (255, 0)
ORACLE_SAMPLE_EXAMPLES = 256

# HBM traffic per launch (bytes) from two rocprofv3 --pmc runs of this script (FETCH_SIZE, then
# WRITE_SIZE, KiB per dispatch), each scaled by what the same counter read for the 1 GiB
# device-to-device copy of --copy-calibration (FETCH_SIZE x2.000, WRITE_SIZE x1.000); see
# profiles/bench_cfg4_hbm_traffic.txt.  Valid for the default workload and seed only.  (The
# counters sit between L2 and the memory fabric: re-reads that the 256 MB Infinity Cache serves
# are included, which is what the sliding-window figure above its algorithmic 9.38 GB shows.)
MEASURED_TRAFFIC_BYTES = {"gdpa_fwd": 4958000000, "gdpa_bwd": 9782000000, "swa_fwd": 9377000000}


def device_normal(torch, shape, sigma, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    out = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    step = max(1, (1 << 27) // (shape[1] * shape[2]))
    for s in range(0, shape[0], step):
        e = min(shape[0], s + step)
        out[s:e] = (torch.randn((e - s,) + tuple(shape[1:]), generator=g, device="cuda", dtype=torch.float32)
                    * sigma).to(torch.bfloat16)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--skip-other-configs", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device-to-device copy (untimed) so that a rocprofv3 --pmc run has a "
                         "kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on ONE GPU (no collectives, no sharding); --gpus must be 1. "
              "The path would shard by example: every example is independent.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2602_10016_amd import binding as kb
    from paper_2602_10016_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    r = W.CONFIGS[WORKLOAD]
    B, H, d, Nq, tau = r["B"], r["H"], r["d"], r["Nq"], r["tau"]
    lengths = W.make_lengths(WORKLOAD, args.seed)
    off_np = W.offsets_from_lengths(lengths)
    T = int(off_np[-1])
    max_kv = int(r["lengths"][4])
    off = torch.from_numpy(off_np).cuda()
    q = device_normal(torch, (B * Nq, H, d), r["sigma"], 11 + args.seed)
    k = device_normal(torch, (T, H, d), r["sigma"], 12 + args.seed)
    v = device_normal(torch, (T, H, d), r["sigma"], 13 + args.seed)
    d_o = device_normal(torch, (B * Nq, H, d), 1.0, 14 + args.seed)
    qs = device_normal(torch, (T, H, d), r["sigma"], 15 + args.seed)   # self-attention queries
    scale_gdpa = 1.0 / tau
    scale_swa = 1.0 / math.sqrt(d)
    act = kb.ACT_GELU

    o = torch.empty_like(q)
    o_swa = torch.empty_like(qs)
    ws_f = torch.empty(kb.workspace_bytes(kb.OP_GDPA_FWD, B, H, d, Nq, max_kv, B * Nq, T), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(max(256, kb.workspace_bytes(kb.OP_GDPA_BWD, B, H, d, Nq, max_kv, B * Nq, T)), dtype=torch.uint8, device="cuda")
    ws_s = torch.empty(kb.workspace_bytes(kb.OP_SWA_FWD, B, H, d, max_kv, max_kv, T, T), dtype=torch.uint8, device="cuda")

    def call_fwd():
        kb.gdpa_fwd(q, k, v, off, scale_gdpa, act, max_q=Nq, max_kv=max_kv, out=o, want_lse=False, workspace=ws_f)

    grads = {}

    def call_bwd():
        grads["g"] = kb.gdpa_bwd(q, k, v, d_o, off, scale_gdpa, act, max_q=Nq, max_kv=max_kv, workspace=ws_b)

    def call_swa():
        kb.swa_fwd(qs, k, v, off, WINDOW[0], WINDOW[1], scale_swa, max_len=max_kv, out=o_swa, want_lse=False, workspace=ws_s)

    calls = [("gdpa_fwd", call_fwd), ("gdpa_bwd", call_bwd), ("swa_fwd", call_swa)]
    pairs = W.swa_pairs(lengths, *WINDOW)
    flops = {"gdpa_fwd": W.gdpa_flops(H, d, Nq, T), "gdpa_bwd": W.gdpa_flops(H, d, Nq, T, backward=True),
             "swa_fwd": W.swa_flops(H, d, pairs)}
    nbytes = {"gdpa_fwd": W.gdpa_bytes(H, d, B * Nq, T), "gdpa_bwd": W.gdpa_bytes(H, d, B * Nq, T, backward=True),
              "swa_fwd": W.swa_bytes(H, d, T)}

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        for _, fn in calls:
            fn()
    torch.cuda.synchronize()

    # events on the stream the kernels are launched on (torch's current stream, which the binding uses)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        ev[s][0].record()
        for i, (_, fn) in enumerate(calls):
            fn()
            ev[s][i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    call_ms = {name: sum(ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(args.steps)) / args.steps
               for i, (name, _) in enumerate(calls)}

    total_flops = sum(flops.values())
    value_step = total_flops / (ms_per_step * 1e-3) / 1e12
    ms_gdpa = call_ms["gdpa_fwd"] + call_ms["gdpa_bwd"]
    value = (flops["gdpa_fwd"] + flops["gdpa_bwd"]) / (ms_gdpa * 1e-3) / 1e12
    breakdown = {}
    for name, _ in calls:
        t = call_ms[name] * 1e-3
        breakdown[name] = {"ms": round(call_ms[name], 4), "tflops": round(flops[name] / t / 1e12, 2),
                           "pct_mfma_peak": round(100 * flops[name] / t / MFMA_BF16_PEAK, 2),
                           "gbps": round(nbytes[name] / t / 1e9, 1),
                           "pct_hbm_roofline": round(100 * nbytes[name] / t / HBM_PEAK, 2),
                           "gflop": round(flops[name] / 1e9, 2), "mbytes": round(nbytes[name] / 1e6, 1)}
    dom = max(call_ms, key=call_ms.get)
    achieved = nbytes[dom] / (call_ms[dom] * 1e-3) / 1e9
    roofline = {"kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                "frac": round(achieved / (HBM_PEAK / 1e9), 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get(dom) if args.seed == 0 else None,
                "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, taken offline "
                                  "(profiles/bench_cfg4_hbm_traffic.txt), not measured in this run",
                "algorithmic_bytes": int(nbytes[dom])}

    # What the memory system sustains for the ACCESS PATTERN of each call, measured now: the same tensors, offsets,
    # issue order and persistent launch, one walk per (example, head) that only moves the bytes
    # (kunlun_jagged_stream_probe; the Q / O / dQ rows, 3 % of the bytes, are left out).  Best of 1, 2 and 4
    # workgroups per compute unit.  A flat sweep over contiguous buffers (device_calibration below) runs faster
    # than any such walk: many independent walkers at unrelated places load the memory channels unevenly.
    def probe_ms(fn, n=5):
        fn()
        a_, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a_.record()
        for _ in range(n):
            fn()
        b_.record()
        torch.cuda.synchronize()
        return a_.elapsed_time(b_) / n

    _, dk_, dv_ = grads["g"]
    ws_p = torch.empty(256 + (4 * (B + 1) + 255) // 256 * 256, dtype=torch.uint8, device="cuda")
    pattern = {}
    for name, (pa, pb, pc, oa, ob, nr, nw) in {"gdpa_fwd": (k, v, None, None, None, 2, 0), "gdpa_bwd": (k, v, None, dk_, dv_, 2, 2),
                                               "swa_fwd": (qs, k, v, o_swa, None, 3, 1)}.items():
        best = min(probe_ms(lambda: kb.jagged_stream_probe(pa, pb, pc, oa, ob, off, max_kv, nr, nw, wg, workspace=ws_p))
                   for wg in (1, 2, 4))
        moved = (nr + nw) * T * H * d * 2
        pattern[name] = {"probe_gbps": round(moved / best / 1e6, 1), "probe_ms": round(best, 4),
                         "kernel_gbps": breakdown[name]["gbps"],
                         "kernel_vs_probe": round(breakdown[name]["gbps"] / (moved / best / 1e6), 3)}
    roofline["access_pattern_roof"] = {"unit": "GB/s", "achieved_by_byte_moving_probe": pattern[dom]["probe_gbps"],
                                       "frac_of_probe": pattern[dom]["kernel_vs_probe"]}
    del dk_, dv_

    # The other the benchmark spec workloads (parity-test cases, small): timed separately, no part of
    # `value`; reported for their achieved HBM GB/s.  Their inputs fit the 256 MB Infinity Cache, so
    # back-to-back launches are warm-cache figures: the primary numbers (us, gbps, tflops) are COLD
    # (before every launch 1 GiB of unrelated writes, then 1 GiB of reads streamed through: nothing of the
    # inputs is cached and no write-back of the flush is pending), the warm ones are given alongside, and so
    # is the figure after the writes alone (`us_after_write_only_flush`: 256 MB of dirty lines are then
    # written back during the timed launch, which is what earlier figures of these rows contained).
    other = {}
    if not args.skip_other_configs:
        flush = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")   # 4x the 256 MB Infinity Cache

        sink = torch.empty(4096, dtype=torch.uint8, device="cuda")

        def timed(fn, n=20):
            """(warm, cold, cold_dirty) microseconds per call.  warm = back-to-back launches (inputs that fit stay in the
            Infinity Cache).  cold = median of single launches, each after 1 GiB of unrelated writes AND then 1 GiB
            of reads streamed through (kunlun_stream_probe): nothing of the inputs is cached, and the cache holds clean
            lines.  cold_dirty = after the 1 GiB of writes only: the Infinity Cache is then full of dirty lines whose
            write-back (256 MB) lands in the timed region - a property of that flush, not of the kernel; kept because
            earlier figures were taken this way."""
            for _ in range(3):
                fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record()
            for _ in range(n):
                fn()
            b.record()
            torch.cuda.synchronize()
            warm = a.elapsed_time(b) / n
            cold, dirty = [], []
            for i in range(14):
                flush.fill_(i)
                if i % 2 == 0:
                    kb.stream_probe(flush, None, None, sink, 1, 0)
                a.record()
                fn()
                b.record()
                torch.cuda.synchronize()
                (cold if i % 2 == 0 else dirty).append(a.elapsed_time(b))
            return warm * 1e3, float(np.median(cold)) * 1e3, float(np.median(dirty)) * 1e3

        def entry(us_warm, us_cold, us_dirty, by, fl):
            return {"us": round(us_cold, 1), "gbps": round(by / us_cold / 1e3, 1), "tflops": round(fl / us_cold / 1e6, 1),
                    "us_warm": round(us_warm, 1), "gbps_warm": round(by / us_warm / 1e3, 1),
                    "us_after_write_only_flush": round(us_dirty, 1)}

        dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(torch.bfloat16).cuda()
        w2 = W.make("cfg2", args.seed)
        q2, k2, v2, do2 = dev(w2.q), dev(w2.k), dev(w2.v), dev(w2.d_o)
        off2 = torch.from_numpy(w2.kv_offsets).cuda()
        o2 = torch.empty_like(q2)
        need = max(kb.workspace_bytes(kb.OP_GDPA_BWD, w2.B, w2.H, w2.d, w2.Nq, 1024, w2.total_q, w2.total_kv),
                   kb.workspace_bytes(kb.OP_SWA_FWD, 128, 4, 128, 2048, 2048, 1 << 20, 1 << 20),
                   kb.workspace_bytes(kb.OP_GDPA_FWD, 32, 8, 128, 512, 2048, 32 * 512, 32 * 2048))
        wsx = torch.empty(need, dtype=torch.uint8, device="cuda")
        t = timed(lambda: kb.gdpa_fwd(q2, k2, v2, off2, w2.scale, act, max_q=w2.Nq, max_kv=1024, out=o2, want_lse=False, workspace=wsx))
        other["cfg2_gdpa_fwd"] = entry(*t, W.gdpa_bytes(w2.H, w2.d, w2.total_q, w2.total_kv),
                                       W.gdpa_flops(w2.H, w2.d, w2.Nq, w2.total_kv))
        t = timed(lambda: kb.gdpa_bwd(q2, k2, v2, do2, off2, w2.scale, act, max_q=w2.Nq, max_kv=1024, workspace=wsx))
        other["cfg5_gdpa_bwd"] = entry(*t, W.gdpa_bytes(w2.H, w2.d, w2.total_q, w2.total_kv, backward=True),
                                       W.gdpa_flops(w2.H, w2.d, w2.Nq, w2.total_kv, backward=True))
        # the same bytes moved without arithmetic: one walk per (example, head) over the cfg2 histories (best launch
        # width of 1, 2, 4 workgroups per compute unit), and a flat sweep over contiguous buffers of the same size
        dk2, dv2 = torch.empty_like(k2), torch.empty_like(v2)
        kv_bytes2 = 2 * k2.numel() * 2
        flat_a = torch.empty(kv_bytes2, dtype=torch.uint8, device="cuda")
        flat_b = torch.empty_like(flat_a)
        for key, nr, nw, oa, ob in (("cfg2_gdpa_fwd", 2, 0, None, None), ("cfg5_gdpa_bwd", 2, 2, dk2, dv2)):
            walk = min((timed(lambda: kb.jagged_stream_probe(k2, v2, None, oa, ob, off2, 1024, nr, nw, wg, workspace=wsx), n=10)
                        for wg in (1, 2, 4)), key=lambda t: t[1])
            flat = timed(lambda: kb.stream_probe(flat_a, None, None, flat_b, 1, 1 if nw else 0), n=10)
            other[key]["byte_moving_walk_us"] = round(walk[1], 1)
            other[key]["byte_moving_walk_us_warm"] = round(walk[0], 1)
            other[key]["flat_sweep_same_bytes_us"] = round(flat[1], 1)
            other[key]["kernel_vs_walk"] = round(walk[1] / other[key]["us"], 3)
        del dk2, dv2, flat_a, flat_b
        w3 = W.make("cfg3", args.seed)
        q3, k3, v3 = dev(w3.q), dev(w3.k), dev(w3.v)
        off3 = torch.from_numpy(w3.kv_offsets).cuda()
        o3 = torch.empty_like(q3)
        t = timed(lambda: kb.swa_fwd(q3, k3, v3, off3, w3.window[0], w3.window[1], w3.scale, max_len=2048, out=o3, want_lse=False, workspace=wsx))
        other["cfg3_swa_fwd"] = entry(*t, W.swa_bytes(w3.H, w3.d, w3.total_kv),
                                      W.swa_flops(w3.H, w3.d, W.swa_pairs(w3.lengths, *w3.window)))

        # The rows built beyond the three calls of the step: sliding-window backward on the cfg3 batch
        # and the PFFN direction of GDPA (the cfg3 sequences are the queries, 32 context tokens per
        # example are keys and values), forward and backward.
        do3 = dev(np.random.default_rng(args.seed + 5).standard_normal(w3.q.shape, dtype=np.float32))
        ws3 = torch.empty(kb.workspace_bytes(kb.OP_SWA_BWD, w3.B, w3.H, w3.d, 2048, 2048, w3.total_kv, w3.total_kv),
                          dtype=torch.uint8, device="cuda")
        o3f, lse3 = kb.swa_fwd(q3, k3, v3, off3, w3.window[0], w3.window[1], w3.scale, max_len=2048, workspace=ws3)
        t = timed(lambda: kb.swa_bwd(q3, k3, v3, o3f, lse3, do3, off3, w3.window[0], w3.window[1], w3.scale, max_len=2048, workspace=ws3), n=10)
        other["cfg3_swa_bwd"] = entry(*t, 2 * W.swa_bytes(w3.H, w3.d, w3.total_kv),
                                      2.5 * W.swa_flops(w3.H, w3.d, W.swa_pairs(w3.lengths, *w3.window)))
        n_ctx = 32
        kc3 = device_normal(torch, (w3.B * n_ctx, w3.H, w3.d), 0.5, 31)
        vc3 = device_normal(torch, (w3.B * n_ctx, w3.H, w3.d), 0.5, 32)
        offc = torch.arange(0, (w3.B + 1) * n_ctx, n_ctx, dtype=torch.int32, device="cuda")
        wsp = torch.empty(kb.workspace_bytes(kb.OP_GDPA_BWD, w3.B, w3.H, w3.d, 2048, n_ctx, w3.total_kv, w3.B * n_ctx),
                          dtype=torch.uint8, device="cuda")
        elt = w3.H * w3.d * 2
        t = timed(lambda: kb.gdpa_fwd(q3, kc3, vc3, offc, 1.0 / n_ctx, act, q_offsets=off3, max_q=2048, max_kv=n_ctx, out=o3, want_lse=False, workspace=wsp), n=10)
        other["pffn_direction_gdpa_fwd"] = entry(*t, 2 * w3.total_kv * elt + 2 * w3.B * n_ctx * elt,
                                                 4.0 * w3.d * w3.H * n_ctx * w3.total_kv)
        t = timed(lambda: kb.gdpa_bwd(q3, kc3, vc3, do3, offc, 1.0 / n_ctx, act, q_offsets=off3, max_q=2048, max_kv=n_ctx, workspace=wsp), n=10)
        other["pffn_direction_gdpa_bwd"] = entry(*t, 3 * w3.total_kv * elt + 4 * w3.B * n_ctx * elt,
                                                 10.0 * w3.d * w3.H * n_ctx * w3.total_kv)

        # The step's three calls on the same batch at head dimension 32 (a 256-wide layer with 8
        # heads, the paper's example of a click-sequence layer): a quarter of the bytes.
        d32 = 32
        q32 = device_normal(torch, (B * Nq, H, d32), r["sigma"], 51)
        k32 = device_normal(torch, (T, H, d32), r["sigma"], 52)
        v32 = device_normal(torch, (T, H, d32), r["sigma"], 53)
        do32 = device_normal(torch, (B * Nq, H, d32), 1.0, 54)
        qs32 = device_normal(torch, (T, H, d32), r["sigma"], 55)
        o32, os32 = torch.empty_like(q32), torch.empty_like(qs32)
        t = timed(lambda: kb.gdpa_fwd(q32, k32, v32, off, scale_gdpa, act, max_q=Nq, max_kv=max_kv, out=o32, want_lse=False, workspace=ws_f), n=10)
        h32 = {"gdpa_fwd": entry(*t, W.gdpa_bytes(H, d32, B * Nq, T), W.gdpa_flops(H, d32, Nq, T))}
        t = timed(lambda: kb.gdpa_bwd(q32, k32, v32, do32, off, scale_gdpa, act, max_q=Nq, max_kv=max_kv, workspace=ws_b), n=10)
        h32["gdpa_bwd"] = entry(*t, W.gdpa_bytes(H, d32, B * Nq, T, backward=True), W.gdpa_flops(H, d32, Nq, T, backward=True))
        t = timed(lambda: kb.swa_fwd(qs32, k32, v32, off, WINDOW[0], WINDOW[1], 1.0 / math.sqrt(d32), max_len=max_kv, out=os32, want_lse=False, workspace=ws_s), n=10)
        h32["swa_fwd"] = entry(*t, W.swa_bytes(H, d32, T), W.swa_flops(H, d32, pairs))
        other["cfg4_batch_at_head_dim_32"] = h32
        del q32, k32, v32, do32, qs32, o32, os32

        # SumKronLinear (stage 3 of hierarchical seed pooling) at the paper's typical configuration:
        # matrix-core-bound (about 570 flop per byte of X).
        Bk, Sk, Tk, Dk, kk = 1024, 256, 32, 384, 8
        xk = device_normal(torch, (Bk, Sk, Dk), 1.0, 41)
        zk = device_normal(torch, (kk, Sk, Tk), 1.0 / math.sqrt(Sk), 42)
        wk = device_normal(torch, (kk, Dk, Dk), 1.0 / math.sqrt(Dk), 43)
        yk = torch.empty((Bk, Tk, Dk), dtype=torch.bfloat16, device="cuda")
        wsk = torch.empty(kb.sumkron_workspace_bytes(Bk, Sk, Tk, Dk, kk), dtype=torch.uint8, device="cuda")
        tw, tc, *_ = timed(lambda: kb.sumkron_fwd(xk, zk, wk, out=yk, workspace=wsk), n=10)
        fl = 2.0 * Bk * kk * Tk * Dk * (Sk + Dk)
        other["sumkron_fwd_S256_T32_D384_k8_B1024"] = {"us": round(tc, 1), "us_warm": round(tw, 1), "tflops": round(fl / tc / 1e6, 1),
                                                       "pct_mfma_peak": round(100 * fl / (tc * 1e-6) / MFMA_BF16_PEAK, 2),
                                                       "tflops_warm": round(fl / tw / 1e6, 1),
                                                       "pct_mfma_peak_warm": round(100 * fl / (tw * 1e-6) / MFMA_BF16_PEAK, 2),
                                                       "note": "cold: X (201 MB) comes from HBM; warm: back-to-back calls, X "
                                                               "largely out of the 256 MB Infinity Cache"}
        dyk = device_normal(torch, (Bk, Tk, Dk), 1.0, 44)
        wsb = torch.empty(kb.sumkron_bwd_workspace_bytes(Bk, Sk, Tk, Dk, kk), dtype=torch.uint8, device="cuda")
        tw, tc, *_ = timed(lambda: kb.sumkron_bwd(xk, zk, wk, dyk, workspace=wsb), n=10)
        fl = 2.0 * Bk * kk * Tk * Dk * (3 * Sk + 2 * Dk)   # U, G, dX, dW, dZ: each intermediate computed once
        other["sumkron_bwd_S256_T32_D384_k8_B1024"] = {"us": round(tc, 1), "us_warm": round(tw, 1), "tflops": round(fl / tc / 1e6, 1),
                                                       "pct_mfma_peak": round(100 * fl / (tc * 1e-6) / MFMA_BF16_PEAK, 2)}
        del xk, yk, wsk, dyk, wsb

        # Diagnostic, not a workload of the paper: the same forward entry point on a shape that IS
        # matrix-core-bound (512 queries per example: 512 flop per K/V byte, above the ridge), to show
        # what the MFMA pipeline of these kernels sustains when HBM is out of the way.
        Bd, Nd, Ld = 32, 512, 2048
        qd = device_normal(torch, (Bd * Nd, H, d), 0.5, 21)
        kd = device_normal(torch, (Bd * Ld, H, d), 0.5, 22)
        vd = device_normal(torch, (Bd * Ld, H, d), 0.5, 23)
        offd = torch.arange(0, (Bd + 1) * Ld, Ld, dtype=torch.int32, device="cuda")
        od = torch.empty_like(qd)
        fl = W.gdpa_flops(H, d, Nd, Bd * Ld)
        diag = {}
        for name, a, sc_ in (("gelu", act, 1.0 / Ld), ("gelu_poly", kb.ACT_GELU_POLY, 1.0 / Ld),
                             ("softmax", kb.ACT_SOFTMAX, 1.0 / math.sqrt(d))):
            tw, *_ = timed(lambda: kb.gdpa_fwd(qd, kd, vd, offd, sc_, a, max_q=Nd, max_kv=Ld, out=od, want_lse=False, workspace=wsx), n=10)
            diag[name] = {"us": round(tw, 1), "tflops": round(fl / tw / 1e6, 1),
                          "pct_mfma_peak": round(100 * fl / (tw * 1e-6) / MFMA_BF16_PEAK, 2)}
        other["diagnostic_mfma_bound_gdpa_fwd_Nq512"] = diag

        # Seed-level attention with batch-shared seeds (Sec. "Hierarchical Seed Pooling", stage 1: S = 256 learnable
        # seeds attend to every history under softmax) on the bench batch: forward, and backward with the seed
        # gradient summed over the batch in fixed order.
        n_seeds = 256
        e_seed = device_normal(torch, (n_seeds, H, d), r["sigma"], 31 + args.seed)
        do_s = device_normal(torch, (B * n_seeds, H, d), 1.0, 32 + args.seed)
        o_se = torch.empty((B * n_seeds, H, d), dtype=torch.bfloat16, device="cuda")
        lse_se = torch.empty((H, B * n_seeds), dtype=torch.float32, device="cuda")
        ws_sf = torch.empty(kb.workspace_bytes(kb.OP_SEED_FWD, B, H, d, n_seeds, max_kv, B * n_seeds, T), dtype=torch.uint8, device="cuda")
        ws_sb = torch.empty(kb.workspace_bytes(kb.OP_SEED_BWD, B, H, d, n_seeds, max_kv, B * n_seeds, T), dtype=torch.uint8, device="cuda")
        tf_, *_ = timed(lambda: kb.seed_attn_fwd(e_seed, k, v, off, scale_swa, max_kv=max_kv, out=o_se, lse=lse_se, workspace=ws_sf), n=5)
        tb_, *_ = timed(lambda: kb.seed_attn_bwd(e_seed, k, v, do_s, off, scale_swa, o=o_se, lse=lse_se, max_kv=max_kv, workspace=ws_sb), n=3)
        fl_f, fl_b = W.gdpa_flops(H, d, n_seeds, T), W.gdpa_flops(H, d, n_seeds, T, backward=True)
        # (the same 256 shared seeds under the activation score functions of Eq. (GDPA): GELU by erf, and the
        # polynomial GELU that needs no transcendental)
        by_act = {}
        for name, a in (("gelu", kb.ACT_GELU), ("gelu_poly", kb.ACT_GELU_POLY)):
            ta_, *_ = timed(lambda: kb.seed_attn_fwd(e_seed, k, v, off, scale_gdpa, a, max_kv=max_kv, out=o_se, want_lse=False, workspace=ws_sf), n=5)
            by_act[name] = round(ta_ / 1e3, 3)
        other["seed_attention_256_shared_seeds_bench_batch"] = {
            "fwd_ms_gelu": by_act["gelu"], "fwd_ms_gelu_poly": by_act["gelu_poly"],
            "fwd_ms": round(tf_ / 1e3, 3), "fwd_tflops": round(fl_f / tf_ / 1e6, 1), "fwd_pct_mfma_peak": round(100 * fl_f / (tf_ * 1e-6) / MFMA_BF16_PEAK, 2),
            "bwd_ms": round(tb_ / 1e3, 3), "bwd_tflops": round(fl_b / tb_ / 1e6, 1), "bwd_pct_mfma_peak": round(100 * fl_b / (tb_ * 1e-6) / MFMA_BF16_PEAK, 2)}
        del e_seed, do_s, o_se, lse_se, ws_sf, ws_sb

        # Measured speed of light of this device, by library routines of the harness (torch): a 1 GiB
        # device-to-device copy (read + write) and a large bf16 GEMM.
        # What this memory system sustains depends on the read : write mix of a stream, so the calls
        # are put next to plain streaming kernels of their own mix (1 GiB fp32 operands): a sum (reads
        # only, like gdpa_fwd), a copy (1 : 1, like gdpa_bwd), a + b * c (3 reads : 1 write, like swa_fwd).
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        tw, *_ = timed(lambda: flush.copy_(src), n=10)
        fa, fb = src.view(torch.float32), flush.view(torch.float32)
        fc, fd = torch.ones_like(fa), torch.empty_like(fa)
        t31, *_ = timed(lambda: torch.addcmul(fa, fb, fc, out=fd), n=10)
        tr, *_ = timed(lambda: torch.sum(fa), n=10)
        ga = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
        gb = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
        tg, *_ = timed(lambda: torch.matmul(ga, gb), n=10)
        # the same three mixes by the library's own plain streaming kernel (kunlun_stream_probe: 16 KB per
        # workgroup and stream, non-temporal), the best of the access patterns tried on this device
        probe = {}
        for name, reads, write in (("read_only", 3, 0), ("one_read_one_write", 1, 1), ("three_reads_one_write", 3, 1)):
            tp, *_ = timed(lambda: kb.stream_probe(src, flush, fc.view(torch.uint8), fd.view(torch.uint8), reads, write), n=10)
            probe[name + "_gbps"] = round((reads + write) * (1 << 30) / tp / 1e3, 1)
        other["device_calibration"] = {"stream_probe_1GiB_operands": probe,
                                       "torch_sum_1GiB_gbps": round((1 << 30) / tr / 1e3, 1),
                                       "torch_copy_1GiB_gbps_read_plus_write": round(2 * (1 << 30) / tw / 1e3, 1),
                                       "torch_addcmul_three_reads_one_write_gbps": round(4 * (1 << 30) / t31 / 1e3, 1),
                                       "bf16_gemm_8192_tflops": round(2 * 8192 ** 3 / tg / 1e6, 1)}
        del src, ga, gb, flush, fa, fb, fc, fd

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        n = min(ORACLE_SAMPLE_EXAMPLES, B)
        kv_n = int(off_np[n])
        host = lambda t: t.float().cpu().numpy().astype(np.float64)
        hq, hk, hv, hdo, hqs = host(q[:n * Nq]), host(k[:kv_n]), host(v[:kv_n]), host(d_o[:n * Nq]), host(qs[:kv_n])
        sub_off = off_np[:n + 1]
        t1 = time.perf_counter()
        oracle.gdpa_fwd(hq, hk, hv, sub_off, scale_gdpa, act, max_q=Nq)
        oracle.gdpa_bwd(hq, hk, hv, hdo, sub_off, scale_gdpa, act, max_q=Nq)
        oracle.swa_fwd(hqs, hk, hv, sub_off, WINDOW[0], WINDOW[1], scale_swa)
        cpu_s = time.perf_counter() - t1
        sub_flops = (W.gdpa_flops(H, d, Nq, kv_n) + W.gdpa_flops(H, d, Nq, kv_n, backward=True)
                     + W.swa_flops(H, d, W.swa_pairs(lengths[:n], *WINDOW)))
        cpu_baseline = {"value": round(sub_flops / cpu_s / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.num_threads(),
                        "kind": "oracle", "seconds": round(cpu_s, 2),
                        "sample": f"first {n} of {B} examples of the same batch ({kv_n} history tokens), same three "
                                  f"calls, fp64"}

    out = {
        "metric": "GDPA fwd/bwd TFLOP/s + % of MI355X bf16 MFMA peak, jagged B=1024",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "pct_mfma_peak": round(100 * value * 1e12 / MFMA_BF16_PEAK, 2),
        "value_covers": "gdpa_fwd + gdpa_bwd (the metric); their flops over their share of the timed steps",
        "ms_gdpa_fwd_bwd": round(ms_gdpa, 4),
        "value_whole_step": round(value_step, 2),
        # this operator does about Nq = 64 flops per K/V byte: at 8 TB/s that caps it near 20 % of the MFMA peak
        "hbm_bound_cap_pct_mfma_peak": round(100 * (flops["gdpa_fwd"] + flops["gdpa_bwd"]) /
                                             ((nbytes["gdpa_fwd"] + nbytes["gdpa_bwd"]) / HBM_PEAK) / MFMA_BF16_PEAK, 2),
        "config": {"workload": f"{WORKLOAD}: B={B} H={H} d={d} Nq={Nq}, history lengths lognormal(median 800, "
                               f"sigma 1) clipped [32,4096], T={T} tokens; step = gdpa_fwd(gelu, 1/tau) + gdpa_bwd + "
                               f"swa_fwd(window 256 causal) on the same batch; value = the two GDPA calls", "seed": args.seed,
                   "step_gflop": round(total_flops / 1e9, 1)},
        "breakdown": breakdown, "roofline": roofline, "access_pattern_probe": pattern, "cpu_baseline": cpu_baseline,
        "other_configs": other,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
