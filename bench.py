#!/usr/bin/env python3
"""Benchmark of the USP hot path on one MI355X.

One "step" = one pass of the hot path on the FLUX-1024 Ulysses shard (workload
`flux1024_u`): FP8 pack of the [4608, 3072] bf16 All-to-All payload (usp_fp8_quant),
its unpack (usp_fp8_dequant), and attention of the [1, 24, 4608, 128] bf16 shard
(usp_ring_attn_fwd, one KV chunk).  All inputs are seeded synthetic data already
resident in HBM.  `value` is attention TFLOP/s over the whole step time (the FP8
pack/unpack time is inside the step); per-kernel figures follow in the same JSON line.

Prints ONE JSON line.  Extra legs outside the timed region: the ring shards
(`flux1024_r4`, `flux2048_u2r8`: merge + double buffering over a side stream and with the
transfers inside the attention launches, hidden fraction), and the fp64 oracle timed on
the host cores as `cpu_baseline`.
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

PEAK_BF16_TFLOPS = 2516.6   # 256 CU x 4096 flop/clk x 2.4 GHz (dense, no sparsity)
PEAK_HBM_GBS = 8000.0
PREHEAT_S = 1.5             # untimed run of the same step before the warm-up and the timed region


def measured_traffic(workload, kernel):
    """HBM bytes per launch (fetch + write) from the rocprofv3 --pmc summary kept under profiles/,
    or None if there is no entry for this workload and kernel."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 4 and not line.startswith("#") and parts[0] == workload and parts[1] == kernel:
                    return {"bytes": float(parts[2]) + float(parts[3]), "fetch_bytes": float(parts[2]),
                            "write_bytes": float(parts[3]), "source": "profiles/hbm_traffic_per_launch.txt"}
    except OSError:
        pass
    return None


def _events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the GPU needs a few hundred ms of sustained load before its clocks settle: a fixed pre-heat
    # (PREHEAT_S of the same step, untimed, whatever --warmup says) precedes the W warm-up steps
    ap.add_argument("--steps", type=int, default=2500)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ring", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain elementwise kernel that reads 256 MiB and writes 256 MiB "
                         "(torch.add on int32), as the known-traffic reference for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE runs")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a one-GPU hot path (one rank's share of USP attention); "
              "--gpus %d is not supported, run with --gpus 1" % args.gpus, file=sys.stderr)
        return 2

    import torch
    import paper_2602_10940_amd as P
    from paper_2602_10940_amd import diag as D
    from paper_2602_10940_amd import workloads as W

    P.load_library()                      # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    def up_bf16(x32):
        bits = W.f32_to_bf16_bits(x32)
        return torch.from_numpy(bits.view(np.int16).copy()).to(dev).view(torch.bfloat16).reshape(x32.shape)

    # ---------------- workload: FLUX-1024 shard, Ulysses only --------------------------------
    wl = W.WORKLOADS["flux1024_u"]
    inp = W.make_attention_inputs(wl)
    q, k, v = up_bf16(inp.q), up_bf16(inp.k[0]), up_bf16(inp.v[0])
    out = torch.empty_like(q)
    lse = torch.empty((wl.B, wl.H, wl.Sq), dtype=torch.float32, device=dev)
    scale = float(inp.softmax_scale)
    x0 = up_bf16(W.make_payload(wl))
    R, C = x0.shape
    NBUF = 24                              # 24 x (28.3 + 14.2 + 28.3) MB > 512 MB: FP8 kernels cannot live in cache
    xs = [x0] + [torch.roll(x0, i, 0).contiguous() for i in range(1, NBUF)]
    qs = [torch.empty((R, C), dtype=torch.uint8, device=dev) for _ in range(NBUF)]
    ss = [torch.empty((R,), dtype=torch.float32, device=dev) for _ in range(NBUF)]
    ys = [torch.empty((R, C), dtype=torch.bfloat16, device=dev) for _ in range(NBUF)]

    desc = P.make_attn_desc(q, [k], out, scale, 0)
    ws = torch.empty((max(P.usp_ring_attn_workspace_bytes(desc), 256),), dtype=torch.uint8, device=dev)

    def step(i, ev=None):
        j = i % NBUF
        P.usp_fp8_quant(xs[j], qs[j], ss[j])
        P.usp_fp8_dequant(qs[j], ss[j], y=ys[j])
        if ev: ev[0].record()
        P.usp_ring_attn_fwd(q, [k], [v], softmax_scale=scale, out=out, lse=lse, workspace=ws)
        if ev: ev[1].record()

    # pre-heat: the same step, untimed, until PREHEAT_S of wall time have passed (clocks settled)
    t_pre = time.perf_counter()
    n_pre = 0
    while time.perf_counter() - t_pre < PREHEAT_S:
        for i in range(50):
            step(n_pre + i)
        n_pre += 50
        torch.cuda.synchronize()
    preheat_s = time.perf_counter() - t_pre
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    evs = [_events(2) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    t_attn = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))   # per launch, on the launch stream

    # FP8 kernels: back-to-back launches over the rotating buffers between two events
    def per_launch(fn, reps=480, rounds=5, stats=None):
        """Median over `rounds` of (time of `reps` back-to-back launches between two events) / reps;
        `stats`, a dict, also receives the minimum."""
        for i in range(48):
            fn(i)
        ts = []
        for _ in range(rounds):
            a, b = _events(2)
            a.record()
            for i in range(reps):
                fn(i)
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) / reps)
        if stats is not None:
            stats["min_us"] = round(min(ts) * 1e3, 2)
        return float(np.median(ts))
    # The single-payload figures are taken with the calls issued from C (libusp_diag.so loops over the
    # same usp_fp8_quant / usp_fp8_dequant entry points): through the interpreter a call costs the host
    # 7-8 us, which is what such a loop would then measure.
    def per_launch_c(kind, sets=slice(0, NBUF), reps=480, rounds=5, stats=None):
        bufs = (xs[sets], qs[sets], ss[sets], ys[sets])
        D.usp_diag_repeat_payload_calls(kind, 48, *bufs)
        ts = []
        for _ in range(rounds):
            a, b = _events(2)
            a.record()
            D.usp_diag_repeat_payload_calls(kind, reps, *bufs)
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) / reps)
        if stats is not None:
            stats["min_us"] = round(min(ts) * 1e3, 2)
        return float(np.median(ts))
    st_q, st_d = {}, {}
    t_quant = per_launch_c(0, stats=st_q)
    t_deq = per_launch_c(1, stats=st_d)
    t_quant_py = per_launch(lambda i: P.usp_fp8_quant(xs[i % NBUF], qs[i % NBUF], ss[i % NBUF]), rounds=3)
    # what bounds a single payload launch: the pack's grid doing nothing, only reading, only writing
    t_floor = [per_launch_c(k, rounds=3) for k in (2, 3, 4)]
    # the same launches on one buffer set (71 MB: served by the 256 MB Infinity Cache)
    t_quant_warm = per_launch_c(0, sets=slice(0, 1), rounds=3)
    t_deq_warm = per_launch_c(1, sets=slice(0, 1), rounds=3)
    # the same kernels on 8 payloads stacked into one [36864, 3072] call: launch overhead amortised
    xb = torch.cat(xs[:8], 0)
    qb = torch.empty((8 * R, C), dtype=torch.uint8, device=dev)
    sb = torch.empty((8 * R,), dtype=torch.float32, device=dev)
    yb = torch.empty((8 * R, C), dtype=torch.bfloat16, device=dev)
    t_quant8 = per_launch(lambda i: P.usp_fp8_quant(xb, qb, sb), reps=100, rounds=3)
    t_deq8 = per_launch(lambda i: P.usp_fp8_dequant(qb, sb, y=yb), reps=100, rounds=3)
    # ... and on 3 payloads (the Q, K and V of one attention layer entering the All-to-All) in one call
    R3 = 3 * R
    x3 = torch.cat(xs[:24], 0)                      # 8 disjoint sets of three payloads: 1.7 GB with codes and outputs
    q3 = torch.empty((24 * R, C), dtype=torch.uint8, device=dev)
    s3 = torch.empty((24 * R,), dtype=torch.float32, device=dev)
    y3 = torch.empty((24 * R, C), dtype=torch.bfloat16, device=dev)
    sl = lambda t, i: t[(i % 8) * R3:(i % 8) * R3 + R3]
    t_quant3 = per_launch(lambda i: P.usp_fp8_quant(sl(x3, i), sl(q3, i), sl(s3, i)), reps=200, rounds=3)
    t_deq3 = per_launch(lambda i: P.usp_fp8_dequant(sl(q3, i), sl(s3, i), y=sl(y3, i)), reps=200, rounds=3)
    del x3, q3, s3, y3
    # pack / unpack in the layouts around the All-to-All (section 2.2.1), 8 peers: the same 28.3 MB as
    # [1, 24, 4608, 128] on the sequence-sharded side -> send blocks [8][1][3][4608] rows of 128 ->
    # (exchange) -> [1, 3, 36864, 128] on the head-sharded side
    Nr, Hh, Sl, Dd = 8, 24, R, 128
    Hn = Hh // Nr
    n4 = (Nr, 1, Hn, Sl)
    dense = (Hn * Sl, Hn * Sl, Sl, 1)
    seq_sh = (Hn * Sl * Dd, Hh * Sl * Dd, Sl * Dd, Dd)
    head_sh = (Sl * Dd, Hn * Nr * Sl * Dd, Nr * Sl * Dd, Dd)
    qm = [torch.empty((Hh * Sl, Dd), dtype=torch.uint8, device=dev) for _ in range(NBUF)]
    sm = [torch.empty((Hh * Sl,), dtype=torch.float32, device=dev) for _ in range(NBUF)]
    t_quant_map = per_launch(lambda i: P.usp_fp8_quant_mapped(xs[i % NBUF], n4, seq_sh, dense, Dd, qm[i % NBUF], sm[i % NBUF]), rounds=3)
    t_deq_map = per_launch(lambda i: P.usp_fp8_dequant_mapped(qm[i % NBUF], sm[i % NBUF], n4, dense, head_sh, ys[i % NBUF]), rounds=3)
    map_bytes = R * C * 3 + Hh * Sl * 4
    del qm, sm
    # Algorithm 1 as printed: one scale for the whole tensor = the payload viewed as a single row
    x1 = xs[0].reshape(1, R * C)
    q1 = torch.empty((1, R * C), dtype=torch.uint8, device=dev)
    s1 = torch.empty((1,), dtype=torch.float32, device=dev)
    t_quant_pt = per_launch(lambda i: P.usp_fp8_quant(x1, q1, s1), reps=100, rounds=3)
    del xb, qb, sb, yb, q1, s1

    # standalone merge (the second line under Algorithm 2) on the flux1024_r4 state: 27648 rows x 128,
    # rotating over 8 buffer sets (8 x 21.5 MB x ... beyond what one launch touches, inside the cache)
    mrows = 24 * 1152
    mo1 = [torch.randn((mrows, 128), device=dev).to(torch.bfloat16) for _ in range(24)]
    mo2 = [torch.randn((mrows, 128), device=dev).to(torch.bfloat16) for _ in range(24)]
    ml1 = [torch.randn((mrows,), device=dev) for _ in range(24)]
    ml2 = [torch.randn((mrows,), device=dev) for _ in range(24)]
    mo = [torch.empty_like(x) for x in mo1]
    ml = [torch.empty_like(x) for x in ml1]
    def merge_c(reps=480, rounds=3):
        D.usp_diag_repeat_merge_calls(48, mo1, ml1, mo2, ml2, mo, ml)
        ts = []
        for _ in range(rounds):
            a, b = _events(2)
            a.record()
            D.usp_diag_repeat_merge_calls(reps, mo1, ml1, mo2, ml2, mo, ml)
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) / reps)
        return float(np.median(ts))
    t_merge = merge_c()
    merge_bytes = mrows * 128 * 3 * 2 + mrows * 12
    del mo1, mo2, ml1, ml2, mo, ml

    # what the matrix cores sustain with nothing else issued: one work-group of 8 waves per CU doing
    # back-to-back 32x32x16 bf16 MFMAs on register operands, ~1 ms per launch (the chip lowers its
    # clock under a full matrix-core load, and by how much depends on the operand data)
    def mfma_probe(random_data, shape=0):
        n_cu = torch.cuda.get_device_properties(dev).multi_processor_count
        iters = 1000
        pout = torch.empty((n_cu * 512,), dtype=torch.float32, device=dev)
        pclk = torch.zeros((2,), dtype=torch.int64, device=dev)
        t = per_launch(lambda i: D.usp_diag_mfma_rate(n_cu, iters, random_data, pout, pclk, shape=shape), reps=20, rounds=3)
        cyc, ticks = [int(v) for v in pclk.cpu()]
        fl = n_cu * 8 * iters * 32 * 32768.0
        return {"tflops": round(fl / (t * 1e-3) * 1e-12, 1), "shader_mhz": round(cyc / max(ticks, 1) * 100.0),
                "frac_of_bf16_peak": round(fl / (t * 1e-3) * 1e-12 / PEAK_BF16_TFLOPS, 4)}
    probe_rand, probe_const = mfma_probe(True), mfma_probe(False)
    probe_rand16 = mfma_probe(True, shape=1)

    traffic = measured_traffic("flux1024_u", "attn_pp_kernel<wide,plain>")
    flops = wl.attn_flops()
    value = flops / (ms_per_step * 1e-3) * 1e-12
    attn_tflops = flops / (t_attn * 1e-3) * 1e-12
    fp8_bytes = R * C * 3 + R * 4          # quant: 2 B in + 1 B out per element + scales; dequant mirrored
    quant_gbs = fp8_bytes / (t_quant * 1e-3) * 1e-9
    deq_gbs = fp8_bytes / (t_deq * 1e-3) * 1e-9

    result = {
        "metric": "ring-attn TFLOP/s + FP8 quant GB/s, % of MI355X peak, FLUX-1024 shard",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "preheat_s": round(preheat_s, 2), "preheat_steps": n_pre,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "flux1024_u: B=1 H=24 d=128 S=4608 bf16, one KV chunk; FP8 payload [4608,3072] bf16",
                   "step": "fp8_quant + fp8_dequant + ring_attn_fwd"},
        "attn": {"ms": round(t_attn, 4), "tflops": round(attn_tflops, 1),
                 "frac_of_bf16_peak": round(attn_tflops / PEAK_BF16_TFLOPS, 4)},
        "fp8_quant": {"us": round(t_quant * 1e3, 2), "gbs": round(quant_gbs, 1),
                      "frac_of_hbm_peak": round(quant_gbs / PEAK_HBM_GBS, 4), "bytes": fp8_bytes,
                      "min_us": st_q["min_us"], "cache_warm_us": round(t_quant_warm * 1e3, 2),
                      "via_python_binding_us": round(t_quant_py * 1e3, 2),
                      "protocol": "median of 5 x 480 back-to-back calls of the C entry point, issued from C, over 24 rotating "
                                  "buffer sets (1.7 GB)"},
        "fp8_dequant": {"us": round(t_deq * 1e3, 2), "gbs": round(deq_gbs, 1),
                        "frac_of_hbm_peak": round(deq_gbs / PEAK_HBM_GBS, 4), "bytes": fp8_bytes,
                        "min_us": st_d["min_us"], "cache_warm_us": round(t_deq_warm * 1e3, 2)},
        "fp8_launch_floor": {"empty_launch_us": round(t_floor[0] * 1e3, 2), "read_only_us": round(t_floor[1] * 1e3, 2),
                             "write_only_us": round(t_floor[2] * 1e3, 2),
                             "floor_us": round((t_floor[0] + fp8_bytes / (7.45e12) * 1e3) * 1e3, 2),
                             "note": "back-to-back launches of the pack's grid (1152 x 256 threads) that do nothing / read the "
                                     "28.3 MB payload / write 14.2 MB; floor = empty launch + 42.49 MB at 7.45 TB/s, the rate "
                                     "the unpack's body reaches"},
        "fp8_x8_payload": {"quant_us": round(t_quant8 * 1e3, 2), "dequant_us": round(t_deq8 * 1e3, 2),
                           "quant_gbs": round(8 * fp8_bytes / (t_quant8 * 1e-3) * 1e-9, 1),
                           "dequant_gbs": round(8 * fp8_bytes / (t_deq8 * 1e-3) * 1e-9, 1),
                           "note": "[36864,3072] in one call: the dispatch gap that bounds a single 28 MB launch is amortised"},
        "fp8_x3_payload": {"quant_us": round(t_quant3 * 1e3, 2), "dequant_us": round(t_deq3 * 1e3, 2),
                           "quant_gbs": round(3 * fp8_bytes / (t_quant3 * 1e-3) * 1e-9, 1),
                           "dequant_gbs": round(3 * fp8_bytes / (t_deq3 * 1e-3) * 1e-9, 1),
                           "quant_frac_of_hbm_peak": round(3 * fp8_bytes / (t_quant3 * 1e-3) * 1e-9 / PEAK_HBM_GBS, 4),
                           "dequant_frac_of_hbm_peak": round(3 * fp8_bytes / (t_deq3 * 1e-3) * 1e-9 / PEAK_HBM_GBS, 4),
                           "note": "[13824,3072] in one call: the Q, K and V payloads of one attention layer"},
        "fp8_a2a_layouts": {"pack_us": round(t_quant_map * 1e3, 2), "unpack_us": round(t_deq_map * 1e3, 2),
                            "pack_gbs": round(map_bytes / (t_quant_map * 1e-3) * 1e-9, 1),
                            "unpack_gbs": round(map_bytes / (t_deq_map * 1e-3) * 1e-9, 1),
                            "note": "rows of 128 (one scale per head and token), written / read one block per peer, 8 peers"},
        "fp8_quant_per_tensor": {"us": round(t_quant_pt * 1e3, 2),
                                 "gbs": round((R * C * 3 + 4) / (t_quant_pt * 1e-3) * 1e-9, 1),
                                 "note": "the payload as one row (one scale): absmax pass + cast pass, input read twice, cache-warm"},
        "lse_merge": {"us": round(t_merge * 1e3, 2), "gbs": round(merge_bytes / (t_merge * 1e-3) * 1e-9, 1),
                      "bytes": merge_bytes, "frac_of_hbm_peak": round(merge_bytes / (t_merge * 1e-3) * 1e-9 / PEAK_HBM_GBS, 4),
                      "note": "flux1024_r4 state [27648,128] bf16, 24 buffer sets (0.5 GB), calls issued from C"},
        "roofline": {"bound": "mfma", "achieved": round(attn_tflops, 1), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic["bytes"] if traffic else None, "traffic_detail": traffic,
                     "kernel": "attn_pp_kernel<wide, plain>", "flops_per_launch": flops},
        "mfma_sustained": {"random_operands": probe_rand, "constant_operands": probe_const,
                           "random_operands_16x16x32": probe_rand16,
                           "note": "MFMA-only probe on every CU (libusp_diag.so, usp_diag_mfma_rate; 32x32x16 unless named "
                                   "otherwise): the rate and clock the chip holds under a full matrix-core load; the "
                                   "published peak assumes 2400 MHz"},
    }
    result["roofline"]["frac_of_sustained_mfma"] = round(attn_tflops / probe_rand["tflops"], 4)
    result["roofline"]["frac_of_sustained_mfma_16x16x32"] = round(attn_tflops / probe_rand16["tflops"], 4)
    # the same launch on all-zero Q, K, V: the work and its schedule are unchanged, the matrix cores'
    # datapaths do not toggle, and the chip holds a higher clock: what the kernel's schedule is worth
    # when power does not bound it
    zq = torch.zeros_like(q)
    for _ in range(400):
        P.usp_ring_attn_fwd(zq, [zq], [zq], softmax_scale=scale, out=out, lse=lse, workspace=ws)
    torch.cuda.synchronize()
    za, zb = _events(2)
    za.record()
    for _ in range(1000):
        P.usp_ring_attn_fwd(zq, [zq], [zq], softmax_scale=scale, out=out, lse=lse, workspace=ws)
    zb.record()
    torch.cuda.synchronize()
    t_zero = za.elapsed_time(zb) / 1000
    result["attn_zero_operands"] = {"ms": round(t_zero, 4), "tflops": round(flops / (t_zero * 1e-3) * 1e-12, 1),
                                    "frac_of_bf16_peak": round(flops / (t_zero * 1e-3) * 1e-12 / PEAK_BF16_TFLOPS, 4),
                                    "note": "same launch, all-zero operands (no toggling in the matrix datapaths): the "
                                            "difference to attn.ms is the clock the chip gives up under the load"}
    del zq

    if args.calibrate_copy:
        ca = torch.ones((64 << 20,), dtype=torch.int32, device=dev)
        cb = torch.empty_like(ca)
        for _ in range(5):
            torch.add(ca, 1, out=cb)
        torch.cuda.synchronize()
        result["calibrate_copy"] = {"kernel": "torch.add int32", "read_bytes": ca.numel() * 4,
                                    "write_bytes": cb.numel() * 4, "launches": 5}
        del ca, cb

    # ---------------- ring degree 4: merge + double buffering (not part of `value`) -----------
    if not args.no_ring:
        result["ring"] = ring_leg(P, W, torch, dev, up_bf16, "flux1024_r4")
        result["ring_flux2048_u2r8"] = ring_leg(P, W, torch, dev, up_bf16, "flux2048_u2r8", reps=300)

        result["qwen_r2"] = qwen_leg(P, W, torch, dev, up_bf16)
        result["d64"] = d64_leg(P, torch, dev)
        result["ring_over_host_link"] = host_link_leg(P, W, torch, dev, up_bf16)

    # ---------------- oracle on the host cores ------------------------------------------------
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(W, wl)

    print(json.dumps(result))
    return 0


def ring_leg(P, W, torch, dev, up_bf16, name="flux1024_r4", reps=600):
    """A ring shard: all chunks resident (T_c), the chunk copies alone on the side stream (T_m),
    Algorithm 2 pipelined with the side stream (T_p), pipelined with the transfers riding in the
    attention launches (T_f), and copy-then-compute on one stream (T_s)."""
    wl = W.WORKLOADS[name]
    inp = W.make_attention_inputs(wl)
    q = up_bf16(inp.q)
    ks = [up_bf16(x) for x in inp.k]
    vs = [up_bf16(x) for x in inp.v]
    out = torch.empty_like(q)
    lse = torch.empty((wl.B, wl.H, wl.Sq), dtype=torch.float32, device=dev)
    scale = float(inp.softmax_scale)
    side = torch.cuda.Stream()
    desc = P.make_attn_desc(q, ks, out, scale, P.USP_ATTN_DOUBLE_BUFFER)
    ws = torch.empty((P.usp_ring_attn_workspace_bytes(desc),), dtype=torch.uint8, device=dev)
    desc1 = P.make_attn_desc(q, ks, out, scale, P.USP_ATTN_FUSED_PREFETCH)
    ws1 = torch.empty((P.usp_ring_attn_workspace_bytes(desc1),), dtype=torch.uint8, device=dev)
    stage = [torch.empty_like(ks[0]) for _ in range(4)]

    def timed(fn):
        for _ in range(reps // 2):          # also lets the clocks settle
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    def resident():       # one launch per chunk, as in the pipelined schedules
        P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=scale, flags=P.USP_ATTN_STEPWISE, out=out, lse=lse, workspace=ws)

    def one_launch():     # what the plain call does with resident chunks: their tiles as one stream
        P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=scale, out=out, lse=lse, workspace=ws)

    def pipelined():
        P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=scale, flags=P.USP_ATTN_DOUBLE_BUFFER, out=out, lse=lse,
                            workspace=ws, copy_stream=side)

    def fused():          # one launch per chunk, each carrying the transfer of the next chunk
        P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=scale, flags=P.USP_ATTN_FUSED_PREFETCH | P.USP_ATTN_STEPWISE,
                            out=out, lse=lse, workspace=ws1)

    def ring_one_launch():  # Algorithm 2 inside one launch: copy work-groups publish arrival counters
        P.usp_ring_attn_fwd(q, ks, vs, softmax_scale=scale, flags=P.USP_ATTN_FUSED_PREFETCH, out=out, lse=lse,
                            workspace=ws1)

    def copies_only():
        for r in range(1, wl.W):
            stage[0].copy_(ks[r], non_blocking=True)
            stage[1].copy_(vs[r], non_blocking=True)

    def serial():
        # copy-then-compute on one stream: a ring step that waits for its chunk before computing
        kk, vv = [ks[0]], [vs[0]]
        for r in range(1, wl.W):
            stage[2 * (r & 1)].copy_(ks[r], non_blocking=True)
            stage[2 * (r & 1) + 1].copy_(vs[r], non_blocking=True)
            kk.append(stage[2 * (r & 1)]); vv.append(stage[2 * (r & 1) + 1])
        P.usp_ring_attn_fwd(q, kk, vv, softmax_scale=scale, flags=P.USP_ATTN_STEPWISE, out=out, lse=lse, workspace=ws)

    t_c, t_m, t_p, t_f, t_s, t_1, t_r1 = (timed(f) for f in (resident, copies_only, pipelined, fused, serial, one_launch,
                                                            ring_one_launch))
    flops = wl.attn_flops()
    tf = lambda t: round(flops / (t * 1e-3) * 1e-12, 1)

    # The same ring with FP8 E4M3 K/V chunks and per-(head, token) scales (Algorithm 1 applied to the
    # ring payloads): half the bytes to move, a widening pass per chunk on arrival.
    kq, ksc, vq, vsc = [], [], [], []
    for k, v in zip(ks, vs):
        B, H, L, d = k.shape
        a, sa = P.usp_fp8_quant(k.reshape(B * H * L, d))
        b, sb = P.usp_fp8_quant(v.reshape(B * H * L, d))
        kq.append(a.reshape(B, H, L, d)); ksc.append(sa.reshape(B, H, L))
        vq.append(b.reshape(B, H, L, d)); vsc.append(sb.reshape(B, H, L))
    ws8 = torch.empty((max(P.usp_ring_attn_workspace_bytes(P.make_attn_desc(q, kq, out, scale, f))
                           for f in (P.USP_ATTN_STEPWISE, P.USP_ATTN_DOUBLE_BUFFER, P.USP_ATTN_FUSED_PREFETCH,
                                     P.USP_ATTN_FUSED_PREFETCH | P.USP_ATTN_STEPWISE)),),
                      dtype=torch.uint8, device=dev)
    st8 = [[torch.empty_like(kq[0]), torch.empty_like(ksc[0]), torch.empty_like(vq[0]), torch.empty_like(vsc[0])]
           for _ in range(2)]

    def fp8_call(flags, **kw):
        P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, softmax_scale=scale, flags=flags, out=out, lse=lse,
                            workspace=ws8, **kw)

    def fp8_copies_only():
        for r in range(1, wl.W):
            for dst, src in zip(st8[0], (kq[r], ksc[r], vq[r], vsc[r])):
                dst.copy_(src, non_blocking=True)

    def fp8_serial():
        kk, sk, vv, sv = [kq[0]], [ksc[0]], [vq[0]], [vsc[0]]
        for r in range(1, wl.W):
            bufs = st8[r & 1]
            for dst, src in zip(bufs, (kq[r], ksc[r], vq[r], vsc[r])):
                dst.copy_(src, non_blocking=True)
            kk.append(bufs[0]); sk.append(bufs[1]); vv.append(bufs[2]); sv.append(bufs[3])
        P.usp_ring_attn_fwd(q, kk, vv, k_scales=sk, v_scales=sv, softmax_scale=scale, flags=P.USP_ATTN_STEPWISE,
                            out=out, lse=lse, workspace=ws8)

    t8_c, t8_m, t8_p, t8_f, t8_s, t8_1 = (timed(f) for f in (
        lambda: fp8_call(P.USP_ATTN_STEPWISE), fp8_copies_only,
        lambda: fp8_call(P.USP_ATTN_DOUBLE_BUFFER, copy_stream=side),
        lambda: fp8_call(P.USP_ATTN_FUSED_PREFETCH | P.USP_ATTN_STEPWISE), fp8_serial,
        lambda: fp8_call(P.USP_ATTN_FUSED_PREFETCH)))
    kv_bytes = lambda ts, ss: sum(t.numel() * t.element_size() for t in ts[1:]) + sum(t.numel() * 4 for t in ss[1:])
    fp8 = {"t_compute_ms": round(t8_c, 4), "t_copies_ms": round(t8_m, 4), "t_side_stream_ms": round(t8_p, 4),
           "t_fused_prefetch_ms": round(t8_f, 4), "t_serial_ms": round(t8_s, 4),
           "hidden_fraction_fused_prefetch": round(max(0.0, min(1.0, 1.0 - (t8_f - t8_c) / t8_m)), 3) if t8_m > 0 else None,
           "serial_over_fused_prefetch": round(t8_s / t8_f, 3),
           "t_one_launch_ms": round(t8_1, 4), "tflops_one_launch": tf(t8_1),
           "serial_over_one_launch": round(t8_s / t8_1, 3), "one_launch_over_bf16_one_launch": round(t8_1 / t_r1, 3),
           "bytes_moved_bf16": 2 * kv_bytes(ks, []), "bytes_moved_fp8": kv_bytes(kq, ksc) + kv_bytes(vq, vsc),
           "compute_over_bf16": round(t8_c / t_c, 3),
           "note": "per-chunk forms: each chunk's codes are widened to bf16 (scales folded into the per-key records) "
                   "by a launch of its own before its attention launch; one launch: copy work-groups of the "
                   "attention launch decode chunk r+1 while chunk r is computed on (the plain call and "
                   "USP_ATTN_FUSED_PREFETCH give this same launch)"}
    # the same bf16 ring with a key mask on its last chunk (its last tenth of the keys dead, as padded
    # text tokens would be): one launch per chunk against the one launch over the ring
    km = [None] * (wl.W - 1) + [torch.ones((wl.B, wl.chunk_len[-1]), dtype=torch.uint8, device=dev)]
    km[-1][:, -(sum(wl.chunk_len) // 10):] = 0
    t_mk_c = timed(lambda: P.usp_ring_attn_fwd(q, ks, vs, key_mask=km, softmax_scale=scale, flags=P.USP_ATTN_STEPWISE,
                                               out=out, lse=lse, workspace=ws1))
    t_mk_1 = timed(lambda: P.usp_ring_attn_fwd(q, ks, vs, key_mask=km, softmax_scale=scale, out=out, lse=lse, workspace=ws1))
    masked = {"dead_keys": int(sum(wl.chunk_len) // 10), "t_per_chunk_ms": round(t_mk_c, 4), "t_plain_call_ms": round(t_mk_1, 4),
              "plain_call_over_unmasked_one_launch": round(t_mk_1 / t_1, 3),
              "note": "the plain call takes one launch over the ring (per-tile records for every chunk) where the ring "
                      "steps are short or every chunk is masked, else one launch per chunk"}
    hid = lambda t: round(max(0.0, min(1.0, 1.0 - (t - t_c) / t_m)), 3) if t_m > 0 else None
    return {"workload": "%s: Sq=%d, %d chunks of %d, H=%d d=%d bf16" % (name, wl.Sq, wl.W, wl.chunk_len[0], wl.H, wl.d),
            "t_compute_ms": round(t_c, 4), "t_copies_ms": round(t_m, 4),
            "t_side_stream_ms": round(t_p, 4), "t_fused_prefetch_ms": round(t_f, 4), "t_serial_ms": round(t_s, 4),
            "hidden_fraction_side_stream": hid(t_p), "hidden_fraction_fused_prefetch": hid(t_f),
            "serial_over_side_stream": round(t_s / t_p, 3), "serial_over_fused_prefetch": round(t_s / t_f, 3),
            "tflops_resident": tf(t_c), "tflops_side_stream": tf(t_p), "tflops_fused_prefetch": tf(t_f),
            "t_resident_one_launch_ms": round(t_1, 4), "tflops_resident_one_launch": tf(t_1),
            "frac_of_bf16_peak_one_launch": round(flops / (t_1 * 1e-3) * 1e-12 / PEAK_BF16_TFLOPS, 4),
            "t_pipelined_one_launch_ms": round(t_r1, 4), "tflops_pipelined_one_launch": tf(t_r1),
            "hidden_fraction_one_launch": round(max(0.0, min(1.0, 1.0 - (t_r1 - t_1) / t_m)), 3) if t_m > 0 else None,
            "serial_over_pipelined_one_launch": round(t_s / t_r1, 3),
            "fp8_kv": fp8, "masked_last_chunk": masked,
            "note": "on-device copies stand in for ring recv; an xGMI link is ~50x slower"}


def host_link_leg(P, W, torch, dev, up_bf16, name="flux1024_r4", reps=30):
    """The ring with a slow link: chunks 1..W-1 sit in pinned host memory, so every transfer of
    Algorithm 2 crosses the host link (tens of GB/s, the order of one xGMI link) instead of HBM.
    bf16 and FP8 payloads, three schedules each: copy then compute on one stream, the side-stream
    double buffering, and the whole ring as one launch whose copy work-groups pull the chunks."""
    wl = W.WORKLOADS[name]
    inp = W.make_attention_inputs(wl)
    q = up_bf16(inp.q)
    ks = [up_bf16(x) for x in inp.k]
    vs = [up_bf16(x) for x in inp.v]
    out = torch.empty_like(q)
    lse = torch.empty((wl.B, wl.H, wl.Sq), dtype=torch.float32, device=dev)
    scale = float(inp.softmax_scale)
    side = torch.cuda.Stream()
    host = lambda t: torch.empty(t.shape, dtype=t.dtype, pin_memory=True).copy_(t)
    kq, ksc, vq, vsc = [], [], [], []
    for k, v in zip(ks, vs):
        B, H, L, d = k.shape
        a, sa = P.usp_fp8_quant(k.reshape(B * H * L, d))
        b, sb = P.usp_fp8_quant(v.reshape(B * H * L, d))
        kq.append(a.reshape(B, H, L, d)); ksc.append(sa.reshape(B, H, L))
        vq.append(b.reshape(B, H, L, d)); vsc.append(sb.reshape(B, H, L))
    torch.cuda.synchronize()
    far = lambda ts: [ts[0]] + [host(t) for t in ts[1:]]        # chunk 0 is the rank's own
    ks_h, vs_h, kq_h, ksc_h, vq_h, vsc_h = (far(x) for x in (ks, vs, kq, ksc, vq, vsc))
    flags_all = (P.USP_ATTN_STEPWISE, P.USP_ATTN_DOUBLE_BUFFER, P.USP_ATTN_FUSED_PREFETCH)
    size = lambda kk: max(P.usp_ring_attn_workspace_bytes(P.make_attn_desc(q, kk, out, scale, f)) for f in flags_all)
    ws = torch.empty((max(size(ks), size(kq)),), dtype=torch.uint8, device=dev)

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    def schedules(kk, vv, sk=None, sv=None):
        kw = {} if sk is None else {"k_scales": sk, "v_scales": sv}
        stage = [[torch.empty(t[1].shape, dtype=t[1].dtype, device=dev) for t in ((kk, vv) if sk is None else (kk, vv, sk, sv))]
                 for _ in range(2)]

        def serial():
            lists = [[t[0]] for t in ((kk, vv) if sk is None else (kk, vv, sk, sv))]
            for r in range(1, wl.W):
                for j, t in enumerate((kk, vv) if sk is None else (kk, vv, sk, sv)):
                    stage[r & 1][j].copy_(t[r], non_blocking=True)
                    lists[j].append(stage[r & 1][j])
            kw2 = {} if sk is None else {"k_scales": lists[2], "v_scales": lists[3]}
            P.usp_ring_attn_fwd(q, lists[0], lists[1], softmax_scale=scale, flags=P.USP_ATTN_STEPWISE, out=out, lse=lse,
                                workspace=ws, **kw2)

        def copies():
            for r in range(1, wl.W):
                for j, t in enumerate((kk, vv) if sk is None else (kk, vv, sk, sv)):
                    stage[0][j].copy_(t[r], non_blocking=True)

        t_m = timed(copies)
        t_s = timed(serial)
        t_p = timed(lambda: P.usp_ring_attn_fwd(q, kk, vv, softmax_scale=scale, flags=P.USP_ATTN_DOUBLE_BUFFER, out=out, lse=lse,
                                                workspace=ws, copy_stream=side, **kw))
        t_1 = timed(lambda: P.usp_ring_attn_fwd(q, kk, vv, softmax_scale=scale, flags=P.USP_ATTN_FUSED_PREFETCH, out=out, lse=lse,
                                                workspace=ws, **kw))
        nbytes = sum(t[r].numel() * t[r].element_size() for t in ((kk, vv) if sk is None else (kk, vv, sk, sv)) for r in range(1, wl.W))
        return {"bytes_over_link": nbytes, "t_copies_ms": round(t_m, 4), "link_gbs": round(nbytes / (t_m * 1e-3) * 1e-9, 1),
                "t_serial_ms": round(t_s, 4), "t_side_stream_ms": round(t_p, 4), "t_one_launch_ms": round(t_1, 4),
                "serial_over_side_stream": round(t_s / t_p, 3), "serial_over_one_launch": round(t_s / t_1, 3)}

    bf = schedules(ks_h, vs_h)
    f8 = schedules(kq_h, vq_h, ksc_h, vsc_h)
    return {"workload": "%s with chunks 1..%d in pinned host memory" % (name, wl.W - 1), "bf16": bf, "fp8": f8,
            "fp8_over_bf16_one_launch": round(bf["t_one_launch_ms"] / f8["t_one_launch_ms"], 3),
            "note": "the host link stands in for a ring link; compute per call is ~0.08 ms, so every schedule is "
                    "bound by the link and FP8 payloads halve the time"}


def d64_leg(P, torch, dev, reps=200):
    """bf16 with head dimension 64 on the FLUX-1024 token count (one chunk)."""
    B, H, S, d = 1, 24, 4608, 64
    g = torch.Generator(device=dev).manual_seed(5)
    q, k, v = (torch.randn((B, H, S, d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16) for _ in range(3))
    out = torch.empty_like(q)
    lse = torch.empty((B, H, S), dtype=torch.float32, device=dev)
    desc = P.make_attn_desc(q, [k], out, 0.125, 0)
    ws = torch.empty((P.usp_ring_attn_workspace_bytes(desc),), dtype=torch.uint8, device=dev)
    call = lambda: P.usp_ring_attn_fwd(q, [k], [v], softmax_scale=0.125, out=out, lse=lse, workspace=ws)
    for _ in range(reps // 2):
        call()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        call()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / reps
    flops = 4.0 * B * H * S * S * d
    return {"workload": "B=1 H=24 d=64 Sq=S=4608 bf16, one chunk", "ms": round(ms, 4),
            "tflops": round(flops / (ms * 1e-3) * 1e-12, 1),
            "frac_of_bf16_peak": round(flops / (ms * 1e-3) * 1e-12 / PEAK_BF16_TFLOPS, 4),
            "note": "K and V read in place through a 128-byte-row tile layout (no padded copies); per flop the softmax "
                    "work is twice that of d = 128"}


def qwen_leg(P, W, torch, dev, up_bf16, reps=200):
    """Qwen-Image-like shard: FP8 K/V chunks (quantised here by usp_fp8_quant) with per-token scales
    and the key mask of the padded text tokens; all chunks resident."""
    wl = W.WORKLOADS["qwen_r2"]
    inp = W.make_attention_inputs(wl, heads=wl.H)
    q = up_bf16(inp.q)
    kq, ksc, vq, vsc = [], [], [], []
    for k, v in zip(inp.k, inp.v):
        B, H, L, d = k.shape
        a, sa = P.usp_fp8_quant(up_bf16(k).reshape(B * H * L, d))
        b, sb = P.usp_fp8_quant(up_bf16(v).reshape(B * H * L, d))
        kq.append(a.reshape(B, H, L, d)); ksc.append(sa.reshape(B, H, L))
        vq.append(b.reshape(B, H, L, d)); vsc.append(sb.reshape(B, H, L))
    km = [torch.from_numpy(m).to(dev) for m in inp.key_mask]
    out = torch.empty_like(q)
    lse = torch.empty((wl.B, wl.H, wl.Sq), dtype=torch.float32, device=dev)
    scale = float(inp.softmax_scale)
    desc = P.make_attn_desc(q, kq, out, scale, 0)
    ws = torch.empty((P.usp_ring_attn_workspace_bytes(desc),), dtype=torch.uint8, device=dev)

    def call():
        P.usp_ring_attn_fwd(q, kq, vq, k_scales=ksc, v_scales=vsc, key_mask=km, softmax_scale=scale,
                            out=out, lse=lse, workspace=ws)
    for _ in range(reps // 2):
        call()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        call()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / reps
    live = sum(int(m[0].sum()) for m in inp.key_mask)
    return {"workload": "qwen_r2: Sq=4096, 2 chunks of 4096 FP8 E4M3 K/V + per-token scales, H=24 d=128, %d of %d keys live"
                        % (live, wl.S),
            "ms": round(ms, 4), "tflops_nominal": round(wl.attn_flops() / (ms * 1e-3) * 1e-12, 1),
            "tflops_live_keys": round(wl.attn_flops() * live / wl.S / (ms * 1e-3) * 1e-12, 1),
            "includes": "record preparation, FP8 widening of K and dequantisation of V, attention, merge"}


def cpu_baseline(W, wl, heads=24):
    """The fp64 oracle, untuned, on a bounded sample: `heads` of the 24 heads of the shard's
    attention (all queries, all keys) plus the whole FP8 payload pack/unpack."""
    from oracle import usp_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    inp = W.make_attention_inputs(wl, heads=heads)
    x = W.make_payload(wl)
    t0 = time.perf_counter()
    orc.attention(inp.q, inp.k[0], inp.v[0], float(inp.softmax_scale))
    t_attn = time.perf_counter() - t0
    t0 = time.perf_counter()
    codes, s = orc.fp8_quant(x)
    orc.fp8_dequant_bf16(codes, s)
    t_fp8 = time.perf_counter() - t0
    step_s = t_attn * (wl.H / heads) + t_fp8       # scaled to one whole step
    return {"value": round(wl.attn_flops() / step_s * 1e-12, 5), "unit": "TFLOP/s", "cores": int(cores),
            "kind": "oracle",
            "sample": "%d of %d heads of flux1024_u attention (%.1f s) scaled x%g, plus the full "
                      "[4608,3072] FP8 pack+unpack (%.1f s); fp64 numpy reference, not a tuned CPU baseline"
                      % (heads, wl.H, t_attn, wl.H / heads, t_fp8)}


if __name__ == "__main__":
    sys.exit(main())
