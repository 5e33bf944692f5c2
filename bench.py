#!/usr/bin/env python3
"""Benchmark of the GG constrained tensor pass on one MI355X.

A step is one whole pass (per-segment fit -> step Delta = alpha/16 -> quantise -> Map ->
Exp-Golomb-0 bit count and u_max) over the flat 1.5-billion-element fp32 gradient bucket of a
28-layer transformer (253 segments), inputs resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--small] [--no-cpu] [--extra]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "GG fit+quantize+rate+penalty: Gelem/s and % of HBM roofline on 1 MI355X"
HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
ALGO_BYTES_PER_ELEM = 8.0      # fp32 bucket: 4 B read by the moment sweep + 4 B read by the rate sweep

# HBM traffic per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this same command, scaled by a plain-copy calibration; the summaries live under profiles/.
# None until measured for the kernel that currently ships.
MEASURED_TRAFFIC_BYTES = 6174859674 + 510157   # k_quant on the 1,543,655,424-element bucket: FETCH_SIZE 3015068.2 x 2 KiB
#                                                (factor from a 1 GiB copy) + WRITE_SIZE 498.2 KiB; profiles/k_quant_c4_bucket.md


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--small", action="store_true", help="1/64-scale bucket (quick functional run)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--extra", action="store_true", help="also time the penalty variant and the sampler")
    ap.add_argument("--all", action="store_true", help="--extra plus the other benchmark configurations (C1, C2, C3, C5)")
    ap.add_argument("--cpu-sample-elems", type=int, default=380_000_000)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain device copy of known size (counter calibration under rocprofv3 --pmc)")
    return ap.parse_args()


def time_steps(fn, steps, torch):
    """Wall time of `steps` back-to-back calls, bracketed by synchronisation, plus HIP-event time."""
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        fn()
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return wall_ms / steps, ev0.elapsed_time(ev1) / steps


def other_configs(gg, gg_inputs, torch, dev, args):
    """The remaining benchmark configurations, each timed as one whole call (HIP events, 10 calls)."""
    res = {}
    reps = 10

    def timed(fn):
        fn()
        return time_steps(fn, reps, torch)[1]

    # C1: 1024x1024 fp32, fit + Delta=alpha/16 + histogram/entropy/EG bits + penalty written
    n = 1 << 20
    x = gg_inputs.make_tensor((n,), 0.02, 1.0, seed=0, device=dev)
    ws = gg.Workspace(n, 1, device=dev)
    grad = torch.empty(n, dtype=torch.float32, device=dev)
    ms = timed(lambda: gg.gg_fused_segmented(x, [0, n], ws, delta_div=16.0, nbins=4096, lam=1e-4, grad=grad))
    res["C1_1024x1024_f32_fit_hist_penalty"] = {"ms": round(ms, 4), "Gelem/s": round(n / ms / 1e6, 2),
                                                "algorithmic_GB/s": round(12.0 * n / ms / 1e6, 1)}
    # C2: 4096x11008 bf16 weight, fit + rate (Delta=alpha/32) + penalty -> fp32
    n = 4096 * 11008
    x = gg_inputs.make_tensor((n,), 0.015, 1.5, seed=1, device=dev, dtype=torch.bfloat16)
    ws = gg.Workspace(n, 1, device=dev)
    grad = torch.empty(n, dtype=torch.float32, device=dev)
    ms = timed(lambda: gg.gg_fused_segmented(x, [0, n], ws, delta_div=32.0, lam=1e-4, grad=grad))
    res["C2_4096x11008_bf16_fit_rate_penalty"] = {"ms": round(ms, 4), "Gelem/s": round(n / ms / 1e6, 2),
                                                  "algorithmic_GB/s": round(8.0 * n / ms / 1e6, 1)}
    # C3: [8*2048, 4096] bf16 activations with outliers: per-row + per-tensor fit, per-row rates, tensor histogram
    rows, cols = 8 * 2048, 4096
    n = rows * cols
    x = gg_inputs.make_tensor((rows, cols), 0.5, 0.8, seed=2, device=dev, dtype=torch.bfloat16, outlier_frac=1e-3,
                              outlier_scale=20.0).reshape(-1)
    ws = gg.Workspace(n, rows, device=dev)
    r0 = gg.gg_fused_rows(x, rows, cols, ws, delta_div=8.0, want_total=True)
    tot_alpha = float(gg.fit_records(r0["total"])[0]["alpha"])
    ms_rows = timed(lambda: gg.gg_fused_rows(x, rows, cols, ws, delta_div=8.0, want_total=True))
    ms_hist = timed(lambda: gg.gg_quantize_rate(x, tot_alpha / 8.0, ws, nbins=32768))
    res["C3_16384x4096_bf16_rows_fit_rate"] = {"ms": round(ms_rows, 4), "Gelem/s": round(n / ms_rows / 1e6, 2),
                                               "algorithmic_GB/s": round(4.0 * n / ms_rows / 1e6, 1)}
    res["C3_tensor_histogram_32768_bins"] = {"ms": round(ms_hist, 4), "Gelem/s": round(n / ms_hist / 1e6, 2),
                                             "algorithmic_GB/s": round(2.0 * n / ms_hist / 1e6, 1)}
    del x, grad
    if not args.small:
        # C5: 7B-shaped bf16 weight set, fused fit + penalty accumulated into fp32 (and write-only)
        layout = gg_inputs.weights_7b()
        flat, off, _, _ = gg_inputs.make_bucket(layout, seed=4, device=dev, dtype=torch.bfloat16,
                                                alpha_range=(0.005, 0.03), beta_range=(0.6, 2.0), log_alpha=False)
        n, S = int(off[-1]), len(layout)
        ws = gg.Workspace(n, S, device=dev)
        grad = torch.zeros(n, dtype=torch.float32, device=dev)
        reps = 3
        ms_acc = timed(lambda: gg.gg_fused_segmented(flat, off, ws, want_rate=False, lam=1e-4, grad=grad, accumulate=True))
        ms_wr = timed(lambda: gg.gg_fused_segmented(flat, off, ws, want_rate=False, lam=1e-4, grad=grad, accumulate=False))
        res["C5_7B_bf16_fit_penalty_accumulate"] = {"ms": round(ms_acc, 3), "Gelem/s": round(n / ms_acc / 1e6, 2),
                                                    "algorithmic_GB/s": round(12.0 * n / ms_acc / 1e6, 1)}
        res["C5_7B_bf16_fit_penalty_write"] = {"ms": round(ms_wr, 3), "Gelem/s": round(n / ms_wr / 1e6, 2),
                                               "algorithmic_GB/s": round(8.0 * n / ms_wr / 1e6, 1)}
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import gg_inputs
    import paper_2506_00486_amd as gg

    gg.lib()  # fail loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)

    layout = gg_inputs.gradient_bucket_1p5b()
    if args.small:
        layout = gg_inputs.scaled_layout(layout, 64, ragged=False)
    t_gen = time.perf_counter()
    flat, off, _, _ = gg_inputs.make_bucket(layout, seed=3, device=dev, dtype=torch.float32)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    n, S = int(off[-1]), len(layout)
    ws = gg.Workspace(n, S, device=dev)
    fit = torch.empty(S * 40, dtype=torch.uint8, device=dev)
    rate = torch.empty(S * 48, dtype=torch.uint8, device=dev)

    def step():
        gg.gg_fused_segmented(flat, off, ws, delta_div=16.0, eg_k=0, fit=fit, rate=rate)

    for _ in range(args.warmup):
        step()
    ms_wall, ms_ev = time_steps(step, args.steps, torch)
    value = n / (ms_wall * 1e-3) / 1e9

    # dominant kernel: the rate sweep (k_quant).  Timed on its own stream-ordered call with HIP events:
    # the call also enqueues three tiny kernels (table upload, per-unit parameters, finalisation).
    frec = gg.fit_records(fit)
    delta = gg.gg_delta_from_fit(fit, S, 16.0)
    rate2 = torch.empty(S * 48, dtype=torch.uint8, device=dev)

    def rate_only():
        lib_rc = gg.lib().gg_quantize_rate_segmented(flat.data_ptr(), 0, off.ctypes.data, S, delta.data_ptr(), 0, 0, 0,
                                                     None, None, rate2.data_ptr(), ws.ptr, ws.bytes,
                                                     torch.cuda.current_stream().cuda_stream)
        assert lib_rc == 0

    def fit_only():
        gg.gg_fit_segmented(flat, off, ws, out=fit)

    rate_only()
    _, ms_rate = time_steps(rate_only, args.steps, torch)
    _, ms_fit = time_steps(fit_only, args.steps, torch)
    assert rate2.cpu().numpy().tobytes() == rate.cpu().numpy().tobytes()
    algo_bytes_kernel = 4.0 * n
    achieved = algo_bytes_kernel / (ms_rate * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "k_quant (rate sweep)", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None if args.small else MEASURED_TRAFFIC_BYTES,
                "algorithmic_bytes_per_launch": algo_bytes_kernel, "avg_launch_ms": round(ms_rate, 4),
                "fit_sweep_ms": round(ms_fit, 4),
                "whole_pass": {"algorithmic_bytes": ALGO_BYTES_PER_ELEM * n, "ms": round(ms_ev, 4),
                               "achieved": round(ALGO_BYTES_PER_ELEM * n / (ms_ev * 1e-3) / 1e9, 1),
                               "frac": round(ALGO_BYTES_PER_ELEM * n / (ms_ev * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}}

    out = {"metric": METRIC, "value": round(value, 2), "unit": "Gelem/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(ms_wall, 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": ("flat fp32 gradient bucket, 28-layer transformer (hidden 1536, FFN 8960, vocab 151936, "
                                   "GQA kv 256), %d segments, %d elements, GGD(alpha~LogU(1e-5,1e-3), beta~U(0.5,1.5)) seed 3; "
                                   "one gg_fused_segmented call: per-segment fit, Delta=alpha/16, EG-0 bits + u_max" % (S, n))
                      + (" [1/64 scale]" if args.small else ""),
                      "elements": n, "segments": S, "input_generation_s": round(t_gen, 2)},
           "roofline": roofline}

    if args.calibrate_copy:
        # 2^28 fp32 = 1 GiB read + 1 GiB written by a plain copy kernel: what FETCH_SIZE / WRITE_SIZE
        # report for it gives the scale of those counters on this machine
        m = min(n, 1 << 28)
        dst = torch.empty(m, dtype=torch.float32, device=dev)
        for _ in range(3):
            dst.copy_(flat[:m])
        torch.cuda.synchronize()
        out["calibration_copy_bytes_each_way"] = 4 * m
        del dst

    if args.all:
        args.extra = True
    if args.extra:
        extra = {}
        grad = torch.zeros(n, dtype=torch.float32, device=dev)

        def step_pen():
            gg.gg_fused_segmented(flat, off, ws, delta_div=16.0, eg_k=0, fit=fit, rate=rate, lam=1e-4, grad=grad)

        step_pen()
        _, ms_pen = time_steps(step_pen, max(3, args.steps // 2), torch)
        extra["with_penalty_written"] = {"ms": round(ms_pen, 4), "Gelem/s": round(n / ms_pen / 1e6, 2),
                                         "algorithmic_GB/s": round(12.0 * n / ms_pen / 1e6, 1)}
        del grad
        # one-sweep mode: steps given up front (e.g. from the previous training step): x is read once
        delta1 = gg.gg_delta_from_fit(fit, S, 16.0)

        def step_one_sweep():
            gg.gg_fused_segmented(flat, off, ws, delta_div=0.0, delta=delta1, eg_k=0, fit=fit, rate=rate)

        step_one_sweep()
        _, ms_1 = time_steps(step_one_sweep, max(3, args.steps // 2), torch)
        extra["one_sweep_given_steps"] = {"ms": round(ms_1, 4), "Gelem/s": round(n / ms_1 / 1e6, 2),
                                          "algorithmic_GB/s": round(4.0 * n / ms_1 / 1e6, 1)}
        ns = 202_383_360 if not args.small else 202_383_360 // 64
        xs = torch.empty(ns, dtype=torch.bfloat16, device=dev)

        def step_sample():
            gg.gg_sample(ns, 0.0156, 0.9, seed=4, out=xs)

        step_sample()
        _, ms_s = time_steps(step_sample, 5, torch)
        extra["gg_sample_bf16"] = {"elements": ns, "ms": round(ms_s, 4), "Gsamples/s": round(ns / ms_s / 1e6, 2),
                                   "written_GB/s": round(2.0 * ns / ms_s / 1e6, 1),      # ALU-bound: a few % of the HBM peak
                                   "frac_of_hbm_peak": round(2.0 * ns / ms_s / 1e6 / HBM_PEAK_GBS, 4)}
        del xs
        # companions: GCT update over the same bucket (reads g, ghat_prev, w; writes ghat, w = 20 B/elem),
        # rate gradient (4 B read + 4 B written), Exp-Golomb bit-stream encoder on a 64M-symbol slice
        delta = gg.gg_delta_from_fit(fit, S, 16.0)
        wbuf = torch.zeros(n, dtype=torch.float32, device=dev)
        gprev = flat.clone()

        def step_gct():
            gg.gg_gct_update_segmented(wbuf, flat, gprev, off, delta, 1e-3, 0.1, 1e-8, ws)

        step_gct()
        _, ms_g = time_steps(step_gct, 5, torch)
        extra["gct_update_segmented"] = {"ms": round(ms_g, 4), "Gelem/s": round(n / ms_g / 1e6, 2),
                                         "algorithmic_GB/s": round(20.0 * n / ms_g / 1e6, 1)}
        del gprev

        def step_rg():
            gg.gg_rate_grad(flat, 2.0 ** -16, grad=wbuf)

        step_rg()
        _, ms_r = time_steps(step_rg, 5, torch)
        extra["rate_grad"] = {"ms": round(ms_r, 4), "Gelem/s": round(n / ms_r / 1e6, 2),
                              "algorithmic_GB/s": round(8.0 * n / ms_r / 1e6, 1)}
        del wbuf
        m = min(n, 1 << 26)
        wsq = gg.Workspace(m, 1, device=dev)
        rec, _, sym = gg.gg_quantize_rate(flat[:m], float(frec["alpha"][0]) / 16.0, wsq, want_symbols=True)
        bits = int(gg.rate_records(rec)[0]["eg_bits"])

        bufs = gg.eg_buffers(m, (bits + 7) // 8, dev)

        def step_enc():
            gg.gg_eg_encode(sym, 0, buffers=bufs)

        step_enc()
        _, ms_e = time_steps(step_enc, 10, torch)
        stream_e, index_e, _ = gg.gg_eg_encode(sym, 0, buffers=bufs)
        assert int(bufs[2].item()) == bits                 # the stream is exactly as long as the rate sweep said
        back = torch.empty_like(sym)

        def step_dec():
            gg.gg_eg_decode(stream_e, index_e, m, 0, out=back)

        step_dec()
        _, ms_d = time_steps(step_dec, 10, torch)
        assert torch.equal(back, sym)
        d_enc = float(frec["alpha"][0]) / 16.0

        def step_enc_t():
            gg.gg_eg_encode_tensor(flat[:m], d_enc, 0, buffers=bufs)

        step_enc_t()
        _, ms_t = time_steps(step_enc_t, 10, torch)
        assert int(bufs[2].item()) == bits
        extra["eg_encode_tensor"] = {"elements": m, "ms": round(ms_t, 4), "Gelem/s": round(m / ms_t / 1e6, 2)}
        extra["eg_encode"] = {"symbols": m, "stream_bits": bits, "ms": round(ms_e, 4), "Gsymbols/s": round(m / ms_e / 1e6, 2)}
        extra["eg_decode"] = {"symbols": m, "ms": round(ms_d, 4), "Gsymbols/s": round(m / ms_d / 1e6, 2)}
        xhat = torch.zeros(m, device=dev)

        def step_dec_v():
            gg.gg_eg_decode_dequant(stream_e, index_e, m, d_enc, 0, out=xhat, accumulate=True)

        step_dec_v()
        _, ms_v = time_steps(step_dec_v, 10, torch)
        extra["eg_decode_dequant_accumulate"] = {"symbols": m, "ms": round(ms_v, 4), "Gsymbols/s": round(m / ms_v / 1e6, 2)}
        del back, stream_e, index_e, bufs, xhat
        del sym
        # the whole bucket, each segment with its own step, straight to one bit stream (what a compressed
        # gradient exchange would send): its length must be the sum of the segments' eg_bits of the pass
        rrec = gg.rate_records(rate)
        bucket_bits = int(rrec["eg_bits"].astype(np.uint64).sum())
        bbufs = gg.eg_buffers(n, (bucket_bits + 7) // 8, dev)

        def step_enc_b():
            gg.gg_eg_encode_segmented(flat, off, delta, ws, 0, buffers=bbufs)

        step_enc_b()
        _, ms_b = time_steps(step_enc_b, 5, torch)
        assert int(bbufs[2].item()) == bucket_bits
        extra["eg_encode_segmented_bucket"] = {"elements": n, "stream_bits": bucket_bits, "ms": round(ms_b, 4),
                                               "Gelem/s": round(n / ms_b / 1e6, 2),
                                               "bits_per_element": round(bucket_bits / n, 3)}
        # and back: the stream decoded straight to values, each unit with its step, added to an fp32 buffer
        tiles = (n + gg.GG_EG_TILE - 1) // gg.GG_EG_TILE
        xsum = torch.zeros(n, device=dev)

        def step_dec_b():
            gg.gg_eg_decode_dequant_segmented(bbufs[0], bbufs[1][: tiles + 1], off, delta, ws, 0, out=xsum, accumulate=True)

        step_dec_b()
        _, ms_db = time_steps(step_dec_b, 5, torch)
        extra["eg_decode_dequant_segmented_bucket"] = {"elements": n, "ms": round(ms_db, 4), "Gelem/s": round(n / ms_db / 1e6, 2)}
        del bbufs, xsum
        if args.all:
            extra.update(other_configs(gg, gg_inputs, torch, dev, args))
        out["extra"] = extra

    if not args.no_cpu:
        import oracle
        # bounded sample: the leading whole segments of the same bucket, ~cpu_sample_elems elements
        k = int(np.searchsorted(off, args.cpu_sample_elems, side="right")) - 1
        k = max(1, min(k, S))
        m = int(off[k])
        host = flat[:m].cpu().numpy()
        t0 = time.perf_counter()
        ofits, orates = oracle.fused_segmented(host, off[:k + 1], delta_div=16.0)
        dt = time.perf_counter() - t0
        # per-step cost of the oracle on a 16M-element slice (context for the individual rows of the pass)
        sl = host[: min(m, 1 << 24)]
        steps_ns = {}
        t0 = time.perf_counter(); f0 = oracle.fit(sl); steps_ns["fit"] = (time.perf_counter() - t0) / sl.size * 1e9
        t0 = time.perf_counter(); oracle.quantize_rate(sl, f0.alpha / 16.0); steps_ns["quantize_rate"] = (time.perf_counter() - t0) / sl.size * 1e9
        t0 = time.perf_counter(); oracle.penalty_grad(sl, f0.alpha, f0.beta, 1e-4); steps_ns["penalty_grad"] = (time.perf_counter() - t0) / sl.size * 1e9
        t0 = time.perf_counter(); oracle.sample(1 << 22, 0.02, 0.9, 1); steps_ns["sample"] = (time.perf_counter() - t0) / (1 << 22) * 1e9
        cpu_model = ""
        try:
            with open("/proc/cpuinfo") as fh:
                cpu_model = next((l.split(":", 1)[1].strip() for l in fh if l.startswith("model name")), "")
        except OSError:
            pass
        out["cpu_baseline"] = {"value": round(m / dt / 1e9, 4), "unit": "Gelem/s", "cores": 1, "kind": "oracle",
                               "sample": "first %d segments (%d elements) of the same bucket, %.1f s" % (k, m, dt),
                               "ns_per_elem": {k_: round(v, 2) for k_, v in steps_ns.items()},
                               "host": {"cpu": cpu_model, "nproc": os.cpu_count()}}
        # the sample doubles as a last sanity check of the timed configuration
        rrec = gg.rate_records(rate)
        for s in range(k):
            assert abs(float(frec[s]["beta"]) - ofits[s].beta) <= 1e-4 * ofits[s].beta, (s, frec[s], ofits[s])

    print(json.dumps(out))


if __name__ == "__main__":
    main()
