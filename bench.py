#!/usr/bin/env python3
"""Benchmark of the GG constrained tensor pass on one MI355X.

A step is one whole pass (per-segment fit -> step Delta = alpha/16 -> quantise -> Map ->
Exp-Golomb-0 bit count and u_max) over the flat 1.5-billion-element fp32 gradient bucket of a
28-layer transformer (253 segments), inputs resident in HBM.  Prints ONE JSON line: the headline
(`value`, `roofline`), every other benchmark configuration under `configs` (the same bucket with
the penalty gradient written, the 1024x1024 tensor, the bf16 weight, the activation tensor by rows
and its histogram, the 7B weight set, the sampler), and the oracle's speed on the host
(`cpu_baseline`).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--small] [--no-cpu] [--only NAMES] [--extra]
"""
import argparse
import hashlib
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "GG fit+quantize+rate+penalty: Gelem/s and % of HBM roofline on 1 MI355X"
HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
ALGO_BYTES_PER_ELEM = 8.0      # fp32 bucket: 4 B read by the moment sweep + 4 B read by the rate sweep
# gg_sample is bound by the vector ALUs: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-operations/s,
# about 130 issue slots per Marsaglia-Tsang attempt (10 Philox rounds as 20 quarter-rate 32x32->64 multiplies,
# Box-Muller, the accept test, the power) -> 302 G attempts/s
SAMPLER_PEAK_GSAMPLES = 256 * 4 * 16 * 2.4 / 130.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.md")
KERNEL_SOURCES = ("gg_kernels.hip", "gg_device.h", "gg_geometry.h", "gen_solve_curve.py")   # what the pass kernels are built from
CONFIG_NAMES = ("C4_penalty", "C1", "C2", "C3", "C5", "sampler")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--small", action="store_true", help="1/64-scale inputs (quick functional run)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--only", default=None,
                    help="comma-separated subset of the other configurations to time (%s), or 'none'; default: all"
                         % ", ".join(CONFIG_NAMES))
    ap.add_argument("--extra", action="store_true", help="also time the companions (GCT update, rate gradient, bit-stream coder)")
    ap.add_argument("--cpu-sample-elems", type=int, default=380_000_000)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain device copy of known size (counter calibration under rocprofv3 --pmc)")
    return ap.parse_args()


def kernel_source_hash():
    """Fingerprint of the kernel sources: a measured HBM-traffic figure is only quoted for the code it was measured on."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2506_00486_amd", "csrc", name), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(key):
    """Bytes per launch of kernel `key` from the rocprofv3 counter summary under profiles/, or None when there is
    no line for it or the line was measured on other kernel sources than the ones in this tree."""
    try:
        text = open(TRAFFIC_FILE).read()
    except OSError:
        return None
    now = kernel_source_hash()
    for m in re.finditer(r"^traffic\s+(\S+)\s+fetch_bytes=(\d+)\s+write_bytes=(\d+)\s+sources=(\w+)", text, flags=re.M):
        if m.group(1) == key and m.group(4) == now:
            return int(m.group(2)) + int(m.group(3))
    return None


class Timer:
    """Whole calls timed one by one with a HIP event pair each (on torch's current stream, the stream the
    binding launches on): median and mean over the repetitions.  The timed calls write into buffers made
    beforehand, so that no allocation sits between the two events; an empty pair of events reads about 4.5 us
    on this machine, which the figures include."""

    def __init__(self, torch):
        self.torch = torch

    def each(self, fn, reps, warm=3):
        torch = self.torch
        for _ in range(warm):
            fn()
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        torch.cuda.synchronize()
        for a, b in pairs:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        ms = [a.elapsed_time(b) for a, b in pairs]
        return statistics.median(ms), sum(ms) / len(ms)

    def back_to_back(self, fn, steps):
        """Wall time of exactly `steps` calls bracketed by synchronisation on both sides."""
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps


def entry(n, ms_med, ms_mean, bytes_per_elem, kernel, reps, **more):
    """One configuration of the `configs` object: whole-call time and its HBM-roofline fraction."""
    algo = bytes_per_elem * n
    gbs = algo / (ms_med * 1e-3) / 1e9
    e = {"elements": n, "ms": round(ms_med, 4), "ms_mean": round(ms_mean, 4), "timed_calls": reps,
         "Gelem/s": round(n / ms_med / 1e6, 2), "algorithmic_bytes": int(algo), "achieved_GB/s": round(gbs, 1),
         "frac": round(gbs / HBM_PEAK_GBS, 4), "bound": "hbm", "dominant_kernel": kernel}
    e.update(more)
    return e


def other_configs(gg, gg_inputs, torch, dev, args, timer, bucket, want):
    """Every benchmark configuration besides the headline, each timed as whole calls (median of >= 20 where a
    call takes under a few milliseconds)."""
    res = {}
    flat, off, ws, fit, rate = bucket
    n4, scale = flat.numel(), (64 if args.small else 1)
    reps = max(20, args.steps)

    if "C4_penalty" in want:
        # the same bucket with the GG-prior penalty gradient written in the rate sweep: 4 + 4 read, 4 written
        grad = torch.empty(n4, dtype=torch.float32, device=dev)
        med, mean = timer.each(lambda: gg.gg_fused_segmented(flat, off, ws, delta_div=16.0, eg_k=0, fit=fit, rate=rate,
                                                             lam=1e-4, grad=grad), reps)
        res["C4_bucket_fit_rate_penalty_written"] = entry(n4, med, mean, 12.0, "k_quant_parts<float, rate + penalty>", reps,
                                                          traffic=measured_traffic("k_quant_c4_penalty"))
        del grad
    if "C1" in want:
        # 1024x1024 fp32, fit + Delta = alpha/16 + histogram / entropy / EG bits + penalty written
        n = 1 << 20
        x = gg_inputs.make_tensor((n,), 0.02, 1.0, seed=0, device=dev)
        w1 = gg.Workspace(n, 1, device=dev)
        grad = torch.empty(n, dtype=torch.float32, device=dev)
        o1 = gg.gg_fused_segmented(x, [0, n], w1, delta_div=16.0, nbins=4096, lam=1e-4, grad=grad)   # and the output buffers of the timed calls
        med, mean = timer.each(lambda: gg.gg_fused_segmented(x, [0, n], w1, delta_div=16.0, nbins=4096, lam=1e-4, grad=grad,
                                                             fit=o1["fit"], rate=o1["rate"], hist=o1["hist"]), 40)
        res["C1_1024x1024_f32_fit_hist_penalty"] = entry(n, med, mean, 12.0, "k_quant_parts<float, rate + histogram + penalty> (four dependent launches on a 4 MB tensor)", 40,
                                                         traffic=measured_traffic("k_quant_c1"))
        del x, grad
    if "C2" in want:
        # 4096x11008 bf16 weight, fit + rate (Delta = alpha/32) + penalty written as fp32
        n = 4096 * 11008 // scale
        x = gg_inputs.make_tensor((n,), 0.015, 1.5, seed=1, device=dev, dtype=torch.bfloat16)
        w2 = gg.Workspace(n, 1, device=dev)
        grad = torch.empty(n, dtype=torch.float32, device=dev)
        o2 = gg.gg_fused_segmented(x, [0, n], w2, delta_div=32.0, lam=1e-4, grad=grad)
        med, mean = timer.each(lambda: gg.gg_fused_segmented(x, [0, n], w2, delta_div=32.0, lam=1e-4, grad=grad,
                                                             fit=o2["fit"], rate=o2["rate"]), 40)
        res["C2_4096x11008_bf16_fit_rate_penalty"] = entry(n, med, mean, 8.0, "k_quant_parts<bf16, rate + penalty>", 40,
                                                           traffic=measured_traffic("k_quant_c2_penalty"))
        del x, grad
    if "C3" in want:
        # [8*2048, 4096] bf16 activations with outliers: per-row + per-tensor fit and per-row rates in one call,
        # then the tensor's histogram with the step of the whole-tensor fit
        rows, cols = 8 * 2048 // scale, 4096
        n = rows * cols
        x = gg_inputs.make_tensor((rows, cols), 0.5, 0.8, seed=2, device=dev, dtype=torch.bfloat16, outlier_frac=1e-3,
                                  outlier_scale=20.0).reshape(-1)
        w3 = gg.Workspace(n, rows, device=dev)
        r0 = gg.gg_fused_rows(x, rows, cols, w3, delta_div=8.0, want_total=True)
        tot_alpha = float(gg.fit_records(r0["total"])[0]["alpha"])
        med_r, mean_r = timer.each(lambda: gg.gg_fused_rows(x, rows, cols, w3, delta_div=8.0, want_total=True,
                                                            fit=r0["fit"], total=r0["total"], rate=r0["rate"]), 40)
        h0 = gg.gg_quantize_rate(x, tot_alpha / 8.0, w3, nbins=32768)
        med_h, mean_h = timer.each(lambda: gg.gg_quantize_rate(x, tot_alpha / 8.0, w3, nbins=32768, out=h0[0], hist=h0[1]), 40)
        # rows of 8 KiB stay in registers between the moment sums and the code lengths: the input moves once (2 B/element)
        res["C3_16384x4096_bf16_rows_fit_rate"] = entry(n, med_r, mean_r, 2.0, "k_rows_reg<bf16, 8 vectors per lane>", 40,
                                                        traffic=measured_traffic("k_rows_c3"))
        res["C3_tensor_histogram_32768_bins"] = entry(n, med_h, mean_h, 2.0, "k_hist<bf16>", 40,
                                                      traffic=measured_traffic("k_quant_c3_histogram"))
        # both calls against the 2 + 2 bytes per element the configuration has to move (each call reads the input once)
        t_r, t_h = measured_traffic("k_rows_c3"), measured_traffic("k_quant_c3_histogram")
        res["C3_both_calls"] = entry(n, med_r + med_h, mean_r + mean_h, 4.0, "k_rows_reg<bf16> + k_hist<bf16>", 40,
                                     traffic=(t_r + t_h) if (t_r is not None and t_h is not None) else None)
        del x
    if "C5" in want and not args.small:
        # 7B-shaped bf16 weight set, fused fit + penalty accumulated into fp32 (the update step), and written
        layout = gg_inputs.weights_7b()
        f5, o5, _, _ = gg_inputs.make_bucket(layout, seed=4, device=dev, dtype=torch.bfloat16,
                                             alpha_range=(0.005, 0.03), beta_range=(0.6, 2.0), log_alpha=False)
        n, S = int(o5[-1]), len(layout)
        w5 = gg.Workspace(n, S, device=dev)
        grad = torch.zeros(n, dtype=torch.float32, device=dev)
        fit5 = torch.empty(S * 40, dtype=torch.uint8, device=dev)
        med_a, mean_a = timer.each(lambda: gg.gg_fused_segmented(f5, o5, w5, want_rate=False, lam=1e-4, grad=grad, accumulate=True,
                                                                 fit=fit5), 20, warm=2)
        med_w, mean_w = timer.each(lambda: gg.gg_fused_segmented(f5, o5, w5, want_rate=False, lam=1e-4, grad=grad, accumulate=False,
                                                                 fit=fit5), 20, warm=2)
        res["C5_7B_bf16_fit_penalty_accumulate"] = entry(n, med_a, mean_a, 12.0, "k_quant<bf16, penalty, accumulate>", 20,
                                                         segments=S, traffic=measured_traffic("k_quant_c5_accumulate"))
        res["C5_7B_bf16_fit_penalty_write"] = entry(n, med_w, mean_w, 8.0, "k_quant<bf16, penalty, write>", 20, segments=S,
                                                    traffic=measured_traffic("k_quant_c5_write"))
        res["_c5_sample"] = (f5, o5, layout)          # kept for the cpu_baseline leg, removed before printing
        del grad, w5
    if "sampler" in want:
        # re-sampling one layer of the 7B set (202,383,360 bf16 elements) with the Gamma-based GG sampler
        ns = 202_383_360 // scale
        xs = torch.empty(ns, dtype=torch.bfloat16, device=dev)
        med, mean = timer.each(lambda: gg.gg_sample(ns, 0.0156, 0.9, seed=4, out=xs), 20)
        gs = ns / med / 1e6
        res["gg_sample_bf16_one_7B_layer"] = {"elements": ns, "ms": round(med, 4), "ms_mean": round(mean, 4), "timed_calls": 20,
                                              "Gsamples/s": round(gs, 2), "bound": "alu", "peak_Gsamples/s": round(SAMPLER_PEAK_GSAMPLES, 1),
                                              "frac": round(gs / SAMPLER_PEAK_GSAMPLES, 4), "written_GB/s": round(2.0 * gs, 1),
                                              "dominant_kernel": "k_sample<bf16>"}
        del xs
    return res


def companions(gg, torch, dev, args, timer, bucket, frec, np):
    """The training companions over the same bucket (not part of the default line)."""
    flat, off, ws, fit, rate = bucket
    n, S = flat.numel(), len(off) - 1
    extra = {}
    delta1 = gg.gg_delta_from_fit(fit, S, 16.0)
    med, _ = timer.each(lambda: gg.gg_fused_segmented(flat, off, ws, delta_div=0.0, delta=delta1, eg_k=0, fit=fit, rate=rate), 10)
    extra["one_sweep_given_steps"] = {"ms": round(med, 4), "Gelem/s": round(n / med / 1e6, 2), "algorithmic_GB/s": round(4.0 * n / med / 1e6, 1)}
    wbuf = torch.zeros(n, dtype=torch.float32, device=dev)
    gprev = flat.clone()
    med, _ = timer.each(lambda: gg.gg_gct_update_segmented(wbuf, flat, gprev, off, delta1, 1e-3, 0.1, 1e-8, ws), 5, warm=1)
    extra["gct_update_segmented"] = {"ms": round(med, 4), "Gelem/s": round(n / med / 1e6, 2), "algorithmic_GB/s": round(20.0 * n / med / 1e6, 1)}
    del gprev
    med, _ = timer.each(lambda: gg.gg_rate_grad(flat, 2.0 ** -16, grad=wbuf), 5, warm=1)
    extra["rate_grad"] = {"ms": round(med, 4), "Gelem/s": round(n / med / 1e6, 2), "algorithmic_GB/s": round(8.0 * n / med / 1e6, 1)}
    del wbuf
    m = min(n, 1 << 26)
    wsq = gg.Workspace(m, 1, device=dev)
    d_enc = float(frec["alpha"][0]) / 16.0
    rec, _, sym = gg.gg_quantize_rate(flat[:m], d_enc, wsq, want_symbols=True)
    bits = int(gg.rate_records(rec)[0]["eg_bits"])
    bufs = gg.eg_buffers(m, (bits + 7) // 8, dev)
    med_e, _ = timer.each(lambda: gg.gg_eg_encode(sym, 0, buffers=bufs), 10)
    stream_e, index_e, _ = gg.gg_eg_encode(sym, 0, buffers=bufs)
    assert int(bufs[2].item()) == bits                 # the stream is exactly as long as the rate sweep said
    back = torch.empty_like(sym)
    med_d, _ = timer.each(lambda: gg.gg_eg_decode(stream_e, index_e, m, 0, out=back), 10)
    assert torch.equal(back, sym)
    med_t, _ = timer.each(lambda: gg.gg_eg_encode_tensor(flat[:m], d_enc, 0, buffers=bufs), 10)
    assert int(bufs[2].item()) == bits
    extra["eg_encode_tensor"] = {"elements": m, "ms": round(med_t, 4), "Gelem/s": round(m / med_t / 1e6, 2)}
    extra["eg_encode"] = {"symbols": m, "stream_bits": bits, "ms": round(med_e, 4), "Gsymbols/s": round(m / med_e / 1e6, 2)}
    extra["eg_decode"] = {"symbols": m, "ms": round(med_d, 4), "Gsymbols/s": round(m / med_d / 1e6, 2)}
    xhat = torch.zeros(m, device=dev)
    med_v, _ = timer.each(lambda: gg.gg_eg_decode_dequant(stream_e, index_e, m, d_enc, 0, out=xhat, accumulate=True), 10)
    extra["eg_decode_dequant_accumulate"] = {"symbols": m, "ms": round(med_v, 4), "Gsymbols/s": round(m / med_v / 1e6, 2)}
    del back, stream_e, index_e, bufs, xhat, sym
    # the whole bucket, each segment with its own step, straight to one bit stream (what a compressed gradient
    # exchange would send): its length must be the sum of the segments' eg_bits of the pass
    rrec = gg.rate_records(rate)
    bucket_bits = int(rrec["eg_bits"].astype(np.uint64).sum())
    bbufs = gg.eg_buffers(n, (bucket_bits + 7) // 8, dev)
    med_b, _ = timer.each(lambda: gg.gg_eg_encode_segmented(flat, off, delta1, ws, 0, buffers=bbufs), 5, warm=1)
    assert int(bbufs[2].item()) == bucket_bits
    extra["eg_encode_segmented_bucket"] = {"elements": n, "stream_bits": bucket_bits, "ms": round(med_b, 4),
                                           "Gelem/s": round(n / med_b / 1e6, 2), "bits_per_element": round(bucket_bits / n, 3)}
    tiles = (n + gg.GG_EG_TILE - 1) // gg.GG_EG_TILE
    xsum = torch.zeros(n, device=dev)
    med_db, _ = timer.each(lambda: gg.gg_eg_decode_dequant_segmented(bbufs[0], bbufs[1][: tiles + 1], off, delta1, ws, 0, out=xsum,
                                                                     accumulate=True), 5, warm=1)
    extra["eg_decode_dequant_segmented_bucket"] = {"elements": n, "ms": round(med_db, 4), "Gelem/s": round(n / med_db / 1e6, 2)}
    return extra


def cpu_leg(args, np, gg, gg_inputs, torch, bucket, frec, c5):
    """The oracle as it stands, one thread, on the host: the headline workload on a bounded sample of leading whole
    segments, and the other configurations (the small ones whole, the 7B set on its first layer + the embedding)."""
    import oracle
    flat, off, ws, fit, rate = bucket
    S = len(off) - 1
    k = int(np.searchsorted(off, args.cpu_sample_elems, side="right")) - 1
    k = max(1, min(k, S))
    m = int(off[k])
    host = flat[:m].cpu().numpy()
    t0 = time.perf_counter()
    ofits, _ = oracle.fused_segmented(host, off[:k + 1], delta_div=16.0)
    dt = time.perf_counter() - t0
    for s in range(k):                     # the sample doubles as a last sanity check of the timed configuration
        assert abs(float(frec[s]["beta"]) - ofits[s].beta) <= 1e-4 * ofits[s].beta, (s, frec[s], ofits[s])
    # per-step cost on a 16M-element slice (context for the individual rows of the pass)
    sl = host[: min(m, 1 << 24)]
    steps_ns = {}
    t0 = time.perf_counter(); f0 = oracle.fit(sl); steps_ns["fit"] = (time.perf_counter() - t0) / sl.size * 1e9
    t0 = time.perf_counter(); oracle.quantize_rate(sl, f0.alpha / 16.0); steps_ns["quantize_rate"] = (time.perf_counter() - t0) / sl.size * 1e9
    t0 = time.perf_counter(); oracle.penalty_grad(sl, f0.alpha, f0.beta, 1e-4); steps_ns["penalty_grad"] = (time.perf_counter() - t0) / sl.size * 1e9
    t0 = time.perf_counter(); oracle.sample(1 << 22, 0.02, 0.9, 1); steps_ns["sample"] = (time.perf_counter() - t0) / (1 << 22) * 1e9
    cpu_model = ""
    try:
        with open("/proc/cpuinfo") as fh:
            cpu_model = next((ln.split(":", 1)[1].strip() for ln in fh if ln.startswith("model name")), "")
    except OSError:
        pass
    out = {"value": round(m / dt / 1e9, 4), "unit": "Gelem/s", "cores": 1, "kind": "oracle",
           "sample": "first %d segments (%d elements) of the same bucket, %.1f s" % (k, m, dt),
           "ns_per_elem": {k_: round(v, 2) for k_, v in steps_ns.items()},
           "host": {"cpu": cpu_model, "nproc": os.cpu_count()}}
    if args.small or args.only == "none":
        return out
    others = {}
    dev = flat.device

    def timed(label, n_elems, fn, note):
        t0 = time.perf_counter()
        fn()
        sec = time.perf_counter() - t0
        others[label] = {"Gelem/s": round(n_elems / sec / 1e9, 4), "seconds": round(sec, 2), "sample": note}

    # C4 with the penalty: a fifth of the headline sample
    k4 = max(1, int(np.searchsorted(off, args.cpu_sample_elems // 5, side="right")) - 1)
    m4 = int(off[k4])

    def c4_pen():
        for s in range(k4):
            seg = host[int(off[s]):int(off[s + 1])]
            f = oracle.fit(seg)
            oracle.quantize_rate(seg, float(np.float32(f.alpha) / np.float32(16.0)))
            oracle.penalty_grad(seg, f.alpha, f.beta, 1e-4)
    timed("C4_bucket_fit_rate_penalty_written", m4, c4_pen, "first %d segments (%d elements)" % (k4, m4))
    del host
    x1 = gg_inputs.make_tensor((1 << 20,), 0.02, 1.0, seed=0, device=dev).cpu().numpy()

    def c1():
        f = oracle.fit(x1)
        oracle.quantize_rate(x1, float(np.float32(f.alpha) / np.float32(16.0)), nbins=4096)
        oracle.penalty_grad(x1, f.alpha, f.beta, 1e-4)
    timed("C1_1024x1024_f32_fit_hist_penalty", x1.size, c1, "whole tensor")
    x2 = gg_inputs.torch_to_numpy_bits(gg_inputs.make_tensor((4096 * 11008,), 0.015, 1.5, seed=1, device=dev, dtype=torch.bfloat16))

    def c2():
        f = oracle.fit(x2)
        oracle.quantize_rate(x2, float(np.float32(f.alpha) / np.float32(32.0)))
        oracle.penalty_grad(x2, f.alpha, f.beta, 1e-4)
    timed("C2_4096x11008_bf16_fit_rate_penalty", x2.size, c2, "whole tensor")
    del x2
    rows, cols = 8 * 2048, 4096
    x3 = gg_inputs.torch_to_numpy_bits(gg_inputs.make_tensor((rows, cols), 0.5, 0.8, seed=2, device=dev, dtype=torch.bfloat16,
                                                             outlier_frac=1e-3, outlier_scale=20.0).reshape(-1))

    def c3():
        for r in range(rows):
            xs = x3[r * cols:(r + 1) * cols]
            f = oracle.fit(xs)
            oracle.quantize_rate(xs, float(np.float32(f.alpha) / np.float32(8.0)))
        f = oracle.fit(x3)
        oracle.quantize_rate(x3, float(np.float32(f.alpha) / np.float32(8.0)), nbins=32768)
    timed("C3_both_calls", x3.size, c3, "whole tensor: 16384 row fits + rates, tensor fit + histogram")
    del x3
    if c5 is not None:
        f5, o5, layout = c5
        # layer 0 (9 tensors) and the embedding: about 333 M of the 6.7 G elements, the rate scaled by element count
        picks = list(range(9)) + [len(layout) - 2]
        parts = [gg_inputs.torch_to_numpy_bits(f5[int(o5[s]):int(o5[s + 1])]) for s in picks]
        grads = [np.zeros(p.size, dtype=np.float32) for p in parts]

        def c5_acc():
            for p, g in zip(parts, grads):
                f = oracle.fit(p)
                oracle.penalty_grad(p, f.alpha, f.beta, 1e-4, grad=g, accumulate=True)
        timed("C5_7B_bf16_fit_penalty_accumulate", sum(p.size for p in parts), c5_acc,
              "layer 0 and the embedding (%d of %d elements), taken as representative of the set" % (sum(p.size for p in parts), int(o5[-1])))
        del parts, grads
    t0 = time.perf_counter()
    oracle.sample(1 << 23, 0.0156, 0.9, 4)
    sec = time.perf_counter() - t0
    others["gg_sample_bf16_one_7B_layer"] = {"Gsamples/s": round((1 << 23) / sec / 1e9, 4), "seconds": round(sec, 2),
                                             "sample": "8,388,608 of the 202,383,360 draws"}
    out["configs"] = others
    return out


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
    timer = Timer(torch)

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

    # headline: W untimed steps, then exactly K steps between two synchronisations (whole-job throughput)
    for _ in range(args.warmup):
        step()
    ms_wall = timer.back_to_back(step, args.steps)
    value = n / (ms_wall * 1e-3) / 1e9
    reps = max(20, args.steps)
    ms_step_med, ms_step_mean = timer.each(step, reps, warm=0)

    # dominant kernel: the rate sweep (k_quant), as the stream-ordered call that holds it, timed call by call with
    # HIP events; beside k_quant the call enqueues three kernels of a few microseconds (table upload, per-unit
    # parameters, folding of the run slots)
    frec = gg.fit_records(fit)
    delta = gg.gg_delta_from_fit(fit, S, 16.0)
    rate2 = torch.empty(S * 48, dtype=torch.uint8, device=dev)

    def rate_only():
        lib_rc = gg.lib().gg_quantize_rate_segmented(flat.data_ptr(), 0, off.ctypes.data, S, delta.data_ptr(), 0, 0, 0,
                                                     None, None, rate2.data_ptr(), ws.ptr, ws.bytes,
                                                     torch.cuda.current_stream().cuda_stream)
        assert lib_rc == 0

    ms_rate_med, ms_rate = timer.each(rate_only, reps, warm=1)
    ms_fit_med, ms_fit = timer.each(lambda: gg.gg_fit_segmented(flat, off, ws, out=fit), reps, warm=1)
    assert rate2.cpu().numpy().tobytes() == rate.cpu().numpy().tobytes()
    algo_bytes_kernel = 4.0 * n
    achieved = algo_bytes_kernel / (ms_rate * 1e-3) / 1e9
    whole = ALGO_BYTES_PER_ELEM * n / (ms_step_med * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "k_quant (rate sweep)", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": None if args.small else measured_traffic("k_quant_c4_rate"),
                "algorithmic_bytes_per_launch": algo_bytes_kernel, "avg_launch_ms": round(ms_rate, 4),
                "median_launch_ms": round(ms_rate_med, 4), "timed_launches": reps,
                "fit_sweep_ms": round(ms_fit_med, 4), "kernel_sources": kernel_source_hash(),
                "whole_pass": {"algorithmic_bytes": ALGO_BYTES_PER_ELEM * n, "ms": round(ms_step_med, 4),
                               "ms_mean": round(ms_step_mean, 4), "achieved": round(whole, 1),
                               "frac": round(whole / HBM_PEAK_GBS, 4)}}

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

    bucket = (flat, off, ws, fit, rate)
    if args.only == "none":
        want = ()
    elif args.only:
        want = tuple(w for w in args.only.split(",") if w)
        unknown = [w for w in want if w not in CONFIG_NAMES]
        if unknown:
            print("bench.py: unknown configuration(s) %s; known: %s" % (unknown, ", ".join(CONFIG_NAMES)), file=sys.stderr)
            sys.exit(2)
    else:
        want = CONFIG_NAMES
    configs = other_configs(gg, gg_inputs, torch, dev, args, timer, bucket, want) if want else {}
    c5 = configs.pop("_c5_sample", None)
    if configs:
        out["configs"] = configs
    if args.extra:
        out["extra"] = companions(gg, torch, dev, args, timer, bucket, frec, np)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_leg(args, np, gg, gg_inputs, torch, bucket, frec, c5)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
