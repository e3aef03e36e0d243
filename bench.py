"""Benchmark of the HiF8 conversion hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extra] [--no-cpu]

Headline (the one JSON line on stdout): config 2 of the baseline, the dynamic-range sweep --
67,108,864 FP32 values encoded to u8 HiF8 codes, scale = 1, rounding half away from zero.
One step = one hif8_encode_f32 pass over one such tensor; steps rotate over several
distinct resident tensors so that no pass is served from the 256 MB last-level cache.
value = algorithmic bytes (4 B read + 1 B written per element) * steps / wall time.

The same line carries
  roofline      algorithmic bytes per launch / average launch duration (HIP events on the
                launch stream over the timed region) against the 8 TB/s HBM peak;
  cpu_baseline  the CPU oracle (oracle/, untouched) timed on the host cores on the same input;
  extra         the other rows of the hot path (amax, decode, fused fake-quant pipeline,
                gradient tensor TA / HR, LLM weight cast, same-mix stream ceiling).
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Timing:
    """Per-step times of one timed region: wall clock, HIP events over the whole region (mean), and the
    median / min / max over the batches the region was cut into by intermediate events."""

    def __init__(self, wall_ms, ms, batch_ms):
        self.wall_ms, self.ms = wall_ms, ms
        b = sorted(batch_ms)
        self.median_ms = b[len(b) // 2] if len(b) % 2 else 0.5 * (b[len(b) // 2 - 1] + b[len(b) // 2])
        self.min_ms, self.max_ms = b[0], b[-1]


def timed(fn, steps, warmup, batches=10):
    """Runs fn(i) warmup + steps times back to back on the current stream.  Events are recorded before the first
    step, after the last, and between batches of steps (about `batches` of them), never inside a batch."""
    import torch
    for i in range(warmup):
        fn(i)
    nb = max(1, min(batches, steps))
    bounds = [round(k * steps / nb) for k in range(nb + 1)]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(nb + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for k in range(nb):
        for i in range(bounds[k], bounds[k + 1]):
            fn(i)
        ev[k + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per_batch = [ev[k].elapsed_time(ev[k + 1]) / (bounds[k + 1] - bounds[k]) for k in range(nb)]
    return Timing((t1 - t0) * 1e3 / steps, ev[0].elapsed_time(ev[nb]) / steps, per_batch)


def rate(bytes_per_step, tm):
    gbs = bytes_per_step / (tm.ms * 1e-3) / 1e9
    return {"ms": round(tm.ms, 5), "median_ms": round(tm.median_ms, 5), "min_ms": round(tm.min_ms, 5),
            "max_ms": round(tm.max_ms, 5), "GB/s": round(gbs, 1), "frac_of_8TBs": round(gbs / HBM_PEAK_GBS, 4)}


def kernel_source_digest():
    """Digest of the sources the conversion kernels are built from; a profile summary that records it is
    known to describe the kernels of this tree."""
    import hashlib
    h = hashlib.sha256()
    for f in ("hif8_conv.hpp", "hif8_stream.hpp", "hif8_device.hpp", "hif8_lib.hip"):
        h.update(open(os.path.join(ROOT, "paper_2409_16626_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=300,
                    help="untimed launches first; the launch duration settles only after ~150 back-to-back launches")
    ap.add_argument("--no-extra", action="store_true", help="skip the secondary workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--buffers", type=int, default=6, help="distinct resident input tensors to rotate over")
    ap.add_argument("--pmc", action="store_true",
                    help="counter-collection mode for rocprofv3 --pmc: 5 plain 16-byte copies of a known "
                         "size, then 5 headline encode launches; no timing, no JSON")
    ap.add_argument("--pmc-modes", action="store_true",
                    help="counter-collection mode for rocprofv3 --pmc: 5 encode launches per rounding method, on the "
                         "C2 tensor (binary32) and on the C3 tensor (BF16); no timing, no JSON")
    ap.add_argument("--rows", action="store_true",
                    help="profiling mode for rocprofv3 (kernel trace or --pmc): 10 launches of every conversion kernel of the "
                         "hot path (amax, decode, fake-quant, per-tensor scaling in one call, multi-tensor casts) after 10 "
                         "plain copies of a known size; no timing, no JSON")
    ap.add_argument("--gemm-only", action="store_true",
                    help="profiling mode: only the simulated HiF8 GEMM rows (25 launches of 8192^3), no headline")
    ap.add_argument("--sweep-only", action="store_true",
                    help="profiling mode: only the 10-scale sweep over the C3 tensor (25 launches), no headline")
    ap.add_argument("--per-channel-only", action="store_true",
                    help="profiling mode: only the per-channel casts of a [11008, 4096] BF16 matrix (25 rounds), no headline")
    ap.add_argument("--tune", type=str, default="", help="block,wg_per_cu,unroll,ta_impl,tiles_per_wg,amax_nt (prefix allowed)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus %d is not supported "
                 "(no collectives, sharding or rank code exist here)" % args.gpus)

    import numpy as np
    import torch
    from paper_2409_16626_amd import hif8, workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    hif8.hif8_init()
    if args.tune:
        for k, v in enumerate(int(t) for t in args.tune.split(",")):
            hif8.hif8_set_tuning(k, v)
    tune = [hif8.hif8_get_tuning(k) for k in range(hif8.N_TUNE_KEYS)]

    def gemm_operands(gm, gn, gk):
        ws = torch.zeros(hif8.hif8_quantize_workspace_bytes(), dtype=torch.uint8, device=dev)
        am = torch.zeros(2, dtype=torch.float32, device=dev)
        sc = torch.zeros(2, 2, dtype=torch.float32, device=dev)
        act = workloads.activation_bf16(gm, gk, dev)
        wgt = (workloads.normal_f32(gn * gk, dev) * 0.02).to(torch.bfloat16)
        ca = torch.empty(gm, gk, dtype=torch.uint8, device=dev)
        cb = torch.empty(gn, gk, dtype=torch.uint8, device=dev)
        hif8.hif8_quantize_tensor_bf16(act, None, ca, gm * gk, am[0:1], sc[0], ws, hif8.MAX_FINITE, 1, hif8.RM_TA)
        hif8.hif8_quantize_tensor_bf16(wgt, None, cb, gn * gk, am[1:2], sc[1], ws, hif8.MAX_FINITE, 1, hif8.RM_TA)
        torch.cuda.synchronize()
        return ca, cb

    if args.gemm_only:
        gm = gn = gk = 8192
        ca, cb = gemm_operands(gm, gn, gk)
        go = torch.empty(gm, gn, dtype=torch.bfloat16, device=dev)
        tm = timed(lambda i: hif8.hif8_gemm_bf16(ca, cb, go, gm, gn, gk, 1.0, 1.0), 20, 5)
        fl = 2.0 * gm * gn * gk
        res = {"gemm_bf16 M=N=K=8192": {"ms": round(tm.ms, 4), "TFLOP/s": round(fl / (tm.ms * 1e-3) / 1e12, 1),
                                        "frac_of_2.5PFLOPs_bf16": round(fl / (tm.ms * 1e-3) / 2.5e15, 4)}}
        ld = hif8.hif8_expanded_ld(gk)
        xa = torch.empty(gm, ld, dtype=torch.bfloat16, device=dev)
        xb = torch.empty(gn, ld, dtype=torch.bfloat16, device=dev)
        hif8.hif8_expand_bf16(ca, gm, gk, xa, ld)
        hif8.hif8_expand_bf16(cb, gn, gk, xb, ld)
        tm = timed(lambda i: hif8.hif8_gemm_expanded_bf16(xa, xb, go, gm, gn, gk, ld, 1.0, 1.0), 20, 5)
        res["gemm_expanded_bf16 M=N=K=8192"] = {"ms": round(tm.ms, 4), "TFLOP/s": round(fl / (tm.ms * 1e-3) / 1e12, 1),
                                                "frac_of_2.5PFLOPs_bf16": round(fl / (tm.ms * 1e-3) / 2.5e15, 4)}
        tm = timed(lambda i: torch.matmul(xa, xb.t(), out=go), 20, 5)   # comparison: the vendor library on the same operands
        res["comparison: torch.matmul bf16 M=N=K=8192"] = {"ms": round(tm.ms, 4), "TFLOP/s": round(fl / (tm.ms * 1e-3) / 1e12, 1),
                                                           "frac_of_2.5PFLOPs_bf16": round(fl / (tm.ms * 1e-3) / 2.5e15, 4)}
        print(json.dumps(res), flush=True)
        return

    if args.per_channel_only:
        rows_c, cols_c, Rw = 11008, 4096, 3
        g = torch.Generator(device=dev).manual_seed(11008)
        wm = [(torch.randn(rows_c, cols_c, generator=g, device=dev) * 0.02).to(torch.bfloat16) for _ in range(Rw)]   # 270 MB: more than the last-level cache
        cd = torch.empty(rows_c, cols_c, dtype=torch.uint8, device=dev)
        out = {}
        for axis in (0, 1):
            nch = rows_c if axis == 0 else cols_c
            am_c = torch.zeros(nch, dtype=torch.float32, device=dev)
            sc_c = torch.zeros(nch, 2, dtype=torch.float32, device=dev)

            def three(i):
                hif8.hif8_amax_axis_bf16(wm[i % Rw], rows_c, cols_c, axis, am_c)
                hif8.hif8_scale_from_amax_n(am_c, sc_c, nch, hif8.MAX_FINITE, 1)
                hif8.hif8_encode_axis_bf16(wm[i % Rw], cd, rows_c, cols_c, axis, sc_c, hif8.RM_TA)

            tm = timed(three, 20, 5)
            out["axis %d, three launches" % axis] = round(tm.ms * 1e3, 2)
        am_r = torch.zeros(rows_c, dtype=torch.float32, device=dev)
        sc_r = torch.zeros(rows_c, 2, dtype=torch.float32, device=dev)
        tm = timed(lambda i: hif8.hif8_quantize_rows_bf16(wm[i % Rw], cd, rows_c, cols_c, am_r, sc_r, hif8.MAX_FINITE, 1,
                                                                  hif8.RM_TA), 20, 5)
        out["rows in one pass (hif8_quantize_rows_bf16)"] = round(tm.ms * 1e3, 2)
        print(json.dumps({"per-channel casts of a [11008, 4096] BF16 matrix, us per call sequence": out}), flush=True)
        return

    if args.sweep_only:
        a0 = workloads.activation_bf16(8192, 8192, dev).view(-1)
        errs = torch.zeros(16, dtype=torch.float64, device=dev)
        tm = timed(lambda i: hif8.hif8_scale_sweep_bf16(a0, a0.numel(), -4, 10, hif8.RM_TA, errs), 20, 5)
        print(json.dumps({"scale_sweep_bf16 2^26 elements x 10 scales": {
            "ms": round(tm.ms, 5), "casts_per_s": round(10 * a0.numel() / (tm.ms * 1e-3), 0),
            "mse_per_scale": [round(v / a0.numel(), 8) for v in errs[:10].cpu().tolist()]}}), flush=True)
        return

    # ---------------- headline: C2 encode_f32, TA, scale 1 ----------------
    n = 1 << 26
    x0 = workloads.dynamic_range_sweep(n, dev)
    xs = [x0] + [torch.roll(x0, 1009 * (i + 1)) for i in range(args.buffers - 1)]
    outs = [torch.empty(n, dtype=torch.uint8, device=dev) for _ in range(args.buffers)]
    R = args.buffers

    def step(i):
        hif8.hif8_encode_f32(xs[i % R], outs[i % R], n, 1.0, hif8.RM_TA)

    if args.pmc:
        # reference dispatches with known traffic: copy n*4 bytes in, n*4 bytes out
        cp = torch.empty(n, dtype=torch.float32, device=dev)
        for i in range(5):
            hif8.hif8_diag_stream(xs[i % R], cp, n // 4, 16)
        for i in range(5):
            step(i)
        torch.cuda.synchronize()
        log("pmc mode: 5 x k_diag_stream<.,16> (%d B read, %d B written each), 5 x k_encode_f32" % (4 * n, 4 * n))
        return

    if args.pmc_modes:
        from paper_2409_16626_amd import workloads as wl
        act = wl.activation_bf16(8192, 8192, dev).view(-1)
        m = act.numel()
        cd = torch.empty(m, dtype=torch.uint8, device=dev)
        for name in ("TA", "HR", "TE", "SSR", "SR"):
            mode = getattr(hif8, "RM_" + name)
            for i in range(5):
                hif8.hif8_encode_f32(xs[i % R], outs[i % R], n, 1.0, mode)
            for i in range(5):
                hif8.hif8_encode_bf16(act, cd, m, 91.0, mode)
        torch.cuda.synchronize()
        log("pmc-modes: 5 x hif8_encode_f32 (%d elements) and 5 x hif8_encode_bf16 (%d elements) per rounding method "
            "TA, HR, TE, SSR, SR" % (n, m))
        return

    if args.rows:
        reps = 10
        cp = torch.empty(n, dtype=torch.float32, device=dev)
        for i in range(reps):    # calibration: 268,435,456 B read and written per launch
            hif8.hif8_diag_stream(xs[i % R], cp, n // 4, 16)
        del cp
        am = torch.zeros(1, dtype=torch.float32, device=dev)
        sc = torch.tensor([4.0, 0.25], dtype=torch.float32, device=dev)
        for i in range(reps):
            hif8.hif8_amax_f32(xs[i % R], n, am)
        for i in range(reps):
            step(i)
        dec = torch.empty(n, dtype=torch.float32, device=dev)
        for i in range(reps):
            hif8.hif8_decode_f32(outs[i % R], dec, n, 1.0)
        for i in range(reps):
            hif8.hif8_fake_quant_f32(xs[i % R], dec, outs[i % R], n, 1.0, hif8.RM_TA)
        del dec
        log('rows: C2 kernels enqueued')
        a0 = workloads.activation_bf16(8192, 8192, dev).view(-1)
        m = a0.numel()
        acts = [a0] + [torch.roll(a0, 4099 * (i + 1)) for i in range(R - 1)]
        fq = [torch.empty_like(a0) for _ in range(2)]
        cds = [torch.empty(m, dtype=torch.uint8, device=dev) for _ in range(2)]
        qws = torch.empty(hif8.hif8_quantize_workspace_bytes(), dtype=torch.uint8, device=dev)
        for i in range(reps):
            hif8.hif8_amax_bf16(acts[i % R], m, am)
        for i in range(reps):
            hif8.hif8_encode_bf16_ds(acts[i % R], cds[i % 2], m, sc, hif8.RM_TA)
        for i in range(reps):
            hif8.hif8_decode_bf16(cds[i % 2], fq[i % 2], m, 4.0)
        for i in range(reps):
            hif8.hif8_fake_quant_bf16_ds(acts[i % R], fq[i % 2], cds[i % 2], m, sc, hif8.RM_TA)
        for i in range(reps):
            hif8.hif8_fake_quant_bf16_ds(acts[i % R], fq[i % 2], None, m, sc, hif8.RM_TA)
        acc = torch.zeros(1, dtype=torch.float32, device=dev)
        for i in range(reps):
            hif8.hif8_fake_quant_bf16_ds(acts[i % R], fq[i % 2], cds[i % 2], m, sc, hif8.RM_TA, d_amax_accum=acc)
        for i in range(reps):   # the C3 recipe as one call: k_amax<.., partial maxima> then k_fake_quant
            hif8.hif8_quantize_tensor_bf16(acts[i % R], fq[i % 2], cds[i % 2], m, am, sc, qws, hif8.MAX_FINITE, 0, hif8.RM_TA)
        del acts, fq, cds, a0
        torch.cuda.empty_cache()
        # multi-tensor casts on the first two decoder layers of C5 (14 tensors + a small one, 0.75 GiB of BF16)
        log('rows: single-tensor kernels enqueued')
        arena, index = workloads.llm_weights_bf16(dev, layers=2, vocab=16)
        wc = torch.empty(arena.numel(), dtype=torch.uint8, device=dev)
        items = [(arena.data_ptr() + 2 * off, wc.data_ptr() + off, cnt) for _, off, cnt in index]
        plan = hif8.hif8_multi_plan(items, src_is_16bit=True)
        ams = torch.zeros(plan.count, dtype=torch.float32, device=dev)
        scs = torch.zeros(plan.count, 2, dtype=torch.float32, device=dev)
        for i in range(reps):
            hif8.hif8_multi_cast_bf16(plan.d_items, plan.count, plan.total_tiles, ams, scs, hif8.MAX_FINITE, 0, hif8.RM_TA)
        for i in range(reps):
            hif8.hif8_multi_encode_bf16_ds(plan.d_items, plan.count, plan.total_tiles, scs, hif8.RM_TA)
        for i in range(reps):
            hif8.hif8_multi_encode_bf16_ds(plan.d_items, plan.count, plan.total_tiles, scs, hif8.RM_TA, d_amax_accum=ams)
        for i in range(reps):
            hif8.hif8_multi_cast_bf16(plan.d_items, plan.count, plan.total_tiles, ams, scs, hif8.MAX_FINITE, 0, hif8.RM_TA,
                                      host_items=plan.host_items)
        torch.cuda.synchronize()
        log("rows mode: %d launches each; C2 tensor %d FP32, C3 tensor %d BF16, multi-tensor list %d tensors / %d BF16 elements"
            % (reps, n, m, plan.count, arena.numel()))
        return

    tm0 = timed(step, args.steps, args.warmup)
    wall_ms, ev_ms = tm0.wall_ms, tm0.ms
    bytes_step = 5 * n
    value = bytes_step / (wall_ms * 1e-3) / 1e9
    achieved = bytes_step / (ev_ms * 1e-3) / 1e9
    log("C2 encode_f32 TA: wall %.4f ms/step, events %.4f ms/launch (median %.4f, min %.4f, max %.4f over batches), %.1f GB/s"
        % (wall_ms, ev_ms, tm0.median_ms, tm0.min_ms, tm0.max_ms, achieved))

    # HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE, calibrated against a plain copy): taken
    # from the committed summary only if that summary was made from the kernel sources of this tree
    traffic, traffic_note = None, "no counter summary for this kernel source"
    prof = os.path.join(ROOT, "profiles", "encode_f32_ta_c2_pmc.md")
    if os.path.exists(prof):
        fields = dict(l.strip().split(":", 1) for l in open(prof) if re.match(r"^[a-z_]+:", l))
        if fields.get("kernel_source_digest", "").strip() == kernel_source_digest():
            traffic = int(fields["traffic_bytes_per_launch"])
            traffic_note = "profiles/encode_f32_ta_c2_pmc.md (rocprofv3 --pmc on this kernel source, digest %s)" % kernel_source_digest()
        else:
            traffic_note = "profiles/encode_f32_ta_c2_pmc.md describes another kernel source (digest %s, this tree %s)" % (
                fields.get("kernel_source_digest", "?").strip(), kernel_source_digest())
    result = {
        "metric": "HiF8 encode GB/s (FP32 -> u8 codes, TA, algorithmic 5 B/element) on 1 MI355X",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": "C2 dynamic-range sweep: 67,108,864 FP32 = +-2^E (1 + m), E uniform in -30..19, 1% exact rounding ties, "
                               "hif8_encode_f32, scale=1, rounding half away from zero",
                   "elements": n, "elements_per_s": round(n / (wall_ms * 1e-3), 0),
                   "rotating_buffers": R, "tuning_knobs": tune},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_note,
                     "kernel": "k_encode<U, TA table, binary32 source>", "bytes_per_launch": bytes_step,
                     "avg_launch_ms": round(ev_ms, 5), "median_launch_ms": round(tm0.median_ms, 5),
                     "min_launch_ms": round(tm0.min_ms, 5), "max_launch_ms": round(tm0.max_ms, 5)},
    }

    # ---------------- CPU oracle baseline on the same inputs ----------------
    if not args.no_cpu:
        from oracle import hif8_oracle as orc

        def time_oracle(fn, min_s=1.0, min_passes=3):
            passes, dt, res = 0, 0.0, None
            while dt < min_s or passes < min_passes:
                t0 = time.perf_counter()
                res = fn()
                dt += time.perf_counter() - t0
                passes += 1
            return passes, dt, res

        sample = x0.cpu().numpy()
        orc.encode_f32(sample[:1 << 20], 1.0, orc.RM_TA)  # warm up threads / table
        passes, dt, want = time_oracle(lambda: orc.encode_f32(sample, 1.0, orc.RM_TA))   # ~1 s on every host core
        hif8.hif8_encode_f32(xs[0], outs[0], n, 1.0, hif8.RM_TA)
        torch.cuda.synchronize()
        mism = int(np.count_nonzero(outs[0].cpu().numpy() != want))
        result["cpu_baseline"] = {"value": round(5 * n * passes / dt / 1e9, 3), "unit": "GB/s", "cores": orc.threads_used(),
                                  "kind": "oracle",
                                  "sample": "the whole C2 tensor (67,108,864 elements) x %d passes, %.2f s wall, "
                                            "%.0f core-seconds" % (passes, dt, dt * orc.threads_used()),
                                  "elements_per_s": round(n * passes / dt, 0), "gpu_vs_oracle_mismatches": mism}
        log("oracle: %d passes in %.2f s on %d threads; mismatches vs GPU: %d" % (passes, dt, orc.threads_used(), mism))
        del sample, want
        if not args.no_extra:
            # the oracle on the other configurations: C3 whole, C4 and C5 on their first 2^26 elements
            others = {}
            a_host = workloads.activation_bf16(8192, 8192, dev).view(-1).view(torch.int16).cpu().numpy().view(np.uint16)

            def c3_oracle():
                am_ = orc.amax_bf16(a_host)
                return orc.fake_quant_bf16(a_host, orc.scale_from_amax(am_, 32768.0, False), orc.RM_TA)

            p_, d_, _ = time_oracle(c3_oracle, 0.5, 2)
            others["C3 amax + scale + fake_quant_bf16, whole tensor (2^26 BF16), 5 B/elem"] = {
                "GB/s": round(5 * a_host.size * p_ / d_ / 1e9, 3), "elements_per_s": round(a_host.size * p_ / d_, 0)}
            del a_host
            g_host = workloads.gradient_f32(1 << 26, dev).cpu().numpy()
            for name, mode in (("TA", orc.RM_TA), ("HR", orc.RM_HR)):
                p_, d_, _ = time_oracle(lambda: orc.encode_f32(g_host, 1.0, mode), 0.5, 2)
                others["C4 encode_f32 %s, first 2^26 of 2^30 elements (rate extrapolates: element-wise), 5 B/elem" % name] = {
                    "GB/s": round(5 * g_host.size * p_ / d_ / 1e9, 3), "elements_per_s": round(g_host.size * p_ / d_, 0)}
            del g_host
            w_host = (workloads._normal_f32(5, 0, torch.arange(1 << 26, dtype=torch.int64, device=dev)) * 0.02).to(torch.bfloat16) \
                .view(torch.int16).cpu().numpy().view(np.uint16)

            def c5_oracle():
                am_ = orc.amax_bf16(w_host)
                return orc.encode_bf16(w_host, orc.scale_from_amax(am_, 32768.0, False), orc.RM_TA)

            p_, d_, _ = time_oracle(c5_oracle, 0.5, 2)
            others["C5 amax + scale + encode_bf16, first 2^26 of 6.6e9 elements, 3 B/elem"] = {
                "GB/s": round(3 * w_host.size * p_ / d_ / 1e9, 3), "elements_per_s": round(w_host.size * p_ / d_, 0)}
            del w_host
            result["cpu_baseline"]["other_configs"] = others

    # ---------------- the other rows of the hot path ----------------
    if not args.no_extra:
        extra = {}
        K, W = max(20, args.steps // 3), max(5, args.warmup // 3)

        # plain copy kernels with the byte mix of a conversion, launched with the shape of the kernel they are compared
        # with (same-mix copies, not upper bounds: a conversion kernel with a better launch shape can beat them)
        hif8.hif8_set_tuning(hif8.TUNE_FAMILY, hif8.FAM_DIAG)
        for k_, v_ in ((hif8.TUNE_BLOCK, 256), (hif8.TUNE_UNROLL, 4), (hif8.TUNE_TILES_PER_WG, 1)):
            hif8.hif8_set_tuning(k_, v_)
        tm = timed(lambda i: hif8.hif8_diag_stream(xs[i % R], outs[i % R], n // 4, 4), K, W)
        extra["same-mix copy, read 16 B write 4 B per lane (shape of the FP32 TA encode)"] = rate(5 * n, tm)
        for k_, v_ in ((hif8.TUNE_BLOCK, 1024), (hif8.TUNE_UNROLL, 2), (hif8.TUNE_TILES_PER_WG, 0), (hif8.TUNE_WG_PER_CU, 1)):
            hif8.hif8_set_tuning(k_, v_)
        tm = timed(lambda i: hif8.hif8_diag_stream(xs[i % R], None, n // 4, 0), K, W)
        extra["read-only stream, 16 B per lane, 2^26 FP32 (shape of amax)"] = rate(4 * n, tm)
        for k_ in (hif8.TUNE_BLOCK, hif8.TUNE_UNROLL, hif8.TUNE_TILES_PER_WG, hif8.TUNE_WG_PER_CU, hif8.TUNE_FAMILY):
            hif8.hif8_set_tuning(k_, -1)

        # amax FP32 (read only)
        am = torch.zeros(1, dtype=torch.float32, device=dev)
        tm = timed(lambda i: hif8.hif8_amax_f32(xs[i % R], n, am), K, W)
        extra["amax_f32 C2 (4 B/elem)"] = rate(4 * n, tm)

        # decode to FP32 (1 B in, 4 B out)
        dec = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(2)]
        tm = timed(lambda i: hif8.hif8_decode_f32(outs[i % R], dec[i % 2], n, 1.0), K, W)
        extra["decode_f32 C2 codes (5 B/elem)"] = rate(5 * n, tm)
        del dec

        # HR on the C2 tensor
        tm = timed(lambda i: hif8.hif8_encode_f32(xs[i % R], outs[i % R], n, 1.0, hif8.RM_HR), K, W)
        extra["encode_f32 HR C2 (5 B/elem)"] = rate(5 * n, tm)

        # comparison modes on the C2 tensor: TE (tie table), simplified SR everywhere, standard SR
        for name, mode in (("TE", hif8.RM_TE), ("SSR", hif8.RM_SSR), ("SR", hif8.RM_SR)):
            tm = timed(lambda i: hif8.hif8_encode_f32(xs[i % R], outs[i % R], n, 1.0, mode), K, W)
            extra["encode_f32 %s C2 (5 B/elem, comparison mode)" % name] = rate(5 * n, tm)
        del xs, outs, x0
        torch.cuda.empty_cache()

        # C3: BF16 activation, amax -> scale -> fused fake-quant with codes
        a0 = workloads.activation_bf16(8192, 8192, dev).view(-1)
        m = a0.numel()
        acts = [a0] + [torch.roll(a0, 4099 * (i + 1)) for i in range(R - 1)]
        fq = [torch.empty_like(a0) for _ in range(R)]
        cds = [torch.empty(m, dtype=torch.uint8, device=dev) for _ in range(R)]
        sc = torch.zeros(2, dtype=torch.float32, device=dev)

        def c3(i):
            j = i % R
            hif8.hif8_amax_bf16(acts[j], m, am)
            hif8.hif8_scale_from_amax(am, sc, hif8.MAX_FINITE, 0)
            hif8.hif8_fake_quant_bf16_ds(acts[j], fq[j], cds[j], m, sc, hif8.RM_TA)

        tm = timed(c3, K, W)
        extra["C3 amax+scale+fake_quant_bf16 (5 B/elem primary)"] = rate(5 * m, tm)
        extra["C3 amax+scale+fake_quant_bf16 (7 B/elem with amax pass)"] = rate(7 * m, tm)
        qws = torch.empty(hif8.hif8_quantize_workspace_bytes(), dtype=torch.uint8, device=dev)
        tm = timed(lambda i: hif8.hif8_quantize_tensor_bf16(acts[i % R], fq[i % R], cds[i % R], m, am, sc, qws,
                                                                    hif8.MAX_FINITE, 0, hif8.RM_TA), K, W)
        extra["C3 hif8_quantize_tensor_bf16: amax+scale+fake_quant in one call, 2 launches (5 B/elem primary)"] = rate(5 * m, tm)
        extra["C3 hif8_quantize_tensor_bf16 (7 B/elem with amax pass)"] = rate(7 * m, tm)
        tm = timed(lambda i: hif8.hif8_fake_quant_bf16_ds(acts[i % R], fq[i % R], cds[i % R], m, sc, hif8.RM_TA), K, W)
        extra["fake_quant_bf16 alone (5 B/elem)"] = rate(5 * m, tm)
        # the paper's delayed scaling (Sec. 5): the cast uses the scale on the device and accumulates the amax
        # of its input for the next update in the same pass -- C3 in one pass over the tensor
        acc = torch.zeros(1, dtype=torch.float32, device=dev)
        tm = timed(lambda i: hif8.hif8_fake_quant_bf16_ds(acts[i % R], fq[i % R], cds[i % R], m, sc, hif8.RM_TA,
                                                                  d_amax_accum=acc), K, W)
        extra["C3 with delayed scaling: fake_quant_bf16_ds + amax accumulated in the same pass (5 B/elem)"] = rate(5 * m, tm)
        tm = timed(lambda i: hif8.hif8_amax_bf16(acts[i % R], m, am), K, W)
        extra["amax_bf16 (2 B/elem)"] = rate(2 * m, tm)
        tm = timed(lambda i: hif8.hif8_encode_bf16_ds(acts[i % R], cds[i % R], m, sc, hif8.RM_TA), K, W)
        extra["encode_bf16 (3 B/elem)"] = rate(3 * m, tm)
        tm = timed(lambda i: hif8.hif8_encode_bf16_ds(acts[i % R], cds[i % R], m, sc, hif8.RM_HR), K, W)
        extra["encode_bf16 HR (3 B/elem)"] = rate(3 * m, tm)
        tm = timed(lambda i: hif8.hif8_encode_bf16_ds(acts[i % R], cds[i % R], m, sc, hif8.RM_SR), K, W)
        extra["encode_bf16 SR (3 B/elem, comparison mode)"] = rate(3 * m, tm)
        h16 = [a.float().to(torch.float16) for a in acts[:2]]
        tm = timed(lambda i: hif8.hif8_encode_f16(h16[i % 2], cds[i % R], m, 1.0, hif8.RM_TA), K, W)
        extra["encode_f16 (3 B/elem)"] = rate(3 * m, tm)
        tm = timed(lambda i: hif8.hif8_fake_quant_f16(h16[i % 2], fq[i % R], cds[i % R], m, 1.0, hif8.RM_HR), K, W)
        extra["fake_quant_f16 HR with codes (5 B/elem)"] = rate(5 * m, tm)
        del h16
        hif8.hif8_set_tuning(hif8.TUNE_FAMILY, hif8.FAM_DIAG)
        for k_, v_ in ((hif8.TUNE_BLOCK, 512), (hif8.TUNE_UNROLL, 2), (hif8.TUNE_TILES_PER_WG, 2)):
            hif8.hif8_set_tuning(k_, v_)
        tm = timed(lambda i: hif8.hif8_diag_stream(acts[i % R], cds[i % R], m // 8, 8), K, W)
        extra["same-mix copy, read 16 B write 8 B per lane (shape of the BF16 encode)"] = rate(3 * m, tm)
        for k_ in (hif8.TUNE_BLOCK, hif8.TUNE_UNROLL, hif8.TUNE_TILES_PER_WG, hif8.TUNE_FAMILY):
            hif8.hif8_set_tuning(k_, -1)
        # calibration-side rows: scale sweep (10 power-of-two scales in one pass), per-channel cast
        errs = torch.zeros(16, dtype=torch.float64, device=dev)
        tm = timed(lambda i: hif8.hif8_scale_sweep_bf16(acts[i % R], m, -4, 10, hif8.RM_TA, errs), K, W)
        # per element and scale: multiply, two shifts, 16-bit value-table read, shift, multiply, conversion to
        # fp64, fp64 subtract, fp64 fma: 8.5 vector instructions per cast by SQ_INSTS_VALU.  The rate can pass the
        # 39.3 T lane-ops/s of one instruction per SIMD every four cycles: v_fma_f64 partly overlaps with other
        # vector instructions on this chip (a probe mixing it with integer and fp32 instructions issues 44 T/s,
        # any single kind 38 T/s), and it is one instruction in eight here.
        ops = 8.5 * 10 * m
        extra["scale_sweep_bf16 C3 tensor, 10 scales"] = {
            "ms": round(tm.ms, 5), "elements_per_s": round(m / (tm.ms * 1e-3), 0), "casts_per_s": round(10 * m / (tm.ms * 1e-3), 0),
            "bound": "alu", "lane_ops_per_s": round(ops / (tm.ms * 1e-3), 0), "frac_of_39.3T_lane_ops": round(ops / (tm.ms * 1e-3) / 39.3e12, 4),
            "note": "above 1 where v_fma_f64 overlaps with the other vector instructions"}
        rows_c, cols_c = 11008, 4096
        wmats = [a[:rows_c * cols_c] for a in acts]   # rotate the source as well: one 90 MB matrix would sit in the last-level cache
        for axis in (0, 1):
            nch = rows_c if axis == 0 else cols_c
            am_c = torch.zeros(nch, dtype=torch.float32, device=dev)
            sc_c = torch.zeros(nch, 2, dtype=torch.float32, device=dev)

            def per_channel(i):
                hif8.hif8_amax_axis_bf16(wmats[i % R], rows_c, cols_c, axis, am_c)
                hif8.hif8_scale_from_amax_n(am_c, sc_c, nch, hif8.MAX_FINITE, 1)
                hif8.hif8_encode_axis_bf16(wmats[i % R], cds[i % R], rows_c, cols_c, axis, sc_c, hif8.RM_TA)

            tm = timed(per_channel, K, W)
            extra["per-channel amax+scale+encode_bf16 [11008,4096] axis %d (5 B/elem with amax pass)" % axis] = rate(5 * rows_c * cols_c, tm)
        am_r = torch.zeros(rows_c, dtype=torch.float32, device=dev)
        sc_r = torch.zeros(rows_c, 2, dtype=torch.float32, device=dev)
        tm = timed(lambda i: hif8.hif8_quantize_rows_bf16(wmats[i % R], cds[i % R], rows_c, cols_c, am_r, sc_r,
                                                                  hif8.MAX_FINITE, 1, hif8.RM_TA), K, W)
        extra["per-row amax+scale+encode_bf16 [11008,4096] in one pass, hif8_quantize_rows (3 B/elem)"] = rate(3 * rows_c * cols_c, tm)
        del acts, fq, cds, a0, wmats
        torch.cuda.empty_cache()

        # simulated HiF8 GEMM on the matrix cores (code operands expanded in the kernel; operands expanded beforehand),
        # and Algorithm 1 for one layer
        MFMA_PEAK = 2.5e15
        for (gm, gn, gk) in ((8192, 8192, 8192), (8192, 11008, 4096)):
            # operands as a training step has them: the per-tensor-scaled HiF8 cast of an activation tensor with
            # outliers (the C3 recipe) and of N(0, 0.02) weights (the C5 recipe); the matrix-core clock under
            # load, and with it the rate, follows the operand values
            ca, cb = gemm_operands(gm, gn, gk)
            go = torch.empty(gm, gn, dtype=torch.bfloat16, device=dev)
            tm = timed(lambda i: hif8.hif8_gemm_bf16(ca, cb, go, gm, gn, gk, 1.0, 1.0), 20, 5)
            fl = 2.0 * gm * gn * gk
            extra["gemm_bf16 out, HiF8 operands, M=%d N=%d K=%d" % (gm, gn, gk)] = {
                "ms": round(tm.ms, 4), "TFLOP/s": round(fl / (tm.ms * 1e-3) / 1e12, 1), "bound": "mfma",
                "frac_of_2.5PFLOPs_bf16": round(fl / (tm.ms * 1e-3) / MFMA_PEAK, 4)}
            # code operands through a workspace: both expansions and the expanded-operand kernel in one call
            wsg = torch.empty(hif8.hif8_gemm_workspace_bytes(gm, gn, gk), dtype=torch.uint8, device=dev)
            tm = timed(lambda i: hif8.hif8_gemm_ws_bf16(ca, cb, go, gm, gn, gk, wsg, 1.0, 1.0), 20, 5)
            extra["gemm_ws_bf16 out, HiF8 operands expanded into a workspace, M=%d N=%d K=%d" % (gm, gn, gk)] = {
                "ms": round(tm.ms, 4), "TFLOP/s": round(fl / (tm.ms * 1e-3) / 1e12, 1), "bound": "mfma",
                "frac_of_2.5PFLOPs_bf16": round(fl / (tm.ms * 1e-3) / MFMA_PEAK, 4)}
            del wsg
            # the same product on operands expanded to bfloat16 once (expansion timed separately, and together)
            ld = hif8.hif8_expanded_ld(gk)
            xa = torch.empty(gm, ld, dtype=torch.bfloat16, device=dev)
            xb = torch.empty(gn, ld, dtype=torch.bfloat16, device=dev)

            def expand_both(i):
                hif8.hif8_expand_bf16(ca, gm, gk, xa, ld)
                hif8.hif8_expand_bf16(cb, gn, gk, xb, ld)

            tmx = timed(expand_both, 20, 5)
            ldt = hif8.hif8_expanded_ld(gn)
            xt = torch.empty(gk, ldt, dtype=torch.bfloat16, device=dev)
            tmt = timed(lambda i: hif8.hif8_expand_bf16_t(cb, gn, gk, xt, ldt), 20, 5)
            del xt
            tm = timed(lambda i: hif8.hif8_gemm_expanded_bf16(xa, xb, go, gm, gn, gk, ld, 1.0, 1.0), 20, 5)
            extra["gemm_expanded_bf16 out, operands expanded to bf16 beforehand, M=%d N=%d K=%d" % (gm, gn, gk)] = {
                "ms": round(tm.ms, 4), "TFLOP/s": round(fl / (tm.ms * 1e-3) / 1e12, 1), "bound": "mfma",
                "frac_of_2.5PFLOPs_bf16": round(fl / (tm.ms * 1e-3) / MFMA_PEAK, 4),
                "expand_both_operands_ms": round(tmx.ms, 4), "expand_GB/s (3 B/elem)": round(3.0 * (gm + gn) * gk / (tmx.ms * 1e-3) / 1e9, 1),
                "TFLOP/s incl. expansion": round(fl / ((tm.ms + tmx.ms) * 1e-3) / 1e12, 1),
                "transposing_expand_of_B_ms": round(tmt.ms, 4), "transposing_expand_GB/s (3 B/elem)": round(3.0 * gn * gk / (tmt.ms * 1e-3) / 1e9, 1)}
            # comparison, not part of the path: the vendor library's bf16 GEMM (torch.matmul) on the same expanded operands
            tmv = timed(lambda i: torch.matmul(xa, xb.t(), out=go), 20, 5)
            extra["comparison: torch.matmul bf16 on the same expanded operands, M=%d N=%d K=%d" % (gm, gn, gk)] = {
                "ms": round(tmv.ms, 4), "TFLOP/s": round(fl / (tmv.ms * 1e-3) / 1e12, 1),
                "frac_of_2.5PFLOPs_bf16": round(fl / (tmv.ms * 1e-3) / MFMA_PEAK, 4)}
            del ca, cb, go, xa, xb
        lm, ln, lk = 2048, 4096, 4096
        xa = torch.randn(lm, lk, device=dev).to(torch.bfloat16)
        xw = (torch.randn(ln, lk, device=dev) * 0.02).to(torch.bfloat16)
        oref = xa.float() @ xw.float().t()
        nws = hif8.hif8_calibrate_workspace_bytes(lm, ln, lk, 10, 10)
        ws = torch.empty(nws, dtype=torch.uint8, device=dev)
        cerr = torch.zeros(100, dtype=torch.float64, device=dev)
        best = torch.zeros(2, dtype=torch.int32, device=dev)
        tm = timed(lambda i: hif8.hif8_calibrate_layer_bf16(xa, xw, oref, lm, ln, lk, -4, 10, -4, 10, hif8.RM_TA,
                                                                   ws, nws, cerr, best), 3, 1)
        extra["calibrate_layer_bf16 (Algorithm 1, 10x10 scales) M=%d N=%d K=%d" % (lm, ln, lk)] = {
            "ms": round(tm.ms, 3), "TFLOP/s over the 100 GEMMs": round(100 * 2.0 * lm * ln * lk / (tm.ms * 1e-3) / 1e12, 1),
            "best_Ea_Ew": best.cpu().tolist()}
        del xa, xw, oref, ws
        torch.cuda.empty_cache()

        # C4: gradient tensor, 2^30 FP32, TA and HR
        g = workloads.gradient_f32(1 << 30, dev)
        gc = torch.empty(g.numel(), dtype=torch.uint8, device=dev)
        for name, mode in (("TA", hif8.RM_TA), ("HR", hif8.RM_HR)):
            tm = timed(lambda i: hif8.hif8_encode_f32(g, gc, g.numel(), 1.0, mode), 20, 20)
            extra["C4 encode_f32 %s 2^30 (5 B/elem)" % name] = rate(5 * g.numel(), tm)
        del g, gc
        torch.cuda.empty_cache()

        # C5: LLM weight cast, 225 BF16 tensors, amax -> scale -> encode back to back
        arena, index = workloads.llm_weights_bf16(dev)
        wc = torch.empty(arena.numel(), dtype=torch.uint8, device=dev)
        ams = torch.zeros(len(index), dtype=torch.float32, device=dev)
        scs = torch.zeros(len(index), 2, dtype=torch.float32, device=dev)
        ap, cp, amp, scp = arena.data_ptr(), wc.data_ptr(), ams.data_ptr(), scs.data_ptr()

        def c5(i):
            for t, (_, off, cnt) in enumerate(index):
                hif8.hif8_amax_bf16(ap + 2 * off, cnt, amp + 4 * t)
                hif8.hif8_scale_from_amax(amp + 4 * t, scp + 8 * t, hif8.MAX_FINITE, 0)
                hif8.hif8_encode_bf16_ds(ap + 2 * off, cp + off, cnt, scp + 8 * t, hif8.RM_TA)

        tot = arena.numel()
        tm = timed(c5, 5, 1)
        extra["C5 per-tensor calls, 225 x (amax, scale, encode_bf16) (3 B/elem primary)"] = rate(3 * tot, tm)
        extra["C5 per-tensor calls (5 B/elem with amax pass)"] = rate(5 * tot, tm)
        ws = torch.zeros(hif8.hif8_quantize_workspace_bytes(), dtype=torch.uint8, device=dev)

        def c5_qt(i):
            for t, (_, off, cnt) in enumerate(index):
                hif8.hif8_quantize_tensor_bf16(ap + 2 * off, None, cp + off, cnt, amp + 4 * t, scp + 8 * t, ws,
                                               hif8.MAX_FINITE, 0, hif8.RM_TA)

        tm = timed(c5_qt, 5, 1)
        extra["C5 per-tensor calls, 225 x hif8_quantize_tensor_bf16 (2 launches each) (3 B/elem primary)"] = rate(3 * tot, tm)
        items = [(ap + 2 * off, cp + off, cnt) for _, off, cnt in index]
        plan = hif8.hif8_multi_plan(items, src_is_16bit=True)
        d_items, count, tiles = plan
        tm = timed(lambda i: hif8.hif8_multi_cast_bf16(d_items, count, tiles, ams, scs, hif8.MAX_FINITE, 0, hif8.RM_TA,
                                                               host_items=plan.host_items), 5, 1)
        extra["C5 multi-tensor cast, group-wise (amax of a group while the previous one is cast) (3 B/elem primary)"] = rate(3 * tot, tm)
        extra["C5 multi-tensor cast, group-wise (5 B/elem with amax pass)"] = rate(5 * tot, tm)
        tm = timed(lambda i: hif8.hif8_multi_cast_bf16(d_items, count, tiles, ams, scs, hif8.MAX_FINITE, 0, hif8.RM_TA), 5, 1)
        extra["C5 multi-tensor cast, 4 launches (3 B/elem primary)"] = rate(3 * tot, tm)
        extra["C5 multi-tensor cast, 4 launches (5 B/elem with amax pass)"] = rate(5 * tot, tm)
        extra["C5 multi-tensor cast wall ms"] = round(tm.wall_ms, 3)
        # the paper's delayed scaling (Sec. 5): scales from earlier iterations, the amax of each tensor
        # accumulated by the cast itself for the next update -- one pass, one launch per tensor
        accs = torch.zeros(len(index), dtype=torch.float32, device=dev)
        acp = accs.data_ptr()

        def c5_delayed(i):
            for t, (_, off, cnt) in enumerate(index):
                hif8.hif8_encode_bf16_ds(ap + 2 * off, cp + off, cnt, scp + 8 * t, hif8.RM_TA, d_amax_accum=acp + 4 * t)

        tm = timed(c5_delayed, 5, 1)
        extra["C5 with delayed scaling: 225 x encode_bf16_ds + amax accumulated in the same pass (3 B/elem)"] = rate(3 * tot, tm)
        tm = timed(lambda i: hif8.hif8_multi_encode_bf16_ds(d_items, count, tiles, scs, hif8.RM_TA, d_amax_accum=accs), 5, 1)
        extra["C5 with delayed scaling: multi-tensor encode + amax accumulation, 1 launch (3 B/elem)"] = rate(3 * tot, tm)
        result["extra"] = extra
        for k, v in extra.items():
            log("%-64s %s" % (k, v))

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
