#!/usr/bin/env python3
"""Benchmark of the cascade hot path on one MI355X.

A step is one whole pass (pyramid -> stage-1 score map -> compaction -> stage 2 -> compaction ->
stage 3 -> compaction -> merge -> detections on the host) over one synthetic 3840x2160 frame that is
already resident in device memory.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--inflight F] [--workload uhd|uhd_small_faces|fhd|vga]

Every timed leg is preceded by an untimed, time-based pre-warm of the same loop (--prewarm seconds) so that a short
run (--steps 20) measures the same state of the GPU as a long one; the W warm-up steps follow it and the K timed
steps are bracketed by device synchronisation.  The headline is timed twice over exactly K steps, with F frames in
flight on F contexts / streams (with plain launches, and through the ring with one captured graph per frame) and one frame at
a time; `value` is the fastest and all are reported.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "frames/sec at 3840x2160, min face 60 px (full cascade); stage-1 windows/sec"

# Algorithmic work per unit: 2 x the multiply-accumulates of the layer definitions, whatever the kernels execute.
S1_FLOP_PER_WINDOW = 2 * 396
S2_FLOP_PER_CROP = 2 * 161952
S3_FLOP_PER_CROP = 2 * 5473600
S2_CONV_FLOP_PER_CROP = 2 * (80000 + 73728)            # conv kernel of stage 2 (conv1 + conv2)
S3_CONV_FLOP_PER_CROP = 2 * (774400 + 4147200 + 451584)  # conv kernel of stage 3 (conv1..conv3)
MFMA_FLOP = 2 * 16 * 16 * 4                            # one 16x16x4 matrix instruction
SEL_MAC_CNN2 = 48 * 52 * 4 * 16 + 22 * 24 * 19 * 36 + 25 * 19 * 56      # one pass of CNN_2 over a 51x55 region
SEL_MAC_CNN3 = 48 * 52 * 5 * 16 + 22 * 24 * 28 * 45 + 25 * 28 * 56      # one pass of CNN_3
SCAN_FLOP_PER_POSITION = 2 * (1024 + 1584 + 330)       # 27x31 scan: conv1 + conv2 + conv3 MACs per window position at step 4
PEAK_HBM = 8000.0          # GB/s
PEAK_FP32_VECTOR = 157.3   # TFLOP/s, published vector fp32 figure
PEAK_FP32_MFMA = 157.3     # TFLOP/s, published dense fp32 matrix figure
KERNEL_NAMES = {"stage1": "stage1_kernel", "stage2_conv": "eval2_conv_kernel", "stage3_conv": "eval3_conv_kernel",
                "pyramid": "pyramid_kernel"}


def measured_traffic(workload, kernel):
    """HBM bytes per launch (read + written) of `kernel` from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE
    summary of this workload, or None when no such summary exists.  Returns (bytes, file name)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s_pmc.txt" % workload)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith(kernel):
                    cols = line.split()
                    return (float(cols[-2]) + float(cols[-1])) * 1e6, os.path.relpath(path, ROOT)
    except (OSError, ValueError, IndexError):
        pass
    return None, None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--inflight", type=int, default=3, help="frames in flight on separate streams")
    ap.add_argument("--prewarm", type=float, default=1.0, help="seconds of untimed running before each timed leg")
    ap.add_argument("--workload", default="uhd")
    ap.add_argument("--q1", type=float, default=0.02, help="stage-1 survival quantile (the benchmark's rule: 2 %%)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ingest", action="store_true", help="skip the host-memory ingest leg (its frames overlap on several "
                    "streams, which stretches per-kernel durations in a profiler trace)")
    ap.add_argument("--no-paper-path", action="store_true", help="skip the legs in the paper's own geometry")
    ap.add_argument("--chunks", type=int, default=2, help="cnnc_set_async_chunks value of the extra one-frame-at-a-time leg "
                    "(asynchronous mode inside a frame; 0 skips the leg)")
    ap.add_argument("--eval-impl", type=int, default=None, help="cnnc_set_eval_impl value (default: the library's)")
    ap.add_argument("--fused-stage1", type=int, default=None, help="cnnc_set_fused_stage1 value (default: the library's)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives, no sharding)" % a.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import cnnc_inputs as I
    import paper_1508_01292_amd as P
    from oracle import oracle as O

    ci = [c["name"] for c in I.CONFIGS].index(a.workload)
    cfg = I.CONFIGS[ci]
    seed = I.config_seed(ci)
    casc = I.default_cascade()
    W = I.draw_weights(casc, seed)
    frames = I.make_stream(ci)
    frame = frames[0]

    # ---- CPU oracle: thresholds at the survival quantiles (the oracle's job) and the cpu_baseline leg
    thr_pooled = None
    if len(frames) > 1:      # a stream: thresholds sit at the quantiles of the scores pooled over all frames
        pyrs = [O.build_pyramid(f, cfg["min_face"], cfg["scale_step"]) for f in frames]
        s1 = [O.stage1_scores(p, casc[0], W[0]) for p in pyrs]
        t1 = O.threshold_from_quantile(np.concatenate(s1), a.q1)
        s2 = [O.eval_stage(f, p, O.survivors(s, t1), casc[1], W[1]) for f, p, s in zip(frames, pyrs, s1)]
        thr_pooled = (float(t1), float(O.threshold_from_quantile(np.concatenate(s2), 0.2)), 0.0)
    n_cores = O.num_threads()
    t0 = time.perf_counter()
    tr = O.detect(frame, casc, W, cfg["min_face"], cfg["scale_step"], thr=thr_pooled, quantiles=(a.q1, 0.2))
    t_cpu = time.perf_counter() - t0
    n_windows = int(tr.score1.size)
    cpu = None
    if not a.no_cpu_baseline:
        # the first stage in both forms of the oracle (dense single pass; per-window definition), all cores and one
        # thread, and the whole frame on one thread; the per-window form at one thread runs on a sample of levels
        pyr_o = tr.pyramid

        def timed(fn):
            t = time.perf_counter()
            r = fn()
            return time.perf_counter() - t, r

        def level_set(budget_windows):
            """Coarsest levels first until about `budget_windows` windows are covered."""
            lv, n = [], 0
            for l in reversed(pyr_o.levels):
                lv.append(l)
                n += (l.shape[0] - 11) * (l.shape[1] - 11)
                if n >= budget_windows:
                    break
            return lv, n

        s1_forms = {}
        for form, budget1 in (("dense", n_windows), ("windows", 200000)):
            t_all, _ = timed(lambda: [O.stage1_level(l, casc[0], W[0], form) for l in pyr_o.levels])
            lv1, n1w = level_set(budget1)
            O.set_num_threads(1)
            t_one, _ = timed(lambda: [O.stage1_level(l, casc[0], W[0], form) for l in lv1])
            O.set_num_threads(n_cores)
            s1_forms[form] = {"all_cores_windows_per_s": n_windows / t_all, "all_cores_s": t_all, "cores": n_cores,
                              "one_thread_windows_per_s": n1w / t_one, "one_thread_s": t_one,
                              "one_thread_sample_windows": n1w}
        O.set_num_threads(1)
        t_cpu1, _ = timed(lambda: O.detect(frame, casc, W, cfg["min_face"], cfg["scale_step"], thr=tr.thr))
        O.set_num_threads(n_cores)
        cpu = {"value": 1.0 / t_cpu, "unit": "frames/s", "cores": n_cores, "kind": "oracle",
               "sample": "1 whole %dx%d frame through the oracle (dense stage-1 form, fp64, OpenMP): %.2f s on %d threads, "
                         "%.2f s on one thread; stage 1 alone in stage1_forms: 'dense' = single pass over each level, "
                         "'windows' = the per-window definition (its one-thread figure on the coarsest levels holding "
                         "%d windows)" % (cfg["width"], cfg["height"], t_cpu, n_cores, t_cpu1,
                                          s1_forms["windows"]["one_thread_sample_windows"]),
               "one_thread_frames_per_s": 1.0 / t_cpu1, "stage1_forms": s1_forms}

    # ---- GPU
    torch.cuda.set_device(0)
    dev_frames = [torch.from_numpy(f).cuda() for f in frames]
    dev_frame = dev_frames[0]
    F = max(1, a.inflight)
    max_surv = max(32768, 1 << int(np.ceil(np.log2(2 * max(1, len(tr.idx1))))))
    ctxs = [P.Context(casc, W, cfg["width"], cfg["height"], max_surv) for _ in range(F)]
    # streams that are destroyed again before the ingest legs: a process has four hardware queues, and streams left alive
    # (torch's are pooled and never destroyed) would make the ring's four streams share queues among themselves
    streams = [P.Stream() for _ in range(F)]
    for c in ctxs:
        c.set_params(cfg["min_face"], cfg["scale_step"], tr.thr)
        if a.eval_impl is not None:
            c.set_eval_impl(a.eval_impl)
        if a.fused_stage1 is not None:
            c.set_fused_stage1(bool(a.fused_stage1))
    c0 = ctxs[0]

    def run_inflight(n_steps):
        busy = [False] * F
        n_det = 0
        for i in range(n_steps):
            j = i % F
            if busy[j]:
                n_det = len(ctxs[j].fetch_detections(8192))
            ctxs[j].detect_async(dev_frames[i % len(dev_frames)], streams[j])
            busy[j] = True
        for j in range(F):
            if busy[j]:
                n = len(ctxs[j].fetch_detections(8192))
                if j == (n_steps - 1) % F:       # the frame of the last step, as run_serial returns it
                    n_det = n
        return n_det

    def run_serial(n_steps):
        n_det = 0
        for i in range(n_steps):
            n_det = len(c0.detect(dev_frames[i % len(dev_frames)], 8192))
        return n_det

    def prewarm(fn, chunk):
        """Untimed: run the leg's own loop until --prewarm seconds have passed (clocks, caches, first-use costs)."""
        t_end = time.perf_counter() + a.prewarm
        while True:
            fn(chunk)
            if time.perf_counter() >= t_end:
                break
        torch.cuda.synchronize()

    def timed_leg(fn, chunk):
        prewarm(fn, chunk)
        if a.warmup > 0:
            fn(a.warmup)
        torch.cuda.synchronize()
        t = time.perf_counter()
        n = fn(a.steps)
        torch.cuda.synchronize()
        return time.perf_counter() - t, n

    el_inflight, n_det = timed_leg(run_inflight, 4 * F)
    el_serial, n_det_serial = timed_leg(run_serial, 4)
    assert n_det == n_det_serial
    fps_inflight, fps_serial = a.steps / el_inflight, a.steps / el_serial
    # the same F frames in flight, resident in device memory, through the ring (cnnc_pipe_submit_device): a frame is one
    # captured graph launch instead of sixteen or more launches, which counts where the host's calls are the limit
    ring = P.Pipe(casc, W, cfg["width"], cfg["height"], max_surv, depth=F, use_graph=True)
    ring.set_params(cfg["min_face"], cfg["scale_step"], tr.thr)

    def run_ring(n_steps):
        q, n = [], 0
        for i in range(n_steps):
            if len(q) == ring.depth:
                n = len(ring.fetch(q.pop(0), 8192))
            q.append(ring.submit_device(dev_frames[i % len(dev_frames)]))
        for t in q:
            n = len(ring.fetch(t, 8192))
        return n

    el_ring, n_det_ring = timed_leg(run_ring, 4 * F)
    assert n_det_ring == n_det
    ring.close()
    fps_ring = a.steps / el_ring
    elapsed = min(el_inflight, el_serial, el_ring)
    fps = a.steps / elapsed
    latency_ms = el_serial / a.steps * 1e3
    # asynchronous mode inside a frame: stage 1 of the next chunk of pyramid levels overlaps stages 2-3 of the last one
    chunked = None
    if a.chunks > 1:
        c0.set_async_chunks(a.chunks)
        c0.set_params(cfg["min_face"], cfg["scale_step"], tr.thr)
        el_chunked, n_det_chunked = timed_leg(run_serial, 4)
        assert n_det_chunked == n_det
        chunked = {"chunks": a.chunks, "ms_per_frame_one_at_a_time": el_chunked / a.steps * 1e3}
        c0.set_async_chunks(1)
        c0.set_params(cfg["min_face"], cfg["scale_step"], tr.thr)
        run_serial(4)
    # a stream: every frame on its own, to show how much the time depends on the content of the frame
    per_frame = None
    if len(dev_frames) > 1:
        lat = []
        for f in dev_frames:
            c0.detect(f, 8192)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                c0.detect(f, 8192)
            torch.cuda.synchronize()
            lat.append((time.perf_counter() - t0) / 5 * 1e3)
        per_frame = {"min": min(lat), "mean": sum(lat) / len(lat), "max": max(lat)}

    # per-kernel times: HIP events recorded by the library on the stream the kernels run on
    n_timed = max(a.steps, 200) if a.steps >= 20 else a.steps      # (a profiler's counter passes ask for a few steps only)
    c0.set_timing(True)
    c0.get_timings()
    for _ in range(n_timed):
        c0.detect_async(dev_frame, streams[0])
        c0.fetch_detections(8192)
    tm = c0.get_timings()
    c0.set_timing(False)
    # per frame: a step may consist of several launches (a long stage-3 list goes through its kernels in segments)
    ms = {k: v[0] / n_timed for k, v in tm.items()}
    n1, n2, n3 = (c0.survivor_count(s) for s in (1, 2, 3))
    lay = c0.pyramid_layout(cfg["width"], cfg["height"])
    pyr_bytes = lay["pyr_off"][-1]
    mfma2, mfma3 = c0.executed_mfma(2), c0.executed_mfma(3)

    def tflops(flop, t_ms):
        return flop / (t_ms * 1e-3) / 1e12 if t_ms > 0 else 0.0

    def gbs(nbytes, t_ms):
        return nbytes / (t_ms * 1e-3) / 1e9 if t_ms > 0 else 0.0

    paper = None
    if not a.no_paper_path:
        make_pipe = None if a.no_ingest else (lambda: P.Pipe(casc, W, cfg["width"], cfg["height"], max_surv, depth=F + 1, use_graph=True))
        paper = paper_geometry_legs(a, ctxs, streams, dev_frame, frame, cfg, seed, tr, I, O, np, torch, time, tflops, make_pipe)

    kernels = {
        "pyramid": {"bound": "hbm", "ms": ms["pyramid"], "achieved": gbs(cfg["width"] * cfg["height"] + pyr_bytes, ms["pyramid"]),
                    "peak": PEAK_HBM, "unit": "GB/s"},
        "stage1": {"bound": "alu", "ms": ms["stage1"], "achieved": tflops(S1_FLOP_PER_WINDOW * n_windows, ms["stage1"]),
                   "peak": PEAK_FP32_VECTOR, "unit": "TFLOP/s"},
        "compact1": {"bound": "hbm", "ms": ms["compact1"], "achieved": gbs(4 * n_windows + 8 * n1, ms["compact1"]),
                     "peak": PEAK_HBM, "unit": "GB/s"},
        "stage2": {"bound": "mfma", "ms": ms["stage2"], "achieved": tflops(S2_FLOP_PER_CROP * n1, ms["stage2"]),
                   "peak": PEAK_FP32_MFMA, "unit": "TFLOP/s"},
        "stage2_conv": {"bound": "mfma", "ms": ms["stage2_conv"], "achieved": tflops(S2_CONV_FLOP_PER_CROP * n1, ms["stage2_conv"]),
                        "peak": PEAK_FP32_MFMA, "unit": "TFLOP/s",
                        "executed": tflops(MFMA_FLOP * mfma2 * n1, ms["stage2_conv"]), "mfma_per_crop": mfma2},
        "stage3": {"bound": "mfma", "ms": ms["stage3"], "achieved": tflops(S3_FLOP_PER_CROP * n2, ms["stage3"]),
                   "peak": PEAK_FP32_MFMA, "unit": "TFLOP/s"},
        "stage3_conv": {"bound": "mfma", "ms": ms["stage3_conv"], "achieved": tflops(S3_CONV_FLOP_PER_CROP * n2, ms["stage3_conv"]),
                        "peak": PEAK_FP32_MFMA, "unit": "TFLOP/s",
                        "executed": tflops(MFMA_FLOP * mfma3 * n2, ms["stage3_conv"]), "mfma_per_crop": mfma3},
        "compact2": {"ms": ms["compact2"]}, "compact3": {"ms": ms["compact3"]}, "merge": {"ms": ms["merge"]},
    }
    for k in kernels.values():
        if "achieved" in k:
            k["frac"] = k["achieved"] / k["peak"]
        if "executed" in k:
            k["executed_frac"] = k["executed"] / k["peak"]
    # the dominant single kernel: the convolution kernel of the slowest step, or the step's own kernel
    dom = max(("stage1", "stage2_conv", "stage3_conv", "pyramid"), key=lambda k: ms[k])
    traffic, traffic_src = measured_traffic(a.workload, KERNEL_NAMES[dom])
    roof = {"bound": kernels[dom]["bound"], "achieved": kernels[dom]["achieved"], "peak": kernels[dom]["peak"],
            "unit": kernels[dom]["unit"], "frac": kernels[dom]["frac"],
            "traffic": traffic, "traffic_from": traffic_src, "kernel": KERNEL_NAMES[dom], "avg_launch_ms": ms[dom]}
    if "executed" in kernels[dom]:
        # `achieved` counts the multiply-adds of the layer definitions; the Winograd forms execute fewer.  `executed`
        # counts the matrix instructions the kernel really issues: that fraction is the utilisation of the matrix cores.
        roof["executed"] = kernels[dom]["executed"]
        roof["executed_frac"] = kernels[dom]["executed_frac"]
    try:
        mf, vf, hb = P.cnnc_measure_peaks()
        roof["sustained_on_this_gpu"] = {"mfma_f32_tflops": mf, "valu_f32_tflops": vf, "hbm_copy_gbs": hb}
        # the two machine facts the kernels' designs lean on (include/cnnc.h, measurement aids)
        roof["sustained_on_this_gpu"]["issue_ns_per_wave_instruction_and_simd"] = P.cnnc_measure_issue_rates()
        roof["sustained_on_this_gpu"]["lds_read_ns_per_wave_instruction_and_cu"] = {
            "b32_consecutive": P.cnnc_measure_lds_read(list(range(64)), 1),
            "b32_every_second_dword": P.cnnc_measure_lds_read([2 * i for i in range(64)], 1),
            "b64_consecutive": P.cnnc_measure_lds_read([2 * i for i in range(64)], 2),
            "b128_consecutive": P.cnnc_measure_lds_read([4 * i for i in range(64)], 4)}
    except Exception as e:       # a probe failure must not lose the benchmark line
        roof["sustained_on_this_gpu"] = {"error": str(e)}

    # frames from pinned host memory through the ingest ring: copy in + path + results out, PCIe included
    ingest = {}
    D = F + 1                                    # one slot more than frames computing: its copy runs ahead
    torch.cuda.synchronize()
    for s in streams:
        s.close()
    for use_graph in (() if a.no_ingest else (False, True)):
        pipe = P.Pipe(casc, W, cfg["width"], cfg["height"], max_surv, depth=D, use_graph=use_graph)
        pipe.set_params(cfg["min_face"], cfg["scale_step"], tr.thr)
        for j in range(D):                       # the producer's frames sit in the pinned buffers already
            pipe.frame_buffer()[:] = frames[j % len(frames)]
            pipe.fetch(pipe.submit(), 8192)

        def run_pipe(n_steps):
            q = []
            for _ in range(n_steps):
                if len(q) == D:
                    pipe.fetch(q.pop(0), 8192)
                q.append(pipe.submit())
            n = 0
            for t in q:
                n = len(pipe.fetch(t, 8192))
            return n

        dt, n_det_pipe = timed_leg(run_pipe, 4 * D)
        ingest["graph" if use_graph else "eager"] = {"frames_per_s": a.steps / dt, "detections": n_det_pipe,
                                                     "h2d_gb_per_s": a.steps / dt * cfg["width"] * cfg["height"] / 1e9}
        pipe.close()
    ingest["depth"] = D

    out = {
        "metric": METRIC, "value": fps, "unit": "frames/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": elapsed / a.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %d %dx%d uint8 frame(s), min face %g px, scale step %g, %g%% / 20%% survival quantiles, T3 = 0"
                               % (cfg["name"], len(frames), cfg["width"], cfg["height"], cfg["min_face"], cfg["scale_step"],
                                  100 * a.q1),
                   "frames_in_flight": 1 if el_serial <= min(el_inflight, el_ring) else F,
                   "launches": "one at a time" if el_serial <= min(el_inflight, el_ring) else
                               ("one captured graph per frame" if el_ring < el_inflight else "plain launches"),
                   "windows": n_windows,
                   "survivors": [n1, n2, n3], "detections": n_det, "prewarm_s": a.prewarm,
                   "stage1_weights": "instruction literals" if c0.literal_weights() else "memory"},
        "frames_per_s": {"in_flight_%d" % F: fps_inflight, "in_flight_%d_graphs" % F: fps_ring, "one_at_a_time": fps_serial},
        "stage1_windows_per_s": n_windows / (ms["stage1"] * 1e-3) if ms["stage1"] > 0 else None,
        "latency_ms_single_frame": latency_ms,
        "latency_ms_per_frame_of_stream": per_frame,
        "asynchronous_mode_inside_a_frame": chunked,
        "paper_geometry": paper,
        "ingest_from_pinned_host_memory": ingest,
        "sum_of_kernel_ms": sum(v for k, v in ms.items() if not k.endswith("_conv") and k not in ("scan", "select")),
        "roofline": roof,
        "kernels": kernels,
        "cpu_baseline": cpu,
    }
    for c in ctxs:
        c.close()
    print(json.dumps(out))


def paper_geometry_legs(a, ctxs, streams, dev_frame, frame, cfg, seed, tr, I, O, np, torch, time, tflops, make_pipe=None):
    """The first stage in the paper's own geometry (27 x 31 window, 4 pixel step) on the same pyramid, the selective
    unit on the positions above the 2 % quantile of that scan, and the merge of what it accepts: reported beside the
    headline, in the paper's unit (window positions at step 4, regions)."""
    c0, stream = ctxs[0], streams[0]
    scan_net = I.paper_stage1()
    w_scan = I.draw_scan_weights(scan_net, seed)
    for c in ctxs:
        c.scan_set_weights(w_scan, 1)
    c0.build_pyramid(dev_frame, stream)
    few = a.steps < 20                       # a profiler's counter passes: a handful of launches of everything
    n_rep = a.steps if few else max(a.steps, 200)
    t_end = time.perf_counter() + min(a.prewarm, 0.3)
    while time.perf_counter() < t_end:
        c0.scan_scoremap(stream)
    c0.set_timing(True)
    c0.get_timings()
    for _ in range(n_rep):
        c0.scan_scoremap(stream)
    tm_scan = c0.get_timings()["scan"]
    c0.set_timing(False)
    ms_scan = tm_scan[0] / tm_scan[1] if tm_scan[1] else 0.0
    n_scan = int(c0.scan_layout(cfg["width"], cfg["height"])["out_off"][-1])
    # Thresholds of the unit from a sample of regions (oracle): T_2 so that CNN_2 leaves no vote in about a third
    # of the regions (they stop there, eq. (2)), T_3 at the median of CNN_3's responses, T_nn = 5.
    n2_net, n3_net = I.paper_stage2(), I.paper_stage3()
    w2_sel, w3_sel = I.draw_scan_weights(n2_net, seed + 1), I.draw_scan_weights(n3_net, seed + 2)
    for c in ctxs:
        c.select_set_weights(w2_sel, w3_sel, 1)
    pyr_o = tr.pyramid
    scan_o = O.scan_scores(pyr_o, scan_net, w_scan)
    t1_scan = float(O.threshold_from_quantile(scan_o, 0.02))
    sample = np.nonzero(scan_o.astype(np.float32) > np.float32(t1_scan))[0][::24]
    ref_sel = O.select_unit(frame, pyr_o, sample, scan_net, n2_net, w2_sel, n3_net, w3_sel, -1e30, -1e30, 1)
    t2_sel = float(np.quantile([r["r2"].max() for r in ref_sel], 0.33))
    t3_sel = float(np.median(np.concatenate([r["r3"].ravel() for r in ref_sel])))
    t_end = time.perf_counter() + min(a.prewarm, 0.3)
    while time.perf_counter() < t_end:
        c0.select_run(t1_scan, t2_sel, t3_sel, 5, stream)
    c0.set_timing(True)
    c0.get_timings()
    for _ in range(a.steps if few else max(50, a.steps // 4)):
        c0.select_run(t1_scan, t2_sel, t3_sel, 5, stream)
    tm_sel = c0.get_timings()["select"]
    c0.set_timing(False)
    ms_sel = tm_sel[0] / tm_sel[1] if tm_sel[1] else 0.0
    sel = c0.select_fetch(65536)
    # merge of the accepted regions: the call waits for its result, so this is wall-clock time per call
    sel_det = c0.select_merge(0.3, 1, 32768, stream)
    n_merge = a.steps if few else 50
    t0 = time.perf_counter()
    for _ in range(n_merge):
        c0.select_merge(0.3, 1, 32768, stream)
    ms_sel_merge = (time.perf_counter() - t0) / n_merge * 1e3
    # the path in the paper's geometry end to end through cnnc_detect_paper: one frame at a time, and frames in flight
    n_paper, n_skip = (a.steps, 1) if few else (max(100, a.steps // 4), 20)
    for it in range(n_paper + n_skip):
        if it == n_skip:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        n_paper_det = len(c0.detect_paper(dev_frame, t1_scan, t2_sel, t3_sel, 5, 0.3, 1, 32768))
    ms_paper_frame = (time.perf_counter() - t0) / n_paper * 1e3
    assert n_paper_det == len(sel_det)
    F = len(ctxs)

    def run_paper(n_steps):
        busy = [False] * F
        for i in range(n_steps):
            j = i % F
            if busy[j]:
                ctxs[j].fetch_paper(32768)
            ctxs[j].detect_paper_async(dev_frame, t1_scan, t2_sel, t3_sel, 5, 0.3, 1, streams[j])
            busy[j] = True
        for j in range(F):
            if busy[j]:
                ctxs[j].fetch_paper(32768)

    n_fly = n_paper if few else 4 * n_paper
    run_paper(F if few else 10 * F)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_paper(n_fly)
    torch.cuda.synchronize()
    ms_paper_inflight = (time.perf_counter() - t0) / n_fly * 1e3
    # the same path fed from pinned host memory through the ingest ring (PCIe included; never the headline value)
    fps_paper_ingest = fps_paper_ring = None
    if make_pipe is not None:
        torch.cuda.synchronize()
        for s in streams:                             # see the note where they are created
            s.close()
        pipe = make_pipe()
        pipe.set_params(cfg["min_face"], cfg["scale_step"], (0.0, 0.0, 0.0))
        pipe.set_paper(w_scan, w2_sel, w3_sel, t1_scan, t2_sel, t3_sel, 5, 0.3, 1)
        D = pipe.depth

        def run_pipe(n_steps):
            q = []
            for _ in range(n_steps):
                if len(q) == D:
                    pipe.fetch_paper(q.pop(0), 32768)
                q.append(pipe.submit())
            return [len(pipe.fetch_paper(t, 32768)) for t in q][-1]

        for j in range(D):
            pipe.frame_buffer()[:] = frame
            pipe.fetch_paper(pipe.submit(), 32768)
        run_pipe(D if few else 10 * D)
        t0 = time.perf_counter()
        n_pipe_det = run_pipe(n_fly)
        fps_paper_ingest = n_fly / (time.perf_counter() - t0)
        assert n_pipe_det == n_paper_det

        def run_pipe_resident(n_steps):               # the same ring fed with the frame that is on the device already
            q = []
            for _ in range(n_steps):
                if len(q) == D:
                    pipe.fetch_paper(q.pop(0), 32768)
                q.append(pipe.submit_device(dev_frame))
            return [len(pipe.fetch_paper(t, 32768)) for t in q][-1]

        run_pipe_resident(D if few else 10 * D)
        t0 = time.perf_counter()
        n_pipe_det = run_pipe_resident(n_fly)
        fps_paper_ring = n_fly / (time.perf_counter() - t0)
        assert n_pipe_det == n_paper_det
        pipe.close()
    sel_flop = 2.0 * sum(2 * SEL_MAC_CNN2 + (2 * SEL_MAC_CNN3 if r.k2 > 0 else 0) for r in sel)
    c0.detect(dev_frame, 8192)           # leaves the context with the cascade's own survivor lists again
    return {
        "stage1": {"window": "27x31", "step": 4, "positions": n_scan, "ms": ms_scan,
                   "positions_per_s": n_scan / (ms_scan * 1e-3) if ms_scan > 0 else None,
                   "bound": "alu", "achieved": tflops(SCAN_FLOP_PER_POSITION * n_scan, ms_scan),
                   "peak": PEAK_FP32_VECTOR, "unit": "TFLOP/s",
                   "frac": tflops(SCAN_FLOP_PER_POSITION * n_scan, ms_scan) / PEAK_FP32_VECTOR},
        "selective_unit": {"regions": len(sel), "stopped_after_cnn2": sum(r.k2 == 0 for r in sel),
                           "faces": sum(r.face for r in sel), "ms": ms_sel,
                           "regions_per_s": len(sel) / (ms_sel * 1e-3) if ms_sel > 0 else None, "bound": "alu",
                           "achieved": tflops(sel_flop, ms_sel), "peak": PEAK_FP32_VECTOR, "unit": "TFLOP/s",
                           "frac": tflops(sel_flop, ms_sel) / PEAK_FP32_VECTOR},
        "merge": {"detections": len(sel_det), "ms_per_call_with_wait_and_readback": ms_sel_merge},
        "whole_path_ms_per_frame_one_at_a_time": ms_paper_frame,
        "whole_path_frames_per_s_%d_in_flight" % F: 1e3 / ms_paper_inflight,
        "whole_path_frames_per_s_3_in_flight_graphs": fps_paper_ring,
        "whole_path_frames_per_s_from_pinned_host_memory": fps_paper_ingest,
        "whole_path_ingest_ring": None if make_pipe is None else {"slots": F + 1, "lanes": min(F + 1, 3), "graphs": True}}


if __name__ == "__main__":
    main()
