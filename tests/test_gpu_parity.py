"""GPU parity tests: the HIP path, called through the C ABI (ctypes binding), against the CPU oracle
on the same seeded inputs, element by element."""
import numpy as np
import pytest

import cnnc_inputs as I
from oracle import oracle as O

from parity import (ATOL, RTOL, assert_scores, assert_survivors, boxes_of, compare_with_trace, greedy_merge_check,
                    run_gpu_steps)

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def _ctx(cascade, weights, w, h, max_surv=200000):
    import paper_1508_01292_amd as P
    return P.Context(cascade, weights, w, h, max_surv)


def _full_case(frame, cascade, weights, min_face, step, quantiles=(0.02, 0.2), name="", det_cap=8192):
    torch = _torch()
    print("case", name, frame.shape, "min_face", min_face, "step", step, flush=True)
    tr = O.detect(frame, cascade, weights, min_face, step, quantiles=quantiles)
    ctx = _ctx(cascade, weights, frame.shape[1], frame.shape[0])
    ctx.set_params(min_face, step, tr.thr)
    g = run_gpu_steps(ctx, torch.from_numpy(frame).cuda(), tr.thr, det_cap=det_cap)
    info = compare_with_trace(g, tr, frame, cascade, weights)
    # the one-call wrapper gives the same detections as the step-by-step calls
    det = [d.as_dict() for d in ctx.detect(torch.from_numpy(frame).cuda(), det_cap)]
    assert det == g["det"]
    ctx.close()
    print("   windows %d -> %d -> %d -> %d -> %d detections; band %s merge_exact %s"
          % (tr.score1.size, len(g["idx1"]), len(g["idx2"]), len(g["idx3"]), len(g["det"]), info["band"],
             info["merge_exact"]), flush=True)
    return tr, g, info


@pytest.mark.parametrize("act", [I.ACT_RATIONAL, I.ACT_SCALED_TANH, I.ACT_TANH])
def test_vga_workload_every_activation(act):
    c = I.CONFIGS[0]
    casc = I.default_cascade(act)
    W = I.draw_weights(casc, I.config_seed(0), bias_sd=0.0 if act == I.ACT_RATIONAL else 0.15)
    frame = I.make_frame(c["width"], c["height"], I.config_seed(0))
    tr, g, _ = _full_case(frame, casc, W, c["min_face"], c["scale_step"], name="vga act %d" % act)
    assert tr.score1.size == 23659 and len(tr.idx1) == 473 and len(tr.idx2) == 94


def test_fhd_workload():
    c = I.CONFIGS[1]
    casc = I.default_cascade()
    W = I.draw_weights(casc, I.config_seed(1))
    frame = I.make_frame(c["width"], c["height"], I.config_seed(1))
    tr, g, _ = _full_case(frame, casc, W, c["min_face"], c["scale_step"], name="fhd")
    assert tr.score1.size == 199030 and len(tr.idx1) == 3980 and len(tr.idx2) == 796


def test_vector_alu_variant_of_later_stages():
    """cnnc_set_eval_impl(0): the direct-convolution kernels kept beside the matrix-core ones."""
    torch = _torch()
    c = I.CONFIGS[0]
    casc = I.default_cascade()
    W = I.draw_weights(casc, 5, bias_sd=0.1)
    frame = I.make_frame(c["width"], c["height"], 55)
    tr = O.detect(frame, casc, W, c["min_face"], c["scale_step"])
    ctx = _ctx(casc, W, c["width"], c["height"])
    ctx.set_params(c["min_face"], c["scale_step"], tr.thr)
    ctx.set_eval_impl(0)
    g = run_gpu_steps(ctx, torch.from_numpy(frame).cuda(), tr.thr)
    compare_with_trace(g, tr, frame, casc, W)
    ctx.close()


@pytest.mark.parametrize("act", [I.ACT_RATIONAL, I.ACT_TANH])
def test_direct_sum_variant_of_stage3(act):
    """cnnc_set_eval_impl(1): the matrix-core kernels with stage-3 conv2 as a direct sum; 2 and 3 use the Winograd
    F(2,5) and F(4,5) forms for it.  Also reports how far each one's scores are from the oracle's."""
    torch = _torch()
    c = I.CONFIGS[0]
    casc = I.default_cascade(act)
    W = I.draw_weights(casc, 6, bias_sd=0.1)
    frame = I.make_frame(c["width"], c["height"], 56)
    tr = O.detect(frame, casc, W, c["min_face"], c["scale_step"], quantiles=(0.05, 0.5))
    ctx = _ctx(casc, W, c["width"], c["height"])
    ctx.set_params(c["min_face"], c["scale_step"], tr.thr)
    ref3 = dict(zip(tr.idx2.tolist(), tr.score3.tolist()))
    for impl in (1, 2, 3):
        ctx.set_eval_impl(impl)
        g = run_gpu_steps(ctx, torch.from_numpy(frame).cuda(), tr.thr)
        compare_with_trace(g, tr, frame, casc, W)
        err = np.abs(g["score3"].astype(np.float64) - np.asarray([ref3.get(i, np.nan) for i in g["idx2"].tolist()]))
        print("   stage-3 score error, implementation %d: max %.3g" % (impl, np.nanmax(err)), flush=True)
        assert np.nanmax(err) < 2e-5          # far inside the 1e-4 bar: headroom for other weights
    ctx.close()


def test_ragged_sizes_and_nonzero_biases():
    """Odd frame sizes: level sizes that leave ragged tile tails in every kernel, small scale steps,
    a pitch larger than the width."""
    torch = _torch()
    casc = I.default_cascade()
    W = I.draw_weights(casc, 77, bias_sd=0.2)
    for (w, h, mf, step) in ((333, 257, 24, 1.2), (131, 97, 12, 1.5), (257, 45, 14, 1.1)):
        frame = I.make_frame(w, h, 1000 + w)
        _full_case(frame, casc, W, mf, step, quantiles=(0.05, 0.3), name="ragged %dx%d" % (w, h))
    # pitched frame (a view into a wider tensor)
    big = I.make_frame(400, 200, 5)
    view = big[10:190, 20:350]
    tr = O.detect(np.ascontiguousarray(view), casc, W, 30, 1.25)
    ctx = _ctx(casc, W, 400, 200)
    ctx.set_params(30, 1.25, tr.thr)
    g = run_gpu_steps(ctx, torch.from_numpy(big).cuda()[10:190, 20:350], tr.thr)
    compare_with_trace(g, tr, np.ascontiguousarray(view), casc, W)
    ctx.close()


def test_degenerate_cases():
    torch = _torch()
    casc = I.default_cascade()
    W = I.draw_weights(casc, 3, bias_sd=0.1)
    # the smallest frame: one level, one window
    frame = I.make_frame(12, 12, 9, n_ellipses=0)
    tr = O.detect(frame, casc, W, 12, 2.0, thr=(-1e30, -1e30, -1e30))
    assert tr.score1.size == 1 and len(tr.det) == 1
    ctx = _ctx(casc, W, 64, 64, 16)
    ctx.set_params(12, 2.0, tr.thr)
    g = run_gpu_steps(ctx, torch.from_numpy(frame).cuda(), tr.thr)
    compare_with_trace(g, tr, frame, casc, W)
    # thresholds nothing passes: every later list is empty, no detections
    frame = I.make_frame(64, 48, 10)
    ctx.set_params(12, 1.5, (1e30, 0.0, 0.0))
    g = run_gpu_steps(ctx, torch.from_numpy(frame).cuda(), (1e30, 0.0, 0.0))
    assert len(g["idx1"]) == 0 and len(g["idx2"]) == 0 and len(g["idx3"]) == 0 and g["det"] == []
    assert ctx.detect(torch.from_numpy(frame).cuda()) == []
    ctx.close()


def test_every_window_survives_and_capacity_overflow():
    """Thresholds at -inf: the cascade degenerates to 'evaluate everything'; then a context whose lists
    are too small must report the overflow and still hold valid truncated lists."""
    import paper_1508_01292_amd as P
    torch = _torch()
    casc = I.default_cascade()
    W = I.draw_weights(casc, 4)
    frame = I.make_frame(48, 40, 12)
    thr = (-1e30, -1e30, -1e30)
    tr = O.detect(frame, casc, W, 12, 1.5, thr=thr)
    n1 = tr.score1.size
    assert len(tr.idx1) == n1 == len(tr.idx3)
    ctx = _ctx(casc, W, 48, 40, 4096)
    ctx.set_params(12, 1.5, thr)
    g = run_gpu_steps(ctx, torch.from_numpy(frame).cuda(), thr)
    compare_with_trace(g, tr, frame, casc, W)
    # densely overlapping boxes give long chains in the merge; also with a neighbour requirement
    for mn, iou in ((3, 0.3), (1, 0.6), (2, 0.05)):
        trn = O.detect(frame, casc, W, 12, 1.5, thr=thr, min_neighbors=mn, iou=iou)
        ctx.set_params(12, 1.5, thr, merge_iou=iou, min_neighbors=mn)
        det = [d.as_dict() for d in ctx.detect(torch.from_numpy(frame).cuda(), 8192)]
        got = [(d["index"], d["neighbors"]) for d in det]
        if got != [(d["index"], d["neighbors"]) for d in trn.det]:
            # with every window accepted many scores lie closer together than the score tolerance, so the greedy
            # order may legitimately differ from the oracle's: then the result must be the greedy merge of the
            # library's own accepted windows and fp32 scores (numpy restatement of the rule in parity.py)
            s3 = np.sort(np.asarray(trn.score3_kept, np.float64))
            assert np.min(np.diff(s3)) <= 2 * (ATOL + RTOL * np.abs(s3).max()), (mn, iou)
            idx3, sc3 = ctx.get_survivors(3)
            bx, by, bs, _ = boxes_of(O.build_pyramid(frame, 12, 1.5), idx3)
            valid = [(int(idx3[p]), int(n)) for p, n in greedy_merge_check(bx, by, bs, sc3, idx3, iou=iou, min_neighbors=mn)]
            assert got == valid, (mn, iou)
    ctx.close()
    small = _ctx(casc, W, 48, 40, 100)
    small.set_params(12, 1.5, thr)
    ft = torch.from_numpy(frame).cuda()
    small.build_pyramid(ft)
    small.stage1_scoremap()
    small.compact_survivors(1, thr[0])
    with pytest.raises(P.CnncError) as e:
        small.survivor_count(1)
    assert e.value.code == -3
    with pytest.raises(P.CnncError) as e:
        small.detect(ft)
    assert e.value.code == -3
    # the first 100 entries are the first 100 windows
    import ctypes as C
    pi, ps = C.c_void_p(0), C.c_void_p(0)
    P.lib().cnnc_get_survivors(small._h, C.c_int(1), C.byref(pi), C.byref(ps))
    from paper_1508_01292_amd.binding import _d2h
    assert _d2h(pi.value, 400, np.uint32).tolist() == list(range(100))
    # the overflowing call still hands over the detections made from the truncated lists, and their count
    from paper_1508_01292_amd.binding import Detection
    out, n = (Detection * 256)(), C.c_int(-7)
    rc = P.lib().cnnc_detect(small._h, *small._frame_args(ft), out, C.c_int(256), C.byref(n))
    assert rc == -3 and 0 < n.value <= 100
    assert all(0 <= out[k].index < 100 for k in range(n.value)) and sum(out[k].neighbors + 1 for k in range(n.value)) == 100
    small.close()


@pytest.mark.parametrize("size", [(64, 56), (100, 80)])
def test_merge_of_a_long_dense_list(size):
    """Every window of a small frame accepted: five thousand and fourteen thousand heavily overlapping boxes, which
    take the merge through several chunks of its sorted list, through both sizes of its overlap work items above the
    smallest and through the form for chunks with more overlapping predecessors than its pair arrays hold; the
    result must be the greedy merge of exactly those boxes."""
    torch = _torch()
    casc = I.default_cascade()
    W = I.draw_weights(casc, 8)
    fw, fh = size
    frame = I.make_frame(fw, fh, 21)
    thr = (-1e30, -1e30, -1e30)
    n = O.pyramid_layout(fw, fh, 12.0, 1.25).score_off[-1]
    assert (2048 < n <= 8192) if fw == 64 else n > 8192
    ctx = _ctx(casc, W, fw, fh, 20000)
    for iou, mn in ((0.3, 1), (0.7, 2)):
        ctx.set_params(12.0, 1.25, thr, merge_iou=iou, min_neighbors=mn)
        det = [d.as_dict() for d in ctx.detect(torch.from_numpy(frame).cuda(), 20000)]
        idx3, sc3 = ctx.get_survivors(3)
        assert len(idx3) == n
        bx, by, bs, _ = boxes_of(O.build_pyramid(frame, 12.0, 1.25), idx3)
        valid = [(int(idx3[p]), int(k)) for p, k in greedy_merge_check(bx, by, bs, sc3, idx3, iou=iou, min_neighbors=mn)]
        assert [(d["index"], d["neighbors"]) for d in det] == valid, (iou, mn)
        # and against the oracle's own merge of the same boxes and fp32 scores
        kept, nbs = O.merge(bx, by, bs, sc3, idx3.astype(np.int64), iou=iou, min_neighbors=mn)
        assert [(int(idx3[p]), int(k)) for p, k in zip(kept, nbs)] == valid
        print("   %d boxes -> %d detections at iou %.1f, min_neighbors %d" % (n, len(det), iou, mn), flush=True)
    ctx.close()


def test_detection_array_too_small_reports_overflow():
    import paper_1508_01292_amd as P
    torch = _torch()
    casc = I.default_cascade()
    W = I.draw_weights(casc, 1508)
    frame = I.make_frame(320, 240, 33)
    tr = O.detect(frame, casc, W, 60, 1.25)
    assert len(tr.det) > 3
    ctx = _ctx(casc, W, 320, 240)
    ctx.set_params(60, 1.25, tr.thr)
    with pytest.raises(P.CnncError) as e:
        ctx.detect(torch.from_numpy(frame).cuda(), cap=3)
    assert e.value.code == -3
    ctx.close()


def test_call_order_and_argument_errors():
    import paper_1508_01292_amd as P
    torch = _torch()
    casc = I.default_cascade()
    W = I.draw_weights(casc, 1)
    ctx = _ctx(casc, W, 128, 128, 1000)
    for call in (lambda: ctx.stage1_scoremap(), lambda: ctx.compact_survivors(1, 0.0), lambda: ctx.eval_stage(2),
                 lambda: ctx.merge_detections(), lambda: ctx.fetch_detections(), lambda: ctx.get_scoremap()):
        with pytest.raises(P.CnncError) as e:
            call()
        assert e.value.code == -5
    for call in (lambda: ctx.compact_survivors(4, 0.0), lambda: ctx.eval_stage(1), lambda: ctx.set_params(6, 1.25),
                 lambda: ctx.set_params(24, 1.0), lambda: ctx.compact_survivors(1, float("nan")),
                 lambda: ctx.build_pyramid(torch.zeros(200, 200, dtype=torch.uint8, device="cuda")),
                 lambda: ctx.build_pyramid(torch.zeros(8, 100, dtype=torch.uint8, device="cuda"))):
        with pytest.raises(P.CnncError) as e:
            call()
        assert e.value.code == -1
    ft = torch.from_numpy(I.make_frame(128, 100, 2)).cuda()
    ctx.set_params(24, 1.25)
    ctx.build_pyramid(ft)
    with pytest.raises(P.CnncError) as e:
        ctx.eval_stage(2)
    assert e.value.code == -5
    ctx.stage1_scoremap()
    with pytest.raises(P.CnncError) as e:
        ctx.compact_survivors(2, 0.0)
    assert e.value.code == -5
    ctx.close()
    # unsupported network shape
    bad = I.default_cascade()
    bad[0] = I.Stage(12, (I.Layer(I.CONV, 1, 4, 3, 1), I.Layer(I.POOL, 4, 4, 2, 0), I.Layer(I.CONV, 4, 6, 3, 1),
                          I.Layer(I.FC, 6, 1, 3, 0)))
    with pytest.raises(P.CnncError) as e:
        P.Context(bad, [np.zeros(bad[0].n_params, np.float32), W[1], W[2]], 128, 128, 100)
    assert e.value.code == -1


def test_layout_matches_oracle_for_all_workloads():
    casc = I.default_cascade()
    W = I.draw_weights(casc, 1)
    ctx = _ctx(casc, W, 3840, 2160, 1000)
    for c in I.CONFIGS[:4]:
        ctx.set_params(c["min_face"], c["scale_step"])
        lay = ctx.pyramid_layout(c["width"], c["height"])
        ref = O.pyramid_layout(c["width"], c["height"], c["min_face"], c["scale_step"])
        assert lay["lvl_w"] == ref.lvl_w and lay["lvl_h"] == ref.lvl_h and lay["scale"] == ref.scale
        assert lay["score_off"] == ref.score_off
    ctx.close()


def test_runs_are_deterministic_and_contexts_reusable():
    torch = _torch()
    casc = I.default_cascade()
    W = I.draw_weights(casc, 1508)
    ctx = _ctx(casc, W, 640, 480)
    f0 = I.make_frame(640, 480, 1)
    f1 = I.make_frame(320, 200, 2)
    thr = (0.5, -0.2, 0.0)
    ctx.set_params(60, 1.25, thr)
    a = run_gpu_steps(ctx, torch.from_numpy(f0).cuda(), thr)
    b = run_gpu_steps(ctx, torch.from_numpy(f1).cuda(), thr)      # other size in between: buffers re-laid out
    a2 = run_gpu_steps(ctx, torch.from_numpy(f0).cuda(), thr)
    for k in ("pyramid", "score1", "idx1", "score2", "idx2", "score3", "idx3"):
        assert np.array_equal(a[k], a2[k]), k
    assert a["det"] == a2["det"] and len(b["score1"]) != len(a["score1"])
    ctx.close()


def test_async_contexts_on_streams_match_synchronous_results():
    """Several frames in flight on separate streams (the paper's asynchronous mode maps to this):
    every frame's detections equal those of a synchronous call."""
    torch = _torch()
    casc = I.default_cascade()
    W = I.draw_weights(casc, I.config_seed(4))
    frames = [I.make_frame(480, 270, I.config_seed(4), i, None) for i in range(6)]
    thr = (0.6, -0.3, 0.0)
    sync = _ctx(casc, W, 480, 270)
    sync.set_params(60, 1.25, thr)
    dev = [torch.from_numpy(f).cuda() for f in frames]
    want = [[d.as_dict() for d in sync.detect(t, 8192)] for t in dev]
    sync.close()
    ctxs = [_ctx(casc, W, 480, 270) for _ in range(3)]
    streams = [torch.cuda.Stream() for _ in range(3)]
    for c in ctxs:
        c.set_params(60, 1.25, thr)
    torch.cuda.synchronize()
    got = [None] * len(frames)
    for base in range(0, len(frames), 3):
        for j in range(3):
            ctxs[j].detect_async(dev[base + j], streams[j])
        for j in range(3):
            got[base + j] = [d.as_dict() for d in ctxs[j].fetch_detections(8192)]
    assert got == want
    for c in ctxs:
        c.close()


def test_a_context_lets_go_of_the_callers_stream_once_it_has_waited_for_it():
    """A stream of the caller may be destroyed after a call that waits for it (fetch, merge, survivor count, the
    synchronous calls): the context refers to it no longer, so calls that wait for earlier work, a change of frame size
    and the end of the context all work afterwards."""
    import paper_1508_01292_amd as P
    torch = _torch()
    casc = I.default_cascade()
    W = I.draw_weights(casc, 3)
    frames = [I.make_frame(320, 240, 30 + k) for k in range(3)]
    ctx = _ctx(casc, W, 320, 240)
    ctx.set_params(24, 1.25, (0.4, -0.2, 0.0))
    dev = [torch.from_numpy(f).cuda() for f in frames]
    want = [[d.as_dict() for d in ctx.detect(t, 8192)] for t in dev]
    for rnd in range(2):
        for k, t in enumerate(dev):
            st = P.Stream()
            ctx.detect_async(t, st)
            got = [d.as_dict() for d in ctx.fetch_detections(8192)]
            st.close()
            assert st.cuda_stream == 0 and got == want[k]
        # step by step on a stream that is gone after the count was read
        st = P.Stream()
        ctx.build_pyramid(dev[0], st)
        ctx.stage1_scoremap(st)
        ctx.compact_survivors(1, 0.4, st)
        n1 = ctx.survivor_count(1, st)
        st.close()
        assert n1 > 0
        ctx.set_timing(True)
        ctx.get_timings()                                 # waits for "the last stream"
        ctx.set_timing(False)
        small = I.make_frame(200, 150, 5)                 # another frame size: buffers are rebuilt after a wait
        assert len(ctx.detect(torch.from_numpy(small).cuda(), 8192)) >= 0
        assert [d.as_dict() for d in ctx.detect(dev[1], 8192)] == want[1]
    st = P.Stream()
    ctx.detect_async(dev[2], st)
    assert [d.as_dict() for d in ctx.fetch_detections(8192)] == want[2]
    st.close()
    ctx.close()


def test_fhd_stream_three_survival_quantiles_async():
    """The 16-frame 1920x1080 stream (0..200 ellipses per frame), thresholds pooled over the stream at three
    stage-1 survival quantiles, frames in flight on three streams.  Every frame's detections are compared with
    the oracle's at the 0.5 % quantile (where the oracle finishes in seconds) and with the synchronous GPU
    path at all three; survivor counts per frame are compared with the oracle's at all three."""
    torch = _torch()
    casc = I.default_cascade()
    W = I.draw_weights(casc, I.config_seed(4))
    c = I.CONFIGS[4]
    frames = I.make_stream(4)
    assert len(frames) == 16
    print("case fhd stream", flush=True)
    pyrs = [O.build_pyramid(f, c["min_face"], c["scale_step"]) for f in frames]
    s1 = [O.stage1_scores(p, casc[0], W[0]) for p in pyrs]
    pooled = np.concatenate(s1)
    dev = [torch.from_numpy(f).cuda() for f in frames]
    ctxs = [_ctx(casc, W, c["width"], c["height"]) for _ in range(3)]
    streams = [torch.cuda.Stream() for _ in range(3)]
    sync = _ctx(casc, W, c["width"], c["height"])
    for q in (0.005, 0.02, 0.10):
        t1 = O.threshold_from_quantile(pooled, q)
        idx1 = [O.survivors(s, t1) for s in s1]
        assert sum(len(i) for i in idx1) == int(np.floor(q * pooled.size))
        if q == 0.005:
            s2 = [O.eval_stage(f, p, i, casc[1], W[1]) for f, p, i in zip(frames, pyrs, idx1)]
            t2 = O.threshold_from_quantile(np.concatenate(s2), 0.2)
        else:
            t2 = 0.0        # any fixed threshold: the later stages are checked against the synchronous path
        thr = (float(t1), float(t2), 0.0)
        sync.set_params(c["min_face"], c["scale_step"], thr)
        for cx in ctxs:
            cx.set_params(c["min_face"], c["scale_step"], thr)
        want = []
        for k, d in enumerate(dev):
            want.append([x.as_dict() for x in sync.detect(d, 8192)])
            g1, _ = sync.get_survivors(1)
            assert_survivors(g1, s1[k], np.arange(s1[k].size), t1, "stage-1 survivors, frame %d, q %g" % (k, q))
        got = [None] * 16
        for base in range(0, 18, 3):
            for j in range(3):
                if base + j < 16:
                    if base:
                        got[base + j - 3] = [x.as_dict() for x in ctxs[j].fetch_detections(8192)]
                    ctxs[j].detect_async(dev[base + j], streams[j])
        for k in range(13, 16):
            got[k] = [x.as_dict() for x in ctxs[k % 3].fetch_detections(8192)]
        assert got == want, "asynchronous detections differ from synchronous ones at q = %g" % q
        if q == 0.005:
            for k in (0, 5, 15):
                tr = O.detect(frames[k], casc, W, c["min_face"], c["scale_step"], thr=thr)
                key = lambda d: (d["x"], d["y"], d["size"], d["neighbors"], d["index"])
                assert [key(d) for d in got[k]] == [key(d) for d in tr.det], "frame %d" % k
    for cx in ctxs + [sync]:
        cx.close()


def test_uhd_headline_workload_full_oracle():
    """The 3840x2160, min-face-60 workload the throughput is quoted on, against the full oracle."""
    c = I.CONFIGS[2]
    casc = I.default_cascade()
    W = I.draw_weights(casc, I.config_seed(2))
    frame = I.make_frame(c["width"], c["height"], I.config_seed(2))
    tr, g, _ = _full_case(frame, casc, W, c["min_face"], c["scale_step"], name="uhd")
    assert tr.score1.size == 856540 and len(tr.idx1) == 17130 and len(tr.idx2) == 3426


def test_uhd_small_faces_full_oracle():
    """3840x2160 with 24-pixel faces (6.6 M windows, 131,773 / 26,354 survivors at the 2 % / 20 % quantiles of the
    oracle's scores): every intermediate of every step against the full oracle, merge included."""
    c = I.CONFIGS[3]
    casc = I.default_cascade()
    W = I.draw_weights(casc, I.config_seed(3))
    frame = I.make_frame(c["width"], c["height"], I.config_seed(3))
    tr, g, _ = _full_case(frame, casc, W, c["min_face"], c["scale_step"], name="uhd small faces", det_cap=32768)
    assert tr.score1.size == 6588676 and len(tr.idx1) == 131773 and len(tr.idx2) == 26354
    assert len(g["det"]) > 4096        # the long form of the merge (several chunks of sorted boxes)


def test_stage3_on_a_list_longer_than_its_hand_over_buffer():
    """Stage 3 works a long survivor list off in segments of 65,536 windows (the buffer between its convolution and its
    fully connected kernel holds that many): 131,773 windows reach it here, two full segments and a short one.  Scores
    around the segment boundaries and a random sample against the oracle; every window must have been written."""
    torch = _torch()
    c = I.CONFIGS[3]
    casc = I.default_cascade()
    W = I.draw_weights(casc, I.config_seed(3))
    frame = I.make_frame(c["width"], c["height"], I.config_seed(3))
    pyr = O.build_pyramid(frame, c["min_face"], c["scale_step"])
    t1 = O.threshold_from_quantile(O.stage1_scores(pyr, casc[0], W[0]), 0.02)
    ctx = _ctx(casc, W, 3840, 2160, 200000)
    thr = (float(t1), -1e30, 1e30)                    # everything passes stage 2, nothing passes stage 3
    ctx.set_params(c["min_face"], c["scale_step"], thr)
    ft = torch.from_numpy(frame).cuda()
    ctx.build_pyramid(ft)
    ctx.stage1_scoremap()
    ctx.compact_survivors(1, thr[0])
    ctx.eval_stage(2)
    ctx.compact_survivors(2, thr[1])
    idx2, _ = ctx.get_survivors(2)
    assert abs(len(idx2) - 131773) <= 3 and len(idx2) > 2 * 65536
    ctx.eval_stage(3)
    sc3 = ctx.get_stage_scores(3)
    assert sc3.size == len(idx2)
    rng = np.random.default_rng(5)
    pick = np.unique(np.concatenate([np.arange(0, 40), np.arange(65536 - 40, 65536 + 40), np.arange(131072 - 40, 131072 + 40),
                                     np.arange(len(idx2) - 40, len(idx2)), rng.choice(len(idx2), 400, replace=False)]))
    print("case long stage-3 list: %d windows, %d compared" % (len(idx2), pick.size), flush=True)
    assert_scores(sc3[pick], O.eval_stage(frame, pyr, idx2[pick], casc[2], W[2]), "stage-3 scores across segments")
    # a second pass over the same list gives the same bits (no window left unwritten or written twice differently)
    ctx.eval_stage(3)
    assert np.array_equal(ctx.get_stage_scores(3), sc3)
    ctx.close()


def test_compaction_of_a_very_long_score_map():
    """More than 4,096 compaction workgroups (8.4 M values): the form with a separate scan of the workgroup counts.
    The list must hold exactly the windows whose fp32 score exceeds the threshold, in ascending order, with their
    scores (a property of the GPU's own score map, whose values the other tests compare with the oracle)."""
    torch = _torch()
    casc = I.default_cascade()
    W = I.draw_weights(casc, 77)
    w, h = 4400, 2100
    frame = I.make_frame(w, h, 77)
    n = O.pyramid_layout(w, h, 12.0, 2.0).score_off[-1]
    assert n > 4096 * 2048
    print("case long score map: %d windows" % n, flush=True)
    ctx = _ctx(casc, W, w, h, 300000)
    ctx.set_params(12.0, 2.0, (0.0, 0.0, 0.0))
    ctx.build_pyramid(torch.from_numpy(frame).cuda())
    ctx.stage1_scoremap()
    s = ctx.get_scoremap()
    assert s.size == n
    thr = float(np.partition(s, n - 200000)[n - 200000])      # about 200,000 windows lie above it
    ctx.compact_survivors(1, thr)
    idx, sc = ctx.get_survivors(1)
    want = np.nonzero(s > np.float32(thr))[0]
    assert np.array_equal(idx, want) and np.array_equal(sc, s[want])
    # and the two-launch form on the same context: a later, shorter list
    ctx.eval_stage(2)
    s2 = ctx.get_stage_scores(2)
    t2 = float(np.median(s2))
    ctx.compact_survivors(2, t2)
    idx2, sc2 = ctx.get_survivors(2)
    keep = s2 > np.float32(t2)
    assert np.array_equal(idx2, idx[keep]) and np.array_equal(sc2, s2[keep])
    ctx.close()
