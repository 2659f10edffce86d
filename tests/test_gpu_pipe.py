"""GPU tests of the frame ingest ring (cnnc_pipe): host frames in, detections out.  Every frame's detections are
compared with the oracle's and with the library's own single-context path, with and without captured graphs; each
slot's graph is replayed several times on different frames with eager work of other slots in between."""
import numpy as np
import pytest

import cnnc_inputs as I
from oracle import oracle as O

pytestmark = pytest.mark.gpu


def _stream_case():
    ci = 4                                            # the 16-frame 1920x1080 stream
    cfg = I.CONFIGS[ci]
    frames = I.make_stream(ci)[:8]
    casc = I.default_cascade()
    W = I.draw_weights(casc, I.config_seed(ci))
    # thresholds at the quantiles of the first frame; the other frames simply use them
    tr0 = O.detect(frames[0], casc, W, cfg["min_face"], cfg["scale_step"])
    return cfg, frames, casc, W, tr0


@pytest.mark.parametrize("use_graph", [False, True])
def test_pipe_matches_single_context_and_oracle(use_graph):
    import torch
    import paper_1508_01292_amd as P
    cfg, frames, casc, W, tr0 = _stream_case()
    w, h = cfg["width"], cfg["height"]
    ctx = P.Context(casc, W, w, h, 100000)
    ctx.set_params(cfg["min_face"], cfg["scale_step"], tr0.thr)
    want = [[d.as_dict() for d in ctx.detect(torch.from_numpy(f).cuda(), 8192)] for f in frames]
    assert [(d["index"], d["neighbors"]) for d in want[0]] == [(d["index"], d["neighbors"]) for d in tr0.det]
    # one more frame straight against the oracle, at the same thresholds
    tr5 = O.detect(frames[5], casc, W, cfg["min_face"], cfg["scale_step"], thr=tr0.thr)
    assert [(d["index"], d["neighbors"]) for d in want[5]] == [(d["index"], d["neighbors"]) for d in tr5.det]

    # four slots on three lanes: a frame is always copied in ahead and meets every lane in turn
    pipe = P.Pipe(casc, W, w, h, 100000, depth=4, use_graph=use_graph)
    pipe.set_params(cfg["min_face"], cfg["scale_step"], tr0.thr)
    print("pipe graph=%s: 4 slots, 3 passes over %d frames" % (use_graph, len(frames)), flush=True)
    got = {}
    tickets = []
    order = list(range(len(frames))) + list(reversed(range(len(frames)))) + list(range(len(frames)))
    for k, fi in enumerate(order):
        if len(tickets) == 4:
            t, f0 = tickets.pop(0)
            got.setdefault(f0, []).append([d.as_dict() for d in pipe.fetch(t, 8192)])
        if k % 2:
            buf = pipe.frame_buffer()                 # producer writes in place
            buf[:] = frames[fi]
            tickets.append((pipe.submit(), fi))
        else:
            tickets.append((pipe.submit(frames[fi]), fi))
        if k % 5 == 0:                                # eager work of another context between the replays
            ctx.detect(torch.from_numpy(frames[(fi + 1) % len(frames)]).cuda(), 8192)
            torch.cuda.synchronize()
    for t, f0 in tickets:
        got.setdefault(f0, []).append([d.as_dict() for d in pipe.fetch(t, 8192)])
    for fi in range(len(frames)):
        assert len(got[fi]) == 3
        for rep in got[fi]:
            assert rep == want[fi], "frame %d" % fi
    pipe.close()
    ctx.close()


def test_pipe_errors_and_parameter_change():
    import paper_1508_01292_amd as P
    casc = I.default_cascade()
    W = I.draw_weights(casc, 2)
    frame = I.make_frame(320, 240, 2)
    tr = O.detect(frame, casc, W, 24.0, 1.25)
    with pytest.raises(P.CnncError):
        P.Pipe(casc, W, 320, 240, 1000, depth=0)
    with pytest.raises(P.CnncError):
        P.Pipe(casc, W, 320, 240, 1000, depth=17)
    pipe = P.Pipe(casc, W, 320, 240, 20000, depth=2, use_graph=True)
    pipe.set_params(24.0, 1.25, tr.thr)
    with pytest.raises(ValueError):
        pipe.submit(frame[:-1])
    t0 = pipe.submit(frame)
    t1 = pipe.submit(frame)
    with pytest.raises(P.CnncError) as e:             # ring full
        pipe.submit(frame)
    assert e.value.code == -5
    with pytest.raises(P.CnncError) as e:
        pipe.frame_buffer()
    assert e.value.code == -5
    with pytest.raises(P.CnncError) as e:             # parameters while frames are in flight
        pipe.set_params(24.0, 1.25, tr.thr)
    assert e.value.code == -5
    with pytest.raises(P.CnncError) as e:             # unknown ticket
        pipe.fetch(99)
    assert e.value.code == -1
    a = [d.as_dict() for d in pipe.fetch(t1)]         # any order
    t2 = pipe.submit(frame)                           # the slot freed out of order takes the next frame at once
    b = [d.as_dict() for d in pipe.fetch(t0)]
    assert [d.as_dict() for d in pipe.fetch(t2)] == a
    assert a == b and [(d["index"], d["neighbors"]) for d in a] == [(d["index"], d["neighbors"]) for d in tr.det]
    with pytest.raises(P.CnncError):                  # already fetched
        pipe.fetch(t0)
    # graphs captured so far are dropped when the thresholds change; results follow the new parameters
    for _ in range(4):
        assert [d.as_dict() for d in pipe.fetch(pipe.submit(frame))] == a
    tr2 = O.detect(frame, casc, W, 24.0, 1.25, quantiles=(0.05, 0.5))
    pipe.set_params(24.0, 1.25, tr2.thr)
    for _ in range(4):
        got = [d.as_dict() for d in pipe.fetch(pipe.submit(frame))]
        assert [(d["index"], d["neighbors"]) for d in got] == [(d["index"], d["neighbors"]) for d in tr2.det]
    # a detection array that is too small reports the overflow and the slot is free again
    with pytest.raises(P.CnncError) as e:
        pipe.fetch(pipe.submit(frame), cap=1)
    assert e.value.code == -3
    assert len(pipe.fetch(pipe.submit(frame))) == len(tr2.det)
    pipe.close()


@pytest.mark.parametrize("use_graph", [False, True])
def test_pipe_more_slots_than_lanes_fetched_in_any_order(use_graph):
    """Five slots on three lanes: two frames wait for a lane.  Asking for a waiting frame first sets the results of
    running ones aside; they are handed out later, unchanged."""
    import torch
    import paper_1508_01292_amd as P
    casc = I.default_cascade()
    W = I.draw_weights(casc, 9)
    frames = [I.make_frame(320, 240, 90 + k) for k in range(5)]
    tr = O.detect(frames[0], casc, W, 24.0, 1.25)
    ctx = P.Context(casc, W, 320, 240, 20000)
    ctx.set_params(24.0, 1.25, tr.thr)
    want = [[d.as_dict() for d in ctx.detect(torch.from_numpy(f).cuda(), 8192)] for f in frames]
    assert [(d["index"], d["neighbors"]) for d in want[0]] == [(d["index"], d["neighbors"]) for d in tr.det]
    assert len({len(x) for x in want}) > 1, "the frames must be told apart by their results"
    pipe = P.Pipe(casc, W, 320, 240, 20000, depth=5, use_graph=use_graph)
    pipe.set_params(24.0, 1.25, tr.thr)
    for rnd, fetch_order in enumerate(([4, 0, 3, 1, 2], [3, 4, 2, 1, 0], [0, 1, 2, 3, 4], [2, 4, 0, 1, 3])):
        t = [pipe.submit(f) for f in frames]
        with pytest.raises(P.CnncError) as e:         # ring full
            pipe.submit(frames[0])
        assert e.value.code == -5
        for k in fetch_order:
            assert [d.as_dict() for d in pipe.fetch(t[k], 8192)] == want[k], "round %d frame %d" % (rnd, k)
        with pytest.raises(P.CnncError):              # all fetched
            pipe.fetch(t[0])
    # frames that are on the device already go through the same ring without a copy (graphs by frame address and lane),
    # mixed with frames from host memory
    import torch
    dev = [torch.from_numpy(f).cuda() for f in frames]
    wide = torch.zeros((240, 384), dtype=torch.uint8, device="cuda")       # a frame with a row pitch of its own
    wide[:, :320] = dev[1]
    torch.cuda.synchronize()
    for rnd in range(3):
        t = [pipe.submit_device(dev[0]), pipe.submit(frames[3]), pipe.submit_device(wide[:, :320]), pipe.submit_device(dev[2]),
             pipe.submit_device(dev[0])]
        for k, fi in ((3, 2), (0, 0), (4, 0), (1, 3), (2, 1)):
            assert [d.as_dict() for d in pipe.fetch(t[k], 8192)] == want[fi], "device frames, round %d ticket %d" % (rnd, k)
    with pytest.raises(ValueError):
        pipe.submit_device(dev[0][:-1])
    with pytest.raises(ValueError):
        pipe.submit_device(dev[0].cpu())
    # a set-aside frame keeps its overflow rule: too small an array at fetch time reports it, and the slot is free again
    t = [pipe.submit(f) for f in frames]
    assert [d.as_dict() for d in pipe.fetch(t[4], 8192)] == want[4]
    with pytest.raises(P.CnncError) as e:
        pipe.fetch(t[0], cap=1)
    assert e.value.code == -3
    for k in (1, 2, 3):
        assert [d.as_dict() for d in pipe.fetch(t[k], 8192)] == want[k]
    assert [d.as_dict() for d in pipe.fetch(pipe.submit(frames[2]), 8192)] == want[2]
    pipe.close()
    ctx.close()


@pytest.mark.parametrize("use_graph", [False, True])
def test_pipe_in_the_paper_geometry(use_graph):
    """The ring driving the path in the paper's geometry (scan, selective unit, merge): every frame's detections equal
    those of cnnc_detect_paper on a single context (which tests/test_gpu_select.py compares with the oracle), and the
    first frame's are compared with the oracle's here as well."""
    import torch
    import paper_1508_01292_amd as P
    ci = 4
    cfg = I.CONFIGS[ci]
    frames = I.make_stream(ci)[:6]
    w, h = cfg["width"], cfg["height"]
    act, t_nn = I.ACT_RATIONAL, 6
    n1, n2, n3 = I.paper_stage1(act), I.paper_stage2(act), I.paper_stage3(act)
    w1, w2, w3 = (I.draw_scan_weights(n, 77 + k) for k, n in enumerate((n1, n2, n3)))
    # thresholds from the oracle on the first frame: 2 % of the scan, a quarter of the responses
    pyr = O.build_pyramid(frames[0], cfg["min_face"], cfg["scale_step"])
    s1 = O.scan_scores(pyr, n1, w1)
    t1 = float(O.threshold_from_quantile(s1, 0.02))
    idx = np.nonzero(s1.astype(np.float32) > np.float32(t1))[0]
    ref = O.select_unit(frames[0], pyr, idx, n1, n2, w2, n3, w3, -1e30, -1e30, 1)
    t2 = float(np.float32(np.quantile(np.concatenate([r["r2"].ravel() for r in ref]), 0.75)))
    t3 = float(np.float32(np.quantile(np.concatenate([r["r3"].ravel() for r in ref]), 0.75)))
    ref = O.select_unit(frames[0], pyr, idx, n1, n2, w2, n3, w3, t2, t3, t_nn)

    casc = I.default_cascade()
    W = I.draw_weights(casc, 5)
    ctx = P.Context(casc, W, w, h, 50000)
    ctx.set_params(cfg["min_face"], cfg["scale_step"], (0.0, 0.0, 0.0))
    ctx.scan_set_weights(w1, act)
    ctx.select_set_weights(w2, w3, act)
    want = [[d.as_dict() for d in ctx.detect_paper(torch.from_numpy(f).cuda(), t1, t2, t3, t_nn, 0.3, 1, cap=20000)] for f in frames]
    assert all(len(x) > 0 for x in want)
    # first frame against the oracle, unless a response sits inside the tolerance band of a threshold
    near = np.any(np.abs(s1 - t1) <= 2e-4) or any(np.any(np.abs(r["r2"] - t2) <= 2e-4) or np.any(np.abs(r["r3"] - t3) <= 2e-4) for r in ref)
    omerge = O.select_merge(pyr, ref, n1, 0.3, 1)
    same = [(d["index"], d["neighbors"], d["x"], d["y"], d["w"], d["h"]) for d in want[0]] == \
        [(d["index"], d["neighbors"], d["x"], d["y"], d["w"], d["h"]) for d in omerge]
    print("paper pipe graph=%s: %d detections on frame 0, equal to the oracle's: %s (a response in a band: %s)"
          % (use_graph, len(want[0]), same, bool(near)), flush=True)
    assert same or near

    pipe = P.Pipe(casc, W, w, h, 50000, depth=3, use_graph=use_graph)
    pipe.set_params(cfg["min_face"], cfg["scale_step"], (0.0, 0.0, 0.0))
    with pytest.raises(P.CnncError) as e:
        pipe.fetch_paper(0)                           # not in paper mode yet
    assert e.value.code == -5
    pipe.set_paper(w1, w2, w3, t1, t2, t3, t_nn, 0.3, 1)
    got, tickets = {}, []
    order = list(range(len(frames))) + list(reversed(range(len(frames)))) + list(range(len(frames)))
    for k, fi in enumerate(order):
        if len(tickets) == 3:
            t, f0 = tickets.pop(0)
            got.setdefault(f0, []).append([d.as_dict() for d in pipe.fetch_paper(t, 20000)])
        tickets.append((pipe.submit(frames[fi]), fi))
        if k == 4:
            with pytest.raises(P.CnncError) as e:
                pipe.fetch(tickets[0][0])             # the cascade's fetch on a paper-geometry pipe
            assert e.value.code == -5
            with pytest.raises(P.CnncError) as e:
                pipe.set_paper(w1, w2, w3, t1, t2, t3, t_nn)      # frames in flight
            assert e.value.code == -5
        if k % 5 == 0:                                # eager work of another context between the replays
            ctx.detect_paper(torch.from_numpy(frames[(fi + 1) % len(frames)]).cuda(), t1, t2, t3, t_nn, 0.3, 1, cap=20000)
    for t, f0 in tickets:
        got.setdefault(f0, []).append([d.as_dict() for d in pipe.fetch_paper(t, 20000)])
    for fi in range(len(frames)):
        assert len(got[fi]) == 3
        for rep in got[fi]:
            assert rep == want[fi], "frame %d" % fi
    pipe.close()
    ctx.close()
