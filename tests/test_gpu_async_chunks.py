"""Asynchronous mode inside a frame (cnnc_set_async_chunks): stage 1 of a later chunk of pyramid levels overlaps the
later stages of earlier chunks on the context's own streams.  Survivor lists and detections must be exactly those of
the one-stream path, which the other tests compare with the oracle."""
import numpy as np
import pytest

import cnnc_inputs as I
from oracle import oracle as O

pytestmark = pytest.mark.gpu


def _lists(ctx):
    return [tuple(a.tolist() for a in ctx.get_survivors(s)) for s in (1, 2, 3)]


def _case(frame, min_face, step, quantiles, chunk_counts, seed, max_surv=200000, det_cap=32768, name=""):
    import torch

    import paper_1508_01292_amd as P
    casc = I.default_cascade()
    W = I.draw_weights(casc, seed)
    print("case async chunks", name, frame.shape, flush=True)
    tr = O.detect(frame, casc, W, min_face, step, quantiles=quantiles)
    ft = torch.from_numpy(frame).cuda()
    ctx = P.Context(casc, W, frame.shape[1], frame.shape[0], max_surv)
    ctx.set_params(min_face, step, tr.thr)
    want_det = [d.as_dict() for d in ctx.detect(ft, det_cap)]
    want_lists = _lists(ctx)
    key = lambda d: (d["x"], d["y"], d["size"], d["neighbors"], d["index"])
    if tr.det:
        assert len(want_det) == len(tr.det)
    stream = torch.cuda.Stream()
    for k in chunk_counts:
        ctx.set_async_chunks(k)
        for rep in range(2):                             # twice: the second frame re-uses events and lists
            ctx.detect_async(ft, stream if rep else None)
            got = [d.as_dict() for d in ctx.fetch_detections(det_cap)]
            assert got == want_det, "detections differ with %d chunks" % k
            assert _lists(ctx) == want_lists, "survivor lists differ with %d chunks" % k
    ctx.set_async_chunks(1)
    assert [d.as_dict() for d in ctx.detect(ft, det_cap)] == want_det
    ctx.close()
    return tr, want_det, key


def test_chunked_path_equals_one_stream_path_small_frames():
    c = I.CONFIGS[0]
    tr, det, key = _case(I.make_frame(c["width"], c["height"], I.config_seed(0)), c["min_face"], c["scale_step"], (0.02, 0.2),
                         (2, 3, 4, 8), I.config_seed(0), name="vga")
    assert [key(d) for d in det] == [key(d) for d in tr.det]
    # ragged sizes; more chunks asked for than the frame has levels
    _case(I.make_frame(333, 217, 9), 14.0, 1.3, (0.05, 0.3), (2, 5, 8), 21, name="ragged")
    _case(I.make_frame(70, 40, 3), 24.0, 1.25, (0.1, 0.5), (2, 8), 22, name="tiny, few levels")


def test_chunked_path_full_size_frames():
    for ci in (2, 3):
        c = I.CONFIGS[ci]
        tr, det, key = _case(I.make_frame(c["width"], c["height"], I.config_seed(ci)), c["min_face"], c["scale_step"], (0.02, 0.2),
                             (2, 4), I.config_seed(ci), name=c["name"])
        if ci == 2:       # (the small-face frame has near ties whose order may differ from the oracle's: compared elsewhere)
            assert [key(d) for d in det] == [key(d) for d in tr.det]


def test_chunked_path_degenerate_lists():
    """Nothing survives; everything survives and the lists overflow (the truncated lists are those of the one-stream path)."""
    import torch

    import paper_1508_01292_amd as P
    casc = I.default_cascade()
    W = I.draw_weights(casc, 4)
    frame = I.make_frame(96, 80, 12)
    ft = torch.from_numpy(frame).cuda()
    ctx = P.Context(casc, W, 96, 80, 300)
    for thr in ((1e30, 0.0, 0.0), (-1e30, 1e30, 0.0), (-1e30, -1e30, -1e30)):
        res = []
        for k in (1, 3):
            ctx.set_async_chunks(k)
            ctx.set_params(12.0, 1.5, thr)
            try:
                det = [d.as_dict() for d in ctx.detect(ft, 4096)]
                code = 0
            except P.CnncError as e:
                det, code = None, e.code
            cnt = []
            for s in (1, 2, 3):
                try:
                    cnt.append(ctx.survivor_count(s))
                except P.CnncError as e:
                    cnt.append(("overflow", e.code))
            res.append((code, det, cnt))
        assert res[0] == res[1], thr
    ctx.close()
