"""GPU parity of the fused stage 1 (score + threshold + survivor list without a score map): against the oracle's
survivor set, and bit for bit against the library's own two-call path."""
import numpy as np
import pytest

import cnnc_inputs as I
from oracle import oracle as O

from parity import assert_scores, assert_survivors

pytestmark = pytest.mark.gpu


def _case(frame, min_face, step, q, act=I.ACT_RATIONAL, seed=3, bias_sd=0.0, max_surv=200000, name=""):
    import torch
    import paper_1508_01292_amd as P
    print("fused stage-1 case", name, frame.shape, "q", q, flush=True)
    casc = I.default_cascade(act)
    W = I.draw_weights(casc, seed, bias_sd=bias_sd)
    pyr = O.build_pyramid(frame, min_face, step)
    s1 = O.stage1_scores(pyr, casc[0], W[0])
    thr = float(O.threshold_from_quantile(s1, q)) if q is not None else -1e30
    ctx = P.Context(casc, W, frame.shape[1], frame.shape[0], max_surv)
    ctx.set_params(min_face, step, (thr, 0.0, 0.0))
    ft = torch.from_numpy(frame).cuda()
    ctx.build_pyramid(ft)
    ctx.stage1_scoremap()
    ctx.compact_survivors(1, thr)
    n_a = ctx.survivor_count(1)
    idx_a, sc_a = ctx.get_survivors(1)
    ctx.build_pyramid(ft)
    ctx.stage1_survivors(thr)
    with pytest.raises(P.CnncError):
        ctx.get_scoremap()                       # the fused step leaves no score map
    n_b = ctx.survivor_count(1)
    idx_b, sc_b = ctx.get_survivors(1)
    assert n_a == n_b
    np.testing.assert_array_equal(idx_a, idx_b)
    np.testing.assert_array_equal(sc_a, sc_b)     # same kernel arithmetic: identical bits
    assert_survivors(idx_b, s1, np.arange(s1.size), thr, name)
    assert_scores(sc_b, s1[idx_b.astype(np.int64)], name)
    # stage 2 runs from the fused list
    ctx.eval_stage(2)
    sc2 = ctx.get_stage_scores(2)
    assert sc2.size == idx_b.size
    ctx.close()
    print("   %d windows, %d survivors" % (s1.size, idx_b.size), flush=True)
    return idx_b


def test_fused_stage1_vga_and_ragged():
    c = I.CONFIGS[0]
    idx = _case(I.make_frame(c["width"], c["height"], I.config_seed(0)), c["min_face"], c["scale_step"], 0.02, name="vga")
    assert idx.size == 473
    # ragged: level widths that are not multiples of 32, many small levels, biases, another activation
    _case(I.make_frame(333, 251, 5), 12.0, 1.3, 0.05, act=I.ACT_TANH, seed=5, bias_sd=0.1, name="333x251")
    _case(I.make_frame(97, 141, 6), 12.0, 1.1, 0.3, seed=6, name="97x141")
    _case(I.make_frame(12, 12, 6), 12.0, 1.5, None, seed=6, name="one window")


def test_fused_stage1_uhd_headline():
    c = I.CONFIGS[2]
    idx = _case(I.make_frame(c["width"], c["height"], I.config_seed(2)), c["min_face"], c["scale_step"], 0.02,
                seed=I.config_seed(2), name="uhd")
    assert idx.size == 17130


def test_fused_stage1_every_window_and_overflow():
    import torch
    import paper_1508_01292_amd as P
    frame = I.make_frame(160, 120, 9)
    casc = I.default_cascade()
    W = I.draw_weights(casc, 9)
    n = O.pyramid_layout(160, 120, 12.0, 1.25).score_off[-1]
    ctx = P.Context(casc, W, 160, 120, 1000)
    ctx.set_params(12.0, 1.25, (-1e30, 0.0, 0.0))
    ctx.build_pyramid(torch.from_numpy(frame).cuda())
    ctx.stage1_survivors(-1e30)                  # everything passes: the list overflows its capacity of 1000
    with pytest.raises(P.CnncError) as e:
        ctx.survivor_count(1)
    assert e.value.code == -3
    import ctypes as C
    from paper_1508_01292_amd.binding import _d2h
    pi, ps = C.c_void_p(0), C.c_void_p(0)
    P.lib().cnnc_get_survivors(ctx._h, C.c_int(1), C.byref(pi), C.byref(ps))
    np.testing.assert_array_equal(_d2h(pi.value, 4000, np.uint32), np.arange(1000, dtype=np.uint32))   # truncated, valid
    ctx.stage1_survivors(1e30)                   # nothing passes
    assert ctx.survivor_count(1) == 0
    with pytest.raises(P.CnncError):
        ctx.stage1_survivors(float("nan"))
    ctx.close()
    ctx2 = P.Context(casc, W, 160, 120, n + 10)
    ctx2.set_params(12.0, 1.25, (-1e30, 0.0, 0.0))
    with pytest.raises(P.CnncError):             # no pyramid yet
        ctx2.stage1_survivors(0.0)
    ctx2.build_pyramid(torch.from_numpy(frame).cuda())
    ctx2.stage1_survivors(-1e30)
    assert ctx2.survivor_count(1) == n
    idx, _ = ctx2.get_survivors(1)
    np.testing.assert_array_equal(idx, np.arange(n, dtype=np.uint32))
    ctx2.close()


def test_detect_with_fused_stage1_gives_the_same_detections():
    import torch
    import paper_1508_01292_amd as P
    c = I.CONFIGS[1]
    frame = I.make_frame(c["width"], c["height"], I.config_seed(1))
    casc = I.default_cascade()
    W = I.draw_weights(casc, I.config_seed(1))
    tr = O.detect(frame, casc, W, c["min_face"], c["scale_step"])
    ctx = P.Context(casc, W, c["width"], c["height"], 100000)
    ctx.set_params(c["min_face"], c["scale_step"], tr.thr)
    ft = torch.from_numpy(frame).cuda()
    a = [d.as_dict() for d in ctx.detect(ft, 8192)]
    ctx.set_fused_stage1(True)
    b = [d.as_dict() for d in ctx.detect(ft, 8192)]
    s = torch.cuda.Stream()
    ctx.detect_async(ft, s)
    b2 = [d.as_dict() for d in ctx.fetch_detections(8192)]
    assert a == b == b2 and len(a) > 0
    assert ctx.survivor_count(1) == len(tr.idx1) or abs(ctx.survivor_count(1) - len(tr.idx1)) <= 2
    ctx.close()
