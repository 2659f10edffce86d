"""GPU tests of stage 1 with its weights as instruction literals: the build of the kernel whose literals the host
overwrites with a context's weight set gives the same bits as the kernel that reads the weights from memory, for
every activation, on ragged sizes, for the score map and for the fused survivor form; the scores are compared with
the oracle as well.  Contexts with equal weights share a module, contexts with other weights get their own, and a
module outlives the other contexts that used it."""
import numpy as np
import pytest

import cnnc_inputs as I
from oracle import oracle as O

from parity import assert_scores

pytestmark = pytest.mark.gpu


def _scoremap(ctx, ft):
    ctx.build_pyramid(ft)
    ctx.stage1_scoremap()
    return ctx.get_scoremap()


@pytest.mark.parametrize("act", [I.ACT_RATIONAL, I.ACT_SCALED_TANH, I.ACT_TANH])
def test_literal_build_equals_memory_build_and_oracle(act):
    import torch
    import paper_1508_01292_amd as P
    for (w, h, mf, step, seed, bias_sd) in ((640, 480, 24.0, 1.25, 11, 0.0), (333, 257, 20.0, 1.31, 12, 0.5), (97, 61, 12.0, 1.5, 13, 1.0)):
        print("literal weights: act", act, (w, h), flush=True)
        frame = I.make_frame(w, h, seed)
        casc = I.default_cascade(act)
        W = I.draw_weights(casc, seed, bias_sd=bias_sd)
        ctx = P.Context(casc, W, w, h, 100000)
        ctx.set_params(mf, step, (0.0, 0.0, 0.0))
        assert ctx.literal_weights(), "the literal build of stage 1 did not load"
        ft = torch.from_numpy(frame).cuda()
        lit = _scoremap(ctx, ft)
        ctx.set_literal_weights(False)
        assert not ctx.literal_weights()
        mem = _scoremap(ctx, ft)
        np.testing.assert_array_equal(lit, mem)
        pyr = O.build_pyramid(frame, mf, step)
        assert_scores(lit, O.stage1_scores(pyr, casc[0], W[0]), "stage 1, literal weights")
        # the fused survivor form in both builds
        thr = float(np.sort(mem)[-max(1, mem.size // 50)])
        lists = []
        for on in (True, False):
            ctx.set_literal_weights(on)
            ctx.build_pyramid(ft)
            ctx.stage1_survivors(thr)
            lists.append(ctx.get_survivors(1))
        np.testing.assert_array_equal(lists[0][0], lists[1][0])
        np.testing.assert_array_equal(lists[0][1], lists[1][1])
        assert len(lists[0][0]) == int((mem > np.float32(thr)).sum())
        ctx.close()


def test_modules_are_per_weight_set_and_outlive_other_contexts():
    import torch
    import paper_1508_01292_amd as P
    frame = I.make_frame(320, 240, 5)
    ft = torch.from_numpy(frame).cuda()
    casc = I.default_cascade()
    Wa, Wb = I.draw_weights(casc, 1), I.draw_weights(casc, 2)
    pyr = O.build_pyramid(frame, 24.0, 1.25)
    want_a, want_b = O.stage1_scores(pyr, casc[0], Wa[0]), O.stage1_scores(pyr, casc[0], Wb[0])
    a1 = P.Context(casc, Wa, 320, 240, 1000)
    a2 = P.Context(casc, Wa, 320, 240, 1000)          # same weights: the same module
    b = P.Context(casc, Wb, 320, 240, 1000)
    for c in (a1, a2, b):
        c.set_params(24.0, 1.25, (0.0, 0.0, 0.0))
        assert c.literal_weights()
    assert_scores(_scoremap(a1, ft), want_a, "a1")
    assert_scores(_scoremap(b, ft), want_b, "b")
    a1.close()                                         # a2 still holds the module of these weights
    assert_scores(_scoremap(a2, ft), want_a, "a2 after a1 closed")
    assert_scores(_scoremap(b, ft), want_b, "b again")
    a2.close()
    a3 = P.Context(casc, Wa, 320, 240, 1000)           # the module is built again
    a3.set_params(24.0, 1.25, (0.0, 0.0, 0.0))
    assert_scores(_scoremap(a3, ft), want_a, "a3")
    a3.close()
    b.close()


@pytest.mark.parametrize("act", [I.ACT_RATIONAL, I.ACT_SCALED_TANH, I.ACT_TANH])
def test_scan_literal_build_equals_memory_build(act):
    """The first stage in the paper's geometry: both builds give the same bits (the memory build is compared with the
    oracle in tests/test_gpu_scan.py; the literal build is the default there too)."""
    import torch
    import paper_1508_01292_amd as P
    for (w, h, mf, step, seed) in ((640, 480, 24.0, 1.25, 21), (301, 263, 16.0, 1.4, 22)):
        frame = I.make_frame(w, h, seed)
        casc = I.default_cascade()
        net = I.paper_stage1(act)
        ws = I.draw_scan_weights(net, seed, bias_sd=0.3)
        ctx = P.Context(casc, I.draw_weights(casc, seed), w, h, 1000)
        ctx.set_params(mf, step, (0.0, 0.0, 0.0))
        ctx.scan_set_weights(ws, act)
        ft = torch.from_numpy(frame).cuda()
        ctx.build_pyramid(ft)
        for side in (16, 8):                                   # both tile shapes of the kernel have both builds
            ctx.scan_set_tile(side)
            ctx.set_literal_weights(True)
            ctx.scan_scoremap()
            lit = ctx.get_scan_scoremap().copy()
            ctx.set_literal_weights(False)
            ctx.scan_scoremap()
            mem = ctx.get_scan_scoremap().copy()
            np.testing.assert_array_equal(lit, mem)
        ctx.scan_set_tile(0)
        ref = O.scan_scores(O.build_pyramid(frame, mf, step), net, ws)
        assert_scores(lit, ref, "scan, literal weights")
        # another weight set on the same context replaces the module
        ws2 = I.draw_scan_weights(net, seed + 100)
        ctx.set_literal_weights(True)
        ctx.scan_set_weights(ws2, act)
        ctx.scan_scoremap()
        assert_scores(ctx.get_scan_scoremap(), O.scan_scores(O.build_pyramid(frame, mf, step), net, ws2), "scan, second weight set")
        ctx.close()


@pytest.mark.parametrize("act", [I.ACT_RATIONAL, I.ACT_SCALED_TANH, I.ACT_TANH])
def test_select_literal_build_equals_memory_build(act):
    """The selective unit: records and both response maps of every listed region are the same bits in both builds (the
    comparison with the oracle is tests/test_gpu_select.py, which runs the literal build by default)."""
    import torch
    import paper_1508_01292_amd as P
    frame = I.make_frame(481, 363, 31)
    casc = I.default_cascade()
    n1, n2, n3 = I.paper_stage1(act), I.paper_stage2(act), I.paper_stage3(act)
    w1, w2, w3 = (I.draw_scan_weights(n, 40 + k, bias_sd=0.2) for k, n in enumerate((n1, n2, n3)))
    ctx = P.Context(casc, I.draw_weights(casc, 4), 481, 363, 20000)
    ctx.set_params(20.0, 1.3, (0.0, 0.0, 0.0))
    ctx.scan_set_weights(w1, act)
    ctx.select_set_weights(w2, w3, act)
    ft = torch.from_numpy(frame).cuda()
    ctx.build_pyramid(ft)
    ctx.scan_scoremap()
    s = ctx.get_scan_scoremap()
    t1 = float(np.sort(s)[-max(2, s.size // 20)])
    out = []
    for on in (True, False):
        ctx.set_literal_weights(on)
        ctx.select_run(t1, 0.0, 0.0, 3)
        recs, m2, m3 = ctx.select_fetch(20000, maps=True)
        out.append(([(r.index, r.k2, r.k3, r.face) for r in recs], m2.copy(), m3.copy()))
    assert len(out[0][0]) > 50 and out[0][0] == out[1][0]
    np.testing.assert_array_equal(out[0][1], out[1][1])
    np.testing.assert_array_equal(out[0][2], out[1][2])
    ctx.close()
