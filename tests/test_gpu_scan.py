"""GPU parity of the first stage in the paper's geometry (27 x 31 window, 4 pixel step): the HIP scan, called
through the C ABI, against the oracle's single pass and per-window definition, response by response."""
import numpy as np
import pytest

import cnnc_inputs as I
from oracle import oracle as O

from parity import ATOL, RTOL

pytestmark = pytest.mark.gpu


def _scan_case(frame, min_face, step, act, seed, bias_sd=0.0, name=""):
    import torch
    import paper_1508_01292_amd as P
    print("scan case", name, frame.shape, "min_face", min_face, "step", step, "act", act, flush=True)
    casc = I.default_cascade()
    ctx = P.Context(casc, I.draw_weights(casc, seed), frame.shape[1], frame.shape[0], 1024)
    ctx.set_params(min_face, step, (0.0, 0.0, 0.0))
    net = I.paper_stage1(act)
    blob = I.draw_scan_weights(net, seed, bias_sd=bias_sd)
    ctx.scan_set_weights(blob, act)
    ctx.build_pyramid(torch.from_numpy(frame).cuda())
    pyr = O.build_pyramid(frame, min_face, step)
    want = O.scan_scores(pyr, net, blob)
    # both builds of the kernel (a workgroup per 8 x 8 and per 16 x 16 responses), then the one chosen from the frame
    maps = {}
    for side in (8, 16, 0):
        ctx.scan_set_tile(side)
        ctx.scan_scoremap()
        assert ctx.scan_tile() == (side or ctx.scan_tile()) and ctx.scan_tile() in (8, 16)
        maps[side] = ctx.get_scan_scoremap()
        assert maps[side].size == want.size
        e = np.abs(maps[side].astype(np.float64) - want)
        assert np.all(e <= ATOL + RTOL * np.abs(want)), "tile side %d: max err %g" % (side, e.max())
    assert np.array_equal(maps[8], maps[16]), "a response is summed in the same order whatever the tile"
    got = maps[0]
    lay = ctx.scan_layout(frame.shape[1], frame.shape[0])
    sizes = [(max(0, (l.shape[0] - 31) // 4 + 1), max(0, (l.shape[1] - 27) // 4 + 1)) if min(l.shape[0] - 31, l.shape[1] - 27) >= 0
             else (0, 0) for l in pyr.levels]
    assert lay["n_levels"] == len(pyr.levels)
    assert [(int(h), int(w)) for h, w in zip(lay["out_h"], lay["out_w"])] == [s if s[0] * s[1] else (0, 0) for s in sizes]
    assert int(lay["out_off"][-1]) == want.size == got.size
    err = np.abs(got.astype(np.float64) - want)
    assert np.all(err <= ATOL + RTOL * np.abs(want)), "max err %g" % err.max()
    ctx.close()
    print("   %d responses on %d levels, max abs err %.2e" % (want.size, sum(1 for s in sizes if s[0] * s[1]), err.max() if want.size else 0),
          flush=True)
    return got, want, pyr, net, blob


@pytest.mark.parametrize("act", [I.ACT_RATIONAL, I.ACT_SCALED_TANH, I.ACT_TANH])
def test_scan_vga_every_activation(act):
    c = I.CONFIGS[0]
    frame = I.make_frame(c["width"], c["height"], I.config_seed(0))
    got, want, pyr, net, blob = _scan_case(frame, c["min_face"], c["scale_step"], act, I.config_seed(0),
                                            bias_sd=0.0 if act == I.ACT_RATIONAL else 0.2, name="vga")
    assert want.size > 600
    # a few responses against the per-window definition (the oracle's other form)
    lvl = pyr.levels[1]
    w_def = O.scan_level(lvl, net, blob, "windows")
    off = ((pyr.levels[0].shape[0] - 31) // 4 + 1) * ((pyr.levels[0].shape[1] - 27) // 4 + 1)
    np.testing.assert_allclose(got[off:off + w_def.size], w_def.ravel(), rtol=RTOL, atol=ATOL)


def test_scan_ragged_sizes_several_tiles():
    # level sizes that are not 3 mod 4, tiles cut at both edges, levels below the window at the end
    for (w, h, mf, st, seed) in ((333, 251, 12.0, 1.3, 5), (97, 141, 12.0, 1.1, 6), (641, 363, 24.0, 1.25, 7)):
        frame = I.make_frame(w, h, seed)
        _scan_case(frame, mf, st, I.ACT_RATIONAL, seed, bias_sd=0.1, name="ragged %dx%d" % (w, h))


def test_scan_uhd_headline_frame():
    c = I.CONFIGS[2]
    frame = I.make_frame(c["width"], c["height"], I.config_seed(2))
    got, want, *_ = _scan_case(frame, c["min_face"], c["scale_step"], I.ACT_RATIONAL, I.config_seed(2), name="uhd")
    assert want.size > 40000
    import paper_1508_01292_amd as P           # a frame of this size is scanned in 16 x 16 tiles, a small one in 8 x 8
    casc = I.default_cascade()
    ctx = P.Context(casc, I.draw_weights(casc, 2), c["width"], c["height"], 1024)
    import torch
    for cfg, side in ((c, 16), (I.CONFIGS[0], 8)):
        ctx.set_params(cfg["min_face"], cfg["scale_step"], (0.0, 0.0, 0.0))
        ctx.scan_set_weights(I.draw_scan_weights(I.paper_stage1(), 2), 1)
        ctx.build_pyramid(torch.from_numpy(I.make_frame(cfg["width"], cfg["height"], 2)).cuda())
        ctx.scan_scoremap()
        assert ctx.scan_tile() == side
    ctx.close()


def test_scan_degenerate_and_call_order():
    import torch
    import paper_1508_01292_amd as P
    casc = I.default_cascade()
    ctx = P.Context(casc, I.draw_weights(casc, 1), 64, 64, 64)
    ctx.set_params(12.0, 1.25, (0.0, 0.0, 0.0))
    net = I.paper_stage1()
    blob = I.draw_scan_weights(net, 1)
    with pytest.raises(P.CnncError):                 # no weights yet
        ctx.scan_scoremap()
    with pytest.raises(P.CnncError):                 # wrong blob size
        ctx.scan_set_weights(blob[:-1], 1)
    with pytest.raises(P.CnncError):                 # activation kind
        ctx.scan_set_weights(blob, 0)
    ctx.scan_set_weights(blob, 1)
    with pytest.raises(P.CnncError):                 # tile side
        ctx.scan_set_tile(12)
    assert ctx.scan_tile() == 0
    with pytest.raises(P.CnncError):                 # no pyramid yet
        ctx.scan_scoremap()
    with pytest.raises(P.CnncError):                 # no map yet
        ctx.get_scan_scoremap()
    # a frame whose every level is smaller than the window: an empty map, no launch
    small = I.make_frame(26, 40, 3)
    ctx.build_pyramid(torch.from_numpy(small).cuda())
    ctx.scan_scoremap()
    assert ctx.get_scan_scoremap().size == 0
    # exactly one window
    one = I.make_frame(27, 31, 4)
    ctx.build_pyramid(torch.from_numpy(one).cuda())
    ctx.scan_scoremap()
    got = ctx.get_scan_scoremap()
    assert got.size == 1
    win = (one.astype(np.float64) - 128) / 128
    assert abs(float(got[0]) - O.scan_window(net, blob, win)) <= ATOL
    ctx.scan_set_tile(16)
    ctx.scan_scoremap()
    assert np.array_equal(ctx.get_scan_scoremap(), got)
    ctx.scan_set_tile(0)
    # the same context still runs the cascade's own stage 1 on that pyramid
    ctx.stage1_scoremap()
    assert ctx.get_scoremap().size == O.pyramid_layout(27, 31, 12.0, 1.25).score_off[-1]
    ctx.close()
