"""Pins of the CPU oracle to things other than itself: the paper's printed constants and error
bound, closed forms, hand-computed windows, library routines (scipy / torch on the CPU in fp64),
brute force on tiny inputs and invariants.  A plausible mistake anywhere in the oracle (dropped
term, wrong sign or index, transposed operand) should fail at least one of these."""
import math
import os

import numpy as np
import pytest
import scipy.ndimage
import scipy.signal
import torch
import torch.nn.functional as F

import cnnc_inputs as I
from cnnc_inputs import CONV, FC, POOL, Layer, Stage
from oracle import oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


# ----------------------------------------------------------------------------------------------
# Activation: Section 3.1, eq. (1)
# ----------------------------------------------------------------------------------------------
def test_rational_tanh_error_bound_of_the_paper():
    """The paper states a relative error of at most 1.8 % on the whole axis."""
    ys = np.concatenate([np.linspace(1e-6, 20, 400001), np.logspace(-8, 3, 2001)])
    approx = np.array([O.rational_tanh(y) for y in ys])
    rel = np.abs(approx - np.tanh(ys)) / np.tanh(ys)
    worst = rel.max()
    assert 0.0170 < worst < 0.0180            # a wrong constant or a dropped term moves this far away
    assert 1.0 < ys[rel.argmax()] < 1.3
    # odd symmetry, zero, saturation
    assert O.rational_tanh(0.0) == 0.0
    for y in (0.1, 0.7, 3.0, 50.0):
        assert O.rational_tanh(-y) == -O.rational_tanh(y)
    assert abs(O.rational_tanh(1e6) - 1.0) < 1e-12


def test_rational_tanh_hand_values_and_scaling():
    rows = _golden_lines("activation_eq1.txt")
    const = {r[0]: float(r[1]) for r in rows if r[0] != "point"}
    for r in rows:
        if r[0] == "point":
            y, denom = float(r[1]), float(r[2])
            assert O.rational_tanh(y) == pytest.approx(1.0 - 1.0 / denom, abs=1e-15)
            x = y / const["slope"]
            assert O.activation(x, I.ACT_RATIONAL) == pytest.approx(const["scale"] * (1 - 1 / denom), abs=1e-14)
            assert O.activation(-x, I.ACT_RATIONAL) == pytest.approx(-const["scale"] * (1 - 1 / denom), abs=1e-14)
    for x in (-2.0, -0.3, 0.0, 0.4, 1.5):
        assert O.activation(x, I.ACT_SCALED_TANH) == pytest.approx(1.7159 * math.tanh(2 * x / 3), abs=1e-15)
        assert O.activation(x, I.ACT_TANH) == pytest.approx(math.tanh(x), abs=1e-15)
        assert O.activation(x, I.ACT_NONE) == x


# ----------------------------------------------------------------------------------------------
# Pyramid sizes and resampling special cases
# ----------------------------------------------------------------------------------------------
def test_pyramid_size_tables():
    for r in _golden_lines("pyramid_sizes.txt"):
        w, h, mf, step = int(r[0]), int(r[1]), float(r[2]), float(r[3])
        want = [tuple(int(v) for v in t.split("x")) for t in r[5:]]
        p = O.pyramid_layout(w, h, mf, step)
        assert list(zip(p.lvl_w, p.lvl_h)) == want
        assert p.scale[0] == mf / 12
        for a, b in zip(p.scale[:-1], p.scale[1:]):
            assert b == a * step


def test_pyramid_stops_below_window_and_rejects_bad_arguments():
    p = O.pyramid_layout(640, 480, 60, 1.25)
    assert min(p.lvl_w[-1], p.lvl_h[-1]) >= 12
    s_next = p.scale[-1] * 1.25
    assert min(math.floor(640 / s_next + 1e-9), math.floor(480 / s_next + 1e-9)) < 12
    assert O.pyramid_layout(11, 11, 12, 1.25).n_levels == 0
    with pytest.raises(ValueError):
        O.pyramid_layout(640, 480, 60, 1.0)
    with pytest.raises(ValueError):
        O.pyramid_layout(640, 480, 6, 1.25)


def test_resample_identity_box_and_point_sampling():
    rng = np.random.default_rng(7)
    f = rng.integers(0, 256, (41, 53), dtype=np.uint8)
    # scale 1: identity
    assert np.array_equal(O.resample_level(f, 1.0, 53, 41), f)
    # even integer scale: both weights are one half -> rounded mean of the central 2x2 block
    g = O.resample_level(f, 2.0, 26, 20)
    f32 = f.astype(np.uint32)
    want = (f32[0:40:2, 0:52:2] + f32[0:40:2, 1:52:2] + f32[1:40:2, 0:52:2] + f32[1:40:2, 1:52:2] + 2) >> 2
    assert np.array_equal(g, want.astype(np.uint8))
    g4 = O.resample_level(f, 4.0, 13, 10)
    want4 = (f32[1:40:4, 1:52:4] + f32[1:40:4, 2:52:4] + f32[2:40:4, 1:52:4] + f32[2:40:4, 2:52:4] + 2) >> 2
    assert np.array_equal(g4, want4.astype(np.uint8))
    # odd integer scale: the sample point is a pixel centre
    assert np.array_equal(O.resample_level(f, 5.0, 10, 8), f[2:40:5, 2:50:5])
    assert np.array_equal(O.resample_level(f, 3.0, 17, 13), f[1:39:3, 1:51:3])


def test_resample_against_library_bilinear():
    """Float bilinear interpolation (scipy) at the same sample points; the 8-bit weights and the
    final rounding bound the difference by one grey level.  Pins orientation and alignment."""
    rng = np.random.default_rng(8)
    f = scipy.ndimage.gaussian_filter(rng.standard_normal((90, 130)), 3.0)
    f = np.clip((f - f.min()) / (f.max() - f.min()) * 255, 0, 255).astype(np.uint8)
    for s, lw, lh in ((1.25, 104, 72), (2.44140625, 53, 36), (7.8125, 16, 11)):
        got = O.resample_level(f, s, lw, lh).astype(np.float64)
        yy = np.clip((np.arange(lh) + 0.5) * s - 0.5, 0, f.shape[0] - 1)
        xx = np.clip((np.arange(lw) + 0.5) * s - 0.5, 0, f.shape[1] - 1)
        ref = scipy.ndimage.map_coordinates(f.astype(np.float64), np.meshgrid(yy, xx, indexing="ij"),
                                            order=1, mode="nearest")
        assert np.abs(got - ref).max() <= 1.0
        assert np.abs(got - ref).mean() < 0.35


def test_resample_constant_and_ramp():
    f = np.full((60, 80), 77, np.uint8)
    assert np.all(O.resample_level(f, 1.7, 47, 35) == 77)
    ramp = np.tile(np.arange(100, dtype=np.uint8) * 2, (50, 1))     # value = 2x: bilinear is exact on it
    g = O.resample_level(ramp, 2.5, 40, 20).astype(np.float64)
    xx = np.clip((np.arange(40) + 0.5) * 2.5 - 0.5, 0, 99)
    assert np.abs(g - 2 * xx[None, :]).max() <= 0.5 + 2 * 2.5 / 512 + 1e-9
    assert np.array_equal(O.resample_level(ramp.T.copy(), 2.5, 20, 40), O.resample_level(ramp, 2.5, 40, 20).T)


# ----------------------------------------------------------------------------------------------
# Networks: closed forms, one-hot windows, library convolution
# ----------------------------------------------------------------------------------------------
def _rational_py(x):
    y = 2.0 * x / 3.0
    return math.copysign(1.7159 * (1 - 1 / (1 + abs(y) + y * y + 1.41645 * y ** 4)), y)


def test_closed_forms_on_constant_windows():
    rows = _golden_lines("closed_forms.txt")
    wts = {r[0]: [float(v) for v in r[1:]] for r in rows if r[0].startswith("stage")}
    fan = {1: [9, 36, 72], 2: [25, 72, 256, 32], 3: [25, 400, 288, 1568, 64]}
    acts = {"scaled_tanh": (I.ACT_SCALED_TANH, lambda v: 1.7159 * math.tanh(2 * v / 3)),
            "rational": (I.ACT_RATIONAL, _rational_py)}
    for r in rows:
        if r[0] not in acts:
            continue
        act, g = acts[r[0]]
        s, printed = int(r[1]), float(r[2])
        w = wts["stage%d" % s]
        a = 0.5
        for f_in, wj in zip(fan[s][:-1], w[:-1]):
            a = g(f_in * wj * a)
        closed = fan[s][-1] * w[-1] * a
        assert closed == pytest.approx(printed, abs=2e-9)
        casc = I.default_cascade(act)
        blobs = I.uniform_weights(casc, [wts["stage1"], wts["stage2"], wts["stage3"]])
        n = casc[s - 1].in_size
        got = O.net_forward(casc[s - 1], blobs[s - 1], np.full((n, n), 0.5))[0]
        # float32 storage of the weights moves the result by ~1e-8 relative
        assert got == pytest.approx(printed, abs=5e-7)


def _one_hot_blob(stage, picks):
    """picks[j] = (oc, ic, a, b) of the single weight set to 1 in the j-th weighted layer."""
    parts, j = [], 0
    for l in stage.layers:
        if l.kind == POOL:
            continue
        w = np.zeros((l.cout, l.cin, l.k, l.k), np.float32)
        w[picks[j]] = 1.0
        parts += [w.ravel(), np.zeros(l.cout, np.float32)]
        j += 1
    return np.concatenate(parts)


def test_hand_computed_one_hot_window_stage1():
    """With one weight per layer set to 1 the score is g(max over a 2x2 block of g(x)) for a pixel
    block that can be found by hand: conv1 tap (a,b) then pool cell (2i'+a'..) then conv2 tap (a2,b2)
    then fc tap (i,j).  Pins tap order, pooling alignment and the [c][y][x] feature order."""
    casc = I.default_cascade(I.ACT_SCALED_TANH)
    st = casc[0]
    g = lambda v: 1.7159 * math.tanh(2 * v / 3)
    win = (np.arange(144, dtype=np.float64).reshape(12, 12) * 3 % 97) / 97.0 - 0.4   # no symmetry
    for (c1, a, b), (c2, a2, b2), (i, j) in [((2, 0, 1), (5, 2, 0), (1, 2)), ((0, 2, 2), (7, 0, 1), (2, 0)),
                                              ((3, 1, 0), (1, 1, 2), (0, 1))]:
        blob = _one_hot_blob(st, [(c1, 0, a, b), (c2, c1, a2, b2), (0, c2, i, j)])
        # fc reads conv2 output (i,j); conv2 reads pooled cell (i+a2, j+b2); that pools conv1
        # outputs rows 2(i+a2)..+1, cols 2(j+b2)..+1; conv1 output (r,c) reads pixel (r+a, c+b)
        r0, q0 = 2 * (i + a2), 2 * (j + b2)
        block = [g(win[r + a, q + b]) for r in (r0, r0 + 1) for q in (q0, q0 + 1)]
        want = g(max(block))
        got = O.net_forward(st, blob, win)[0]
        assert got == pytest.approx(want, abs=1e-14)
        # a weight on another input channel of conv2 must read nothing (conv1 has one live channel)
        blob2 = _one_hot_blob(st, [(c1, 0, a, b), (c2, (c1 + 1) % 4, a2, b2), (0, c2, i, j)])
        assert O.net_forward(st, blob2, win)[0] == pytest.approx(0.0, abs=1e-15)


def _torch_act(x, act):
    if act == I.ACT_SCALED_TANH:
        return 1.7159 * torch.tanh(x * (2.0 / 3.0))
    if act == I.ACT_TANH:
        return torch.tanh(x)
    if act == I.ACT_RATIONAL:
        y = x * (2.0 / 3.0)
        return 1.7159 * torch.sign(y) * (1 - 1 / (1 + y.abs() + y * y + 1.41645 * y ** 4))
    return x


def _torch_forward(stage, blob, x, dilated=False):
    """The network with torch's CPU conv2d / max_pool2d in fp64 (library routines)."""
    x = torch.as_tensor(x, dtype=torch.float64)[None, None]
    off, d = 0, 1
    for l in stage.layers:
        if l.kind == POOL:
            if dilated:
                x = F.max_pool2d(x, 2, stride=1, dilation=d)
                d *= 2
            else:
                x = F.max_pool2d(x, 2, stride=2)
        else:
            w = torch.as_tensor(blob[off:off + l.n_weights].astype(np.float64)).reshape(l.cout, l.cin, l.k, l.k)
            b = torch.as_tensor(blob[off + l.n_weights:off + l.n_params].astype(np.float64))
            off += l.n_params
            x = _torch_act(F.conv2d(x, w, b, dilation=d), l.act)
    return x[0].numpy()


@pytest.mark.parametrize("act", [I.ACT_RATIONAL, I.ACT_SCALED_TANH, I.ACT_TANH])
def test_networks_against_torch_cpu_fp64(act):
    casc = I.default_cascade(act)
    blobs = I.draw_weights(casc, 99, bias_sd=0.3)
    rng = np.random.default_rng(5)
    for st, blob in zip(casc, blobs):
        for _ in range(3):
            win = rng.uniform(-1, 1, (st.in_size, st.in_size))
            want = _torch_forward(st, blob, win).ravel()
            got = O.net_forward(st, blob, win)
            assert np.allclose(got, want, rtol=0, atol=1e-12)


def test_single_conv_layer_is_scipy_valid_correlation():
    rng = np.random.default_rng(11)
    st = Stage(9, (Layer(CONV, 1, 3, 4, I.ACT_NONE),))
    blob = np.concatenate([rng.standard_normal(48), [0.25, -0.5, 1.0]]).astype(np.float32)
    win = rng.standard_normal((9, 9))
    # the last layer's whole map is returned channel-major; the oracle returns cout*6*6 values
    import ctypes as C
    out = np.zeros(3 * 36)
    rc = O.lib().orc_net_forward(O._layers(st), C.c_int(1), O._p(blob), C.c_int(9), O._p(np.ascontiguousarray(win)),
                                 O._p(out))
    assert rc == 0
    for oc in range(3):
        ker = blob[oc * 16:(oc + 1) * 16].astype(np.float64).reshape(4, 4)
        want = scipy.signal.correlate(win, ker, mode="valid") + float(blob[48 + oc])
        assert np.allclose(out.reshape(3, 6, 6)[oc], want, atol=1e-13)


def test_net_forward_rejects_misfit_layers():
    st = Stage(12, (Layer(CONV, 1, 4, 3, 1), Layer(POOL, 4, 4, 2, 0), Layer(CONV, 4, 8, 3, 1), Layer(FC, 8, 1, 2, 0)))
    with pytest.raises(ValueError):
        O.net_forward(st, np.zeros(st.n_params, np.float32), np.zeros((12, 12)))


# ----------------------------------------------------------------------------------------------
# Stage 1: definition vs dense form, equivariance
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("act", [I.ACT_RATIONAL, I.ACT_SCALED_TANH, I.ACT_TANH])
def test_dense_form_equals_per_window_definition(act):
    casc = I.default_cascade(act)
    blob = I.draw_weights(casc, 3, bias_sd=0.2)[0]
    rng = np.random.default_rng(12)
    for shape in ((20, 23), (12, 12), (13, 31), (27, 12)):
        lvl = rng.integers(0, 256, shape, dtype=np.uint8)
        a = O.stage1_level(lvl, casc[0], blob, "windows")
        b = O.stage1_level(lvl, casc[0], blob, "dense")
        assert a.shape == (shape[0] - 11, shape[1] - 11)
        assert np.abs(a - b).max() < 1e-13
        # and each window by the library stack
        for (y, x) in ((0, 0), (a.shape[0] - 1, a.shape[1] - 1), (a.shape[0] // 2, a.shape[1] // 3)):
            win = (lvl[y:y + 12, x:x + 12].astype(np.float64) - 128) / 128
            assert a[y, x] == pytest.approx(float(_torch_forward(casc[0], blob, win).ravel()[0]), abs=1e-12)


def test_dense_form_equals_torch_dilated_stack_for_deeper_nets():
    """The dense routine is general; run it on the stage-2 shape (two pools -> tap spacing 4)."""
    casc = I.default_cascade(I.ACT_SCALED_TANH)
    blob = I.draw_weights(casc, 4, bias_sd=0.1)[1]
    lvl = np.random.default_rng(13).integers(0, 256, (31, 37), dtype=np.uint8)
    got = O.stage1_level(lvl, casc[1], blob, "dense")
    want = _torch_forward(casc[1], blob, (lvl.astype(np.float64) - 128) / 128, dilated=True)[0]
    assert got.shape == want.shape == (8, 14)
    assert np.abs(got - want).max() < 1e-12
    assert np.abs(got - O.stage1_level(lvl, casc[1], blob, "windows")).max() < 1e-12


def test_translation_equivariance_on_a_level_and_through_the_pyramid():
    casc = I.default_cascade()
    blob = I.draw_weights(casc, 1508)[0]
    rng = np.random.default_rng(14)
    big = rng.integers(0, 256, (60, 70), dtype=np.uint8)
    a = O.stage1_level(big[:40, :50], casc[0], blob)
    b = O.stage1_level(big[3:43, 7:57], casc[0], blob)
    full = O.stage1_level(big, casc[0], blob)
    assert np.array_equal(a, full[:29, :39]) and np.array_equal(b, full[3:32, 7:46])
    # pyramid: level 0 of the default workloads has scale 5 -> a 5-pixel frame shift is a 1-pixel level shift
    f = I.make_frame(400, 300, 21)
    p0 = O.build_pyramid(f[:250, :350], 60, 1.25)
    p1 = O.build_pyramid(f[10:260, 15:365], 60, 1.25)
    assert p0.lvl_w[0] == 70 and p0.lvl_h[0] == 50
    assert np.array_equal(p0.levels[0][2:, 3:], p1.levels[0][:-2, :-3])


# ----------------------------------------------------------------------------------------------
# Thresholds and survivors
# ----------------------------------------------------------------------------------------------
def test_survivors_strict_fp32_and_monotone():
    s = np.array([0.5, 0.25, 0.75, 0.25 + 1e-12, -1.0, 0.75])
    assert O.survivors(s, 0.25).tolist() == [0, 2, 5]          # 0.25+1e-12 rounds to 0.25 in fp32: not above
    assert O.survivors(s, -2.0).tolist() == [0, 1, 2, 3, 4, 5]
    assert O.survivors(s, 0.75).tolist() == []
    rng = np.random.default_rng(15)
    sc = rng.standard_normal(5000)
    prev = None
    for t in np.linspace(-3, 3, 25):
        cur = set(O.survivors(sc, t).tolist())
        assert cur == set(np.nonzero(sc.astype(np.float32) > np.float32(t))[0].tolist())
        if prev is not None:
            assert cur <= prev
        prev = cur


def test_quantile_threshold_lets_exactly_k_through():
    rng = np.random.default_rng(16)
    sc = rng.standard_normal(23659)
    for q in (0.005, 0.02, 0.1, 0.2):
        t = O.threshold_from_quantile(sc, q)
        assert len(O.survivors(sc, t)) == int(np.floor(q * sc.size))
    assert len(O.survivors(sc, O.threshold_from_quantile(sc, 0.0))) == 0
    assert len(O.survivors(sc, O.threshold_from_quantile(sc, 1.0))) == sc.size


def test_flat_index_decoding():
    p = O.pyramid_layout(640, 480, 60, 1.25)
    off = p.score_off
    assert off[-1] == 23659 and off[1] == 117 * 85
    lvl, y, x = p.decode(np.array([0, 116, 117, off[1] - 1, off[1], off[-1] - 1]))
    assert lvl.tolist() == [0, 0, 0, 0, 1, 9]
    assert y.tolist() == [0, 0, 1, 84, 0, 0]
    assert x.tolist() == [0, 116, 0, 116, 0, 5]


# ----------------------------------------------------------------------------------------------
# Crops
# ----------------------------------------------------------------------------------------------
def test_crop_exact_special_cases():
    rng = np.random.default_rng(17)
    f = rng.integers(0, 256, (200, 260), dtype=np.uint8)
    norm = lambda v: (v - 128.0) / 128.0
    # scale 2, 24 samples over 24 frame pixels: sample points are pixel centres -> the frame patch itself
    c = O.crop(f, 7, 5, 2.0, 24)
    assert np.array_equal(c, norm(f[10:34, 14:38].astype(np.float64)))
    # scale 4, 48 samples over 48 pixels
    c = O.crop(f, 3, 2, 4.0, 48)
    assert np.array_equal(c, norm(f[8:56, 12:60].astype(np.float64)))
    # scale 4, 24 samples over 48 pixels: each sample sits between two pixels in x and y -> 2x2 mean
    c = O.crop(f, 3, 2, 4.0, 24)
    p = f[8:56, 12:60].astype(np.float64)
    want = (p[0::2, 0::2] + p[0::2, 1::2] + p[1::2, 0::2] + p[1::2, 1::2]) / 4
    assert np.array_equal(c, norm(want))


def test_crop_against_library_bilinear_and_clamping():
    rng = np.random.default_rng(18)
    f = scipy.ndimage.gaussian_filter(rng.standard_normal((300, 400)), 4.0)
    f = np.clip((f - f.min()) / (f.max() - f.min()) * 255, 0, 255).astype(np.uint8)
    for (x, y, s, n) in ((10, 4, 5.0, 24), (3, 9, 7.8125, 48), (0, 0, 9.765625, 24), (21, 12, 12.20703125, 48)):
        got = O.crop(f, x, y, s, n) * 128 + 128
        pos = lambda o, lim: np.clip(o * s + (np.arange(n) + 0.5) * 12 * s / n - 0.5, 0, lim - 1)
        ref = scipy.ndimage.map_coordinates(f.astype(np.float64), np.meshgrid(pos(y, 300), pos(x, 400), indexing="ij"),
                                            order=1, mode="nearest")
        assert np.abs(got - ref).max() < 1.0
    # a window whose rectangle pokes past the right/bottom edge only repeats the edge pixels
    edge = O.crop(f, 21, 13, 12.20703125, 24)
    assert np.isfinite(edge).all() and edge.min() >= -1 and edge.max() <= 127 / 128


# ----------------------------------------------------------------------------------------------
# Boxes and merging
# ----------------------------------------------------------------------------------------------
def test_window_boxes():
    p = O.pyramid_layout(640, 480, 60, 1.25)
    off = p.score_off
    bx, by, bs = O.window_boxes(p, np.array([0, 118, off[2] + 3]))
    assert (bx.tolist(), by.tolist(), bs.tolist()) == ([0, 5, 23], [0, 5, 0], [60, 60, 94])   # 3*7.8125=23.4; 12*7.8125=93.75


def test_merge_special_cases():
    # disjoint boxes: all kept, ordered by score, no neighbours
    bx, by, bs = np.array([0, 100, 200, 300]), np.array([0, 0, 0, 0]), np.array([50, 50, 50, 50])
    kept, nb = O.merge(bx, by, bs, [0.1, 0.9, 0.5, 0.7], [0, 1, 2, 3])
    assert kept.tolist() == [1, 3, 2, 0] and nb.tolist() == [0, 0, 0, 0]
    # identical boxes: the best survives with n-1 neighbours; equal scores resolve by the order key
    kept, nb = O.merge([5] * 6, [7] * 6, [40] * 6, [0.3, 0.8, 0.8, 0.1, 0.8, 0.2], [9, 4, 2, 8, 3, 1])
    assert kept.tolist() == [2] and nb.tolist() == [5]
    # min_neighbors drops lonely boxes
    kept, nb = O.merge([0, 0, 500], [0, 2, 0], [60, 60, 60], [0.9, 0.8, 0.7], [0, 1, 2], min_neighbors=2)
    assert kept.tolist() == [0] and nb.tolist() == [1]
    assert O.merge([], [], [], [], [])[0].tolist() == []


def test_merge_iou_is_strict_and_greedy_not_transitive():
    # 10x10 boxes shifted by dx: inter = 10(10-dx), union = 200 - inter
    # dx=5: 50/150 = 0.333 > 0.3 suppressed; dx=6: 40/160 = 0.25 kept
    kept, nb = O.merge([0, 5], [0, 0], [10, 10], [0.9, 0.8], [0, 1])
    assert kept.tolist() == [0] and nb.tolist() == [1]
    kept, nb = O.merge([0, 6], [0, 0], [10, 10], [0.9, 0.8], [0, 1])
    assert kept.tolist() == [0, 1]
    # exactly 0.3 with a power-of-two threshold stand-in: iou = 0.25 exactly, threshold 0.25 -> not suppressed
    kept, _ = O.merge([0, 6], [0, 0], [10, 10], [0.9, 0.8], [0, 1], iou=0.25)
    assert kept.tolist() == [0, 1]
    # chain A-B-C: A suppresses B, B would have suppressed C but is dead, so C is kept
    kept, nb = O.merge([0, 5, 10], [0, 0, 0], [10, 10, 10], [0.9, 0.8, 0.7], [0, 1, 2])
    assert kept.tolist() == [0, 2] and nb.tolist() == [1, 0]
    # brute force on random boxes: re-run the greedy rule with python ints and exact fractions
    from fractions import Fraction
    rng = np.random.default_rng(19)
    n = 60
    bx, by = rng.integers(0, 200, n), rng.integers(0, 200, n)
    bs, sc = rng.integers(20, 90, n), rng.standard_normal(n).astype(np.float32)
    order = rng.permutation(n)
    kept, nb = O.merge(bx, by, bs, sc, order, iou=0.3)
    thr = Fraction(float(np.float32(0.3)))
    seq = sorted(range(n), key=lambda i: (-float(sc[i]), int(order[i])))
    dead, want, want_nb = set(), [], []
    for a_pos, a in enumerate(seq):
        if a in dead:
            continue
        cnt = 0
        for b in seq[a_pos + 1:]:
            if b in dead:
                continue
            iw = min(bx[a] + bs[a], bx[b] + bs[b]) - max(bx[a], bx[b])
            ih = min(by[a] + bs[a], by[b] + bs[b]) - max(by[a], by[b])
            if iw > 0 and ih > 0:
                inter = int(iw) * int(ih)
                uni = int(bs[a]) ** 2 + int(bs[b]) ** 2 - inter
                if Fraction(inter) > thr * uni:
                    dead.add(b)
                    cnt += 1
        want.append(a)
        want_nb.append(cnt)
    assert kept.tolist() == want and nb.tolist() == want_nb


# ----------------------------------------------------------------------------------------------
# The whole cascade on a small frame: bookkeeping between the stages
# ----------------------------------------------------------------------------------------------
def test_cascade_bookkeeping_small_frame():
    casc = I.default_cascade()
    W = I.draw_weights(casc, 1508)
    f = I.make_frame(320, 240, 33)
    tr = O.detect(f, casc, W, 60, 1.25)
    n1 = len(tr.score1)
    assert n1 == tr.pyramid.score_off[-1]
    assert len(tr.idx1) == int(0.02 * n1) and len(tr.idx2) == int(0.2 * len(tr.idx1))
    assert set(tr.idx2) <= set(tr.idx1) and set(tr.idx3) <= set(tr.idx2)
    assert np.all(np.diff(tr.idx1) > 0) and np.all(np.diff(tr.idx2) > 0)
    # stage-2 score of a survivor = the network on its crop, by the library stack
    lvl, ys, xs = tr.pyramid.decode(tr.idx1[:5])
    for i in range(5):
        c = O.crop(f, xs[i], ys[i], tr.pyramid.scale[lvl[i]], 24)
        assert tr.score2[i] == pytest.approx(float(_torch_forward(casc[1], W[1], c).ravel()[0]), abs=1e-12)
    # detections are a subset of the stage-3 survivors, in descending score order
    sc = [d["score"] for d in tr.det]
    assert sc == sorted(sc, reverse=True)
    assert sum(d["neighbors"] + 1 for d in tr.det) == len(tr.idx3)
    # the per-window form gives the same survivors on this frame
    tr2 = O.detect(f, casc, W, 60, 1.25, form="windows")
    assert np.array_equal(tr.idx1, tr2.idx1) and np.array_equal(tr.idx3, tr2.idx3)


def test_numpy_merge_check_agrees_with_oracle_merge():
    """The test-side greedy merge used as a validity check in the GPU tests is itself checked here."""
    from parity import boxes_of, greedy_merge_check
    rng = np.random.default_rng(23)
    for n in (1, 40, 300):
        bx, by = rng.integers(0, 300, n), rng.integers(0, 300, n)
        bs, sc = rng.integers(20, 120, n), rng.standard_normal(n).astype(np.float32)
        sc[n // 2:] = sc[:n - n // 2]                       # exact ties
        order = rng.permutation(n)
        for mn in (1, 2):
            kept, nb = O.merge(bx, by, bs, sc, order, 0.3, mn)
            assert [(int(p), int(k)) for p, k in zip(kept, nb)] == greedy_merge_check(bx, by, bs, sc, order, 0.3, mn)
    p = O.pyramid_layout(640, 480, 60, 1.25)
    idx = rng.integers(0, p.score_off[-1], 200)
    a = O.window_boxes(p, idx)
    b = boxes_of(p, idx)
    assert all(np.array_equal(u, v) for u, v in zip(a, b[:3]))
