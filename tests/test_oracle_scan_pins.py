"""Pins of the oracle's first stage in the paper's geometry (27 x 31 window, 4 pixel step, no fully
connected layer: paper, Sections 3.1 and 3.3) against things other than itself: torch's CPU conv2d /
max_pool2d in fp64, a hand-computed one-hot window, the per-window definition against the single pass
over the level, and translation by one step.  No GPU."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import cnnc_inputs as I
from cnnc_inputs import CONV, POOL
from oracle import oracle as O


def _torch_scan(net, blob, x):
    """The layer list with library routines on a whole image (fp64); returns the response map."""
    x = torch.as_tensor(x, dtype=torch.float64)[None, None]
    off = 0
    for l in net.layers:
        if l.kind == POOL:
            x = F.max_pool2d(x, 2, 2)
        else:
            w = torch.as_tensor(blob[off:off + l.n_weights].astype(np.float64)).reshape(l.cout, l.cin, l.kh, l.kw)
            b = torch.as_tensor(blob[off + l.n_weights:off + l.n_params].astype(np.float64))
            off += l.n_params
            x = F.conv2d(x, w, b)
            if l.act == I.ACT_TANH:
                x = torch.tanh(x)
            elif l.act == I.ACT_SCALED_TANH:
                x = 1.7159 * torch.tanh(x * (2.0 / 3.0))
            elif l.act != I.ACT_NONE:
                raise AssertionError("library pin uses the exact tanh forms only")
    return x[0, 0].numpy()


def test_shapes_of_the_chosen_network():
    net = I.paper_stage1()
    assert (net.win_w, net.win_h, net.step) == (27, 31, 4)
    assert net.n_params == 806                       # the paper states 797: see the module's note
    assert [l.kind for l in net.layers] == [CONV, POOL, CONV, POOL, CONV]   # no fully connected layer
    w, h = net.win_w, net.win_h
    for l in net.layers:
        if l.kind == POOL:
            assert w % 2 == 0 and h % 2 == 0
            w, h = w // 2, h // 2
        else:
            w, h = w - l.kw + 1, h - l.kh + 1
    assert (w, h) == (1, 1)


@pytest.mark.parametrize("act", [I.ACT_SCALED_TANH, I.ACT_TANH])
def test_window_and_level_against_torch_cpu_fp64(act):
    net = I.paper_stage1(act)
    blob = I.draw_scan_weights(net, 11, bias_sd=0.2)
    rng = np.random.default_rng(5)
    win = rng.uniform(-1, 1, (net.win_h, net.win_w))
    assert O.scan_window(net, blob, win) == pytest.approx(float(_torch_scan(net, blob, win)[0, 0]), abs=1e-12)
    lvl = rng.integers(0, 256, (53, 62), dtype=np.uint8)          # neither side is 3 mod 4: margins are dropped
    want = _torch_scan(net, blob, (lvl.astype(np.float64) - 128) / 128)
    for form in ("fcn", "windows"):
        got = O.scan_level(lvl, net, blob, form)
        assert got.shape == ((53 - 31) // 4 + 1, (62 - 27) // 4 + 1) == want.shape
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("act", [I.ACT_RATIONAL, I.ACT_TANH])
def test_single_pass_equals_per_window_definition(act):
    net = I.paper_stage1(act)
    blob = I.draw_scan_weights(net, 3, bias_sd=0.1)
    rng = np.random.default_rng(9)
    for (h, w) in ((31, 27), (34, 30), (35, 31), (44, 41)):
        lvl = rng.integers(0, 256, (h, w), dtype=np.uint8)
        a, b = O.scan_level(lvl, net, blob, "fcn"), O.scan_level(lvl, net, blob, "windows")
        assert a.shape == ((h - 31) // 4 + 1, (w - 27) // 4 + 1)
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)
        # and the definition itself: cut one window by hand
        j, i = a.shape[0] - 1, a.shape[1] - 1
        win = (lvl[4 * j:4 * j + 31, 4 * i:4 * i + 27].astype(np.float64) - 128) / 128
        assert b[j, i] == pytest.approx(O.scan_window(net, blob, win), abs=1e-15)
    assert O.scan_level(np.zeros((30, 40), np.uint8), net, blob).size == 0      # smaller than the window


def test_hand_computed_one_hot_window():
    """One-hot filters make the response f(f(max of one 4 x 4 pixel block)): with conv1 = delta at tap
    (a, b), conv2 = delta at (channel 0, a', b') into map k, conv3 = delta at (k, row i, column j),
    the block starts at row 4 i + 2 a' + a, column 4 j + 2 b' + b (f is monotone, pools are maxima)."""
    net = I.paper_stage1(I.ACT_RATIONAL)
    (a, b), (a2, b2), (k, i, j) = (1, 3), (2, 0), (7, 5, 2)
    l1, _, l2, _, l3 = net.layers
    w1 = np.zeros((l1.cout, 1, l1.kh, l1.kw), np.float32); w1[0, 0, a, b] = 1
    w2 = np.zeros((l2.cout, l2.cin, l2.kh, l2.kw), np.float32); w2[k, 0, a2, b2] = 1
    w3 = np.zeros((1, l3.cin, l3.kh, l3.kw), np.float32); w3[0, k, i, j] = 1
    blob = np.concatenate([w1.ravel(), np.zeros(l1.cout, np.float32), w2.ravel(), np.zeros(l2.cout, np.float32),
                           w3.ravel(), np.zeros(1, np.float32)])
    assert blob.size == net.n_params
    # a window whose values grow along rows, then columns: the block's maximum is its bottom right pixel
    yy, xx = np.mgrid[0:31, 0:27]
    win = (yy * 27 + xx) / 1000.0 - 0.3
    r0, c0 = 4 * i + 2 * a2 + a, 4 * j + 2 * b2 + b
    inner = win[r0 + 3, c0 + 3]
    want = O.activation(O.activation(inner, I.ACT_RATIONAL), I.ACT_RATIONAL)
    assert O.scan_window(net, blob, win) == pytest.approx(want, abs=1e-15)
    # the mirrored ramp puts the maximum in the block's top left pixel
    want2 = O.activation(O.activation(-win[r0, c0], I.ACT_RATIONAL), I.ACT_RATIONAL)
    assert O.scan_window(net, blob, -win) == pytest.approx(want2, abs=1e-15)


def test_translation_by_one_step():
    net = I.paper_stage1()
    blob = I.draw_scan_weights(net, 21)
    rng = np.random.default_rng(2)
    big = rng.integers(0, 256, (80, 90), dtype=np.uint8)
    a = O.scan_level(big[:, :], net, blob)
    b = O.scan_level(big[8:, 4:], net, blob)                      # two steps down, one step right
    np.testing.assert_array_equal(a[2:, 1:], b[:a.shape[0] - 2, :a.shape[1] - 1])


def test_scan_scores_of_a_pyramid_are_flat_level_row_column():
    net = I.paper_stage1()
    blob = I.draw_scan_weights(net, 1)
    frame = I.make_frame(320, 240, 77)
    pyr = O.build_pyramid(frame, 60, 1.25)
    flat = O.scan_scores(pyr, net, blob)
    sizes = [((l.shape[0] - 31) // 4 + 1) * ((l.shape[1] - 27) // 4 + 1) if l.shape[0] >= 31 and l.shape[1] >= 27 else 0
             for l in pyr.levels]
    assert flat.size == sum(sizes) and sizes[0] > 0 and sizes[-1] == 0
    np.testing.assert_array_equal(flat[:sizes[0]], O.scan_level(pyr.levels[0], net, blob).ravel())
