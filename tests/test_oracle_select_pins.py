"""Pins of the oracle's selective unit in the paper's geometry (Section 3.3: region with neighbourhood scaled to
51 x 55, histogram equalisation, mirror image, 5 x 5 response maps of CNN_2 / CNN_3, the counts K_nn and decision
rule (2)) against closed forms, library routines and the rule's truth table.  No GPU."""
import numpy as np
import pytest
import scipy.ndimage
import torch

import cnnc_inputs as I
from oracle import oracle as O
from test_oracle_scan_pins import _torch_scan


def test_region_exact_special_cases():
    rng = np.random.default_rng(1)
    f = rng.integers(0, 256, (90, 120), dtype=np.uint8)
    # scale 1: the region is the pixels themselves; outside the frame the edge is repeated
    np.testing.assert_array_equal(O.region(f, 7, 5, 1.0, 51, 55), f[5:60, 7:58])
    pad = np.pad(f, 60, mode="edge")
    np.testing.assert_array_equal(O.region(f, -12, -12, 1.0, 51, 55), pad[48:103, 48:99])
    np.testing.assert_array_equal(O.region(f, 100, 70, 1.0, 51, 55), pad[130:185, 160:211])
    # scale 2: every sample is the rounded mean of a 2 x 2 block
    big = rng.integers(0, 256, (200, 200), dtype=np.uint8).astype(np.int64)
    got = O.region(big.astype(np.uint8), 3, 4, 2.0, 51, 55)
    blk = big[8:8 + 110, 6:6 + 102]
    want = (blk[0::2, 0::2] + blk[0::2, 1::2] + blk[1::2, 0::2] + blk[1::2, 1::2] + 2) // 4
    np.testing.assert_array_equal(got, want)
    # a constant frame stays constant at any scale
    assert np.all(O.region(np.full((50, 60), 77, np.uint8), -5, 9, 1.37, 51, 55) == 77)


def test_region_against_library_bilinear():
    rng = np.random.default_rng(2)
    f = scipy.ndimage.gaussian_filter(rng.uniform(0, 255, (300, 400)), 3).astype(np.uint8)
    s, x0, y0 = 1.7, 20, -6
    got = O.region(f, x0, y0, s, 51, 55).astype(np.float64)
    ys = np.clip((y0 + np.arange(55) + 0.5) * s - 0.5, 0, 299)
    xs = np.clip((x0 + np.arange(51) + 0.5) * s - 0.5, 0, 399)
    want = scipy.ndimage.map_coordinates(f.astype(np.float64), np.meshgrid(ys, xs, indexing="ij"), order=1, mode="nearest")
    assert np.abs(got - want).max() <= 1.0          # 8-bit weights and rounding to uint8


def test_histogram_equalisation_closed_forms():
    # two values: the smaller goes to 0, the larger to 255
    a = np.array([10] * 100 + [200] * 50, np.uint8)
    np.testing.assert_array_equal(O.histeq(a), np.array([0] * 100 + [255] * 50, np.uint8))
    # three values with counts 1000, 1200, 605 (n = 2805): middle -> round(1200 * 255 / 1805) = round(169.53) = 170
    b = np.array([3] * 1000 + [90] * 1200 + [91] * 605, np.uint8)
    np.testing.assert_array_equal(np.unique(O.histeq(b)), [0, 170, 255])
    # 255 levels, eleven pixels each (n = 2805): v -> round(11 v * 255 / 2794)
    c = np.repeat(np.arange(255, dtype=np.uint8), 11)
    e = O.histeq(c)
    assert e[0] == 0 and e[-1] == 255 and e[11 * 127] == 128 and e[11 * 100] == 100 and e[11 * 200] == 201
    # rounding ties go up: counts 1, 1, 254 -> middle value maps to 255 / 255 ... use n - c0 = 2: 0.5 * 255 = 127.5 -> 128
    d = np.array([5, 9, 30], np.uint8)
    np.testing.assert_array_equal(O.histeq(d), [0, 128, 255])
    # a constant region is left alone; the map is monotone and order preserving
    np.testing.assert_array_equal(O.histeq(np.full(2805, 42, np.uint8)), np.full(2805, 42, np.uint8))
    rng = np.random.default_rng(3)
    r = rng.integers(40, 180, 2805).astype(np.uint8)
    q = O.histeq(r)
    order = np.argsort(r, kind="stable")
    assert np.all(np.diff(q[order].astype(int)) >= 0) and q.min() == 0 and q.max() == 255
    # the result has a nearly flat cumulative histogram: cdf of the output at level v is about v / 255
    cdf = np.cumsum(np.bincount(q, minlength=256)) / q.size
    assert np.abs(cdf - np.arange(256) / 255.0).max() < 0.02


def _constant_net(net, value):
    """All weights zero, output bias = value: every response equals value."""
    blob = np.zeros(net.n_params, np.float32)
    blob[-1] = value
    return blob


def test_decision_rule_truth_table():
    """Eq. (2): face = (K2 >= T_nn and K3 > 0) or (K2 > 0 and K3 >= T_nn); K3 is not computed when K2 = 0.
    Eq. (3): face = K2 >= T_nn or K3 >= T_nn, CNN_3 always evaluated."""
    n2, n3 = I.paper_stage2(), I.paper_stage3()
    reg = np.random.default_rng(0).integers(0, 256, (55, 51), dtype=np.uint8)
    hi2, lo2, hi3, lo3 = _constant_net(n2, 1.0), _constant_net(n2, -1.0), _constant_net(n3, 1.0), _constant_net(n3, -1.0)
    assert O.select_region(reg, n2, hi2, n3, hi3, 0.0, 0.0, 25)[:3] == (25, 25, True)
    assert O.select_region(reg, n2, hi2, n3, hi3, 0.0, 0.0, 26)[:3] == (25, 25, False)
    assert O.select_region(reg, n2, hi2, n3, lo3, 0.0, 0.0, 1)[:3] == (25, 0, False)
    k2, k3, face, r2, r3 = O.select_region(reg, n2, lo2, n3, hi3, 0.0, 0.0, 1)
    assert (k2, k3, face) == (0, 0, False) and np.all(r3 == 0) and np.all(r2 == -1.0)     # CNN_3 is not run
    # eq. (3), the weaker rule of Section 4.3: face = K2 >= T_nn or K3 >= T_nn
    assert O.select_region(reg, n2, hi2, n3, lo3, 0.0, 0.0, 1, rule=3)[:3] == (25, 0, True)      # rule (2) said no
    assert O.select_region(reg, n2, hi2, n3, lo3, 0.0, 0.0, 26, rule=3)[:3] == (25, 0, False)
    assert O.select_region(reg, n2, hi2, n3, hi3, 0.0, 0.0, 25, rule=3)[:3] == (25, 25, True)
    assert O.select_region(reg, n2, lo2, n3, hi3, 0.0, 0.0, 1, rule=3)[:3] == (0, 25, True)      # CNN_3's votes alone accept
    assert O.select_region(reg, n2, lo2, n3, hi3, 0.0, 0.0, 26, rule=3)[:3] == (0, 25, False)
    assert O.select_region(reg, n2, lo2, n3, lo3, 0.0, 0.0, 1, rule=3)[:3] == (0, 0, False)
    k23 = [(a, b) for a in range(0, 26, 5) for b in range(0, 26, 5)]
    assert all(((a >= 10) or (b >= 10)) >= ((a >= 10 and b > 0) or (a > 0 and b >= 10)) for a, b in k23)   # (3) is weaker
    # the comparison is strict and made in fp32
    assert O.select_region(reg, n2, hi2, n3, hi3, 1.0, 0.0, 1)[:3] == (0, 0, False)
    assert O.select_region(reg, n2, hi2, n3, hi3, float(np.nextafter(np.float32(1.0), np.float32(0.0))), 0.0, 1)[0] == 25


@pytest.mark.parametrize("act", [I.ACT_SCALED_TANH, I.ACT_TANH])
def test_response_maps_mirror_and_counts_against_torch(act):
    n2, n3 = I.paper_stage2(act), I.paper_stage3(act)
    w2, w3 = I.draw_scan_weights(n2, 31, bias_sd=0.1), I.draw_scan_weights(n3, 32, bias_sd=0.1)
    reg = np.random.default_rng(7).integers(0, 256, (55, 51), dtype=np.uint8)
    x = (reg.astype(np.float64) - 128) / 128
    want = {}
    for name, net, blob in (("2", n2, w2), ("3", n3, w3)):
        a = _torch_scan(net, blob, x)
        b = _torch_scan(net, blob, x[:, ::-1].copy())
        assert a.shape == (5, 5)
        want[name] = 0.5 * (a + b[:, ::-1])
    t2 = float(np.sort(want["2"].ravel())[-8])       # exactly seven responses of CNN_2 lie above their eighth largest
    t3 = float(np.sort(want["3"].ravel())[-4])
    k2, k3, face, r2, r3 = O.select_region(reg, n2, w2, n3, w3, np.float32(t2), np.float32(t3), 5)
    np.testing.assert_allclose(r2, want["2"], rtol=0, atol=1e-12)
    np.testing.assert_allclose(r3, want["3"], rtol=0, atol=1e-12)
    assert k2 == int((want["2"].astype(np.float32) > np.float32(t2)).sum()) and k2 in (7, 8)
    assert k3 == int((want["3"].astype(np.float32) > np.float32(t3)).sum()) and k3 in (3, 4)
    assert face is True                               # K2 >= 5 and K3 > 0
    assert O.select_region(reg, n2, w2, n3, w3, np.float32(t2), np.float32(t3), 9)[2] is False
    # eq. (3) through its CNN_3 branch: few votes of CNN_2, many of CNN_3
    t2b, t3b = float(np.sort(want["2"].ravel())[-3]), float(np.sort(want["3"].ravel())[-21])
    k2, k3, face = O.select_region(reg, n2, w2, n3, w3, np.float32(t2b), np.float32(t3b), 10, rule=3)[:3]
    assert k2 in (2, 3) and k3 in (20, 21) and face is True
    assert O.select_region(reg, n2, w2, n3, w3, np.float32(t2b), np.float32(t3b), 22, rule=3)[2] is False
    # eq. (2), second disjunct alone: 0 < K2 < T_nn and K3 >= T_nn is a face ...
    k2, k3, face = O.select_region(reg, n2, w2, n3, w3, np.float32(t2b), np.float32(t3b), 10)[:3]
    assert 0 < k2 < 10 <= k3 and face is True
    # ... and stops being one when K3 falls below T_nn as well (neither disjunct holds)
    assert O.select_region(reg, n2, w2, n3, w3, np.float32(t2b), np.float32(t3b), 22)[2] is False
    # eq. (2), first disjunct needs a vote of CNN_3: K2 >= T_nn with K3 = 0 is no face, though CNN_3 was run
    t3top = float(want["3"].max()) + 1.0
    k2, k3, face, _, r3c = O.select_region(reg, n2, w2, n3, w3, np.float32(t2), np.float32(t3top), 5)
    assert k2 >= 5 and k3 == 0 and face is False and np.abs(r3c - want["3"]).max() <= 1e-12
    # under eq. (3) the same region with K2 = 0 is accepted by CNN_3's votes: CNN_3 is evaluated whatever K2 is
    t2top = float(want["2"].max()) + 1.0
    k2, k3, face, _, r3c = O.select_region(reg, n2, w2, n3, w3, np.float32(t2top), np.float32(t3b), 10, rule=3)
    assert k2 == 0 and k3 in (20, 21) and face is True and np.abs(r3c - want["3"]).max() <= 1e-12
    k2, k3, face, _, r3c = O.select_region(reg, n2, w2, n3, w3, np.float32(t2top), np.float32(t3b), 10)
    assert (k2, k3, face) == (0, 0, False) and np.all(r3c == 0)         # eq. (2): stopped after CNN_2


def test_unit_geometry_window_sits_in_the_middle_of_its_region():
    n1, n2, n3 = I.paper_stage1(), I.paper_stage2(), I.paper_stage3()
    frame = I.make_frame(200, 160, 4)
    pyr = O.build_pyramid(frame, 12.0, 1.25)          # level 0 is the frame itself (scale 1)
    w1 = I.draw_scan_weights(n1, 1)
    s = O.scan_scores(pyr, n1, w1)
    ow0 = (200 - 27) // 4 + 1
    g = 7 * ow0 + 9                                   # window (i, j) = (9, 7) of level 0
    rec = O.select_unit(frame, pyr, [g], n1, n2, _constant_net(n2, 1.0), n3, _constant_net(n3, 1.0), 0.0, 0.0, 1)[0]
    assert (rec["level"], rec["i"], rec["j"], rec["k2"], rec["k3"], rec["face"]) == (0, 9, 7, 25, 25, True)
    raw = O.region(frame, 4 * 9 - 12, 4 * 7 - 12, 1.0, 51, 55)
    np.testing.assert_array_equal(raw[12:43, 12:39], frame[28:59, 36:63])
    # a window of a coarser level: its region is read from the frame at that level's scale
    off1 = ((pyr.levels[0].shape[0] - 31) // 4 + 1) * ow0
    rec1 = O.select_unit(frame, pyr, [off1 + 1], n1, n2, _constant_net(n2, 1.0), n3, _constant_net(n3, 1.0), 0.0, 0.0, 1)[0]
    assert (rec1["level"], rec1["i"], rec1["j"]) == (1, 1, 0)
    assert s.size > off1


def test_rectangle_merge_special_cases_and_square_case():
    """The merge of accepted regions: with equal sides it is the square merge (itself pinned by brute force), and a
    few rectangles decided by hand."""
    rng = np.random.default_rng(41)
    for n in (1, 50, 400):
        bx, by = rng.integers(0, 400, n), rng.integers(0, 300, n)
        bs, sc = rng.integers(20, 120, n), rng.standard_normal(n).astype(np.float32)
        sc[n // 2:] = sc[:n - n // 2]                 # exact ties, resolved by the order key
        order = rng.permutation(n)
        for iou, mn in ((0.3, 1), (0.5, 2)):
            a = O.merge(bx, by, bs, sc, order, iou, mn)
            b = O.merge_rect(bx, by, bs, bs, sc, order, iou, mn)
            assert a[0].tolist() == b[0].tolist() and a[1].tolist() == b[1].tolist()
    # 20 x 10 rectangles shifted along x by dx: inter = 10 (20 - dx), union = 400 - inter
    # dx = 10: 100 / 300 = 0.333 > 0.3 absorbed; dx = 11: 90 / 310 = 0.290 kept
    assert O.merge_rect([0, 10], [0, 0], [20, 20], [10, 10], [0.9, 0.8], [0, 1])[0].tolist() == [0]
    assert O.merge_rect([0, 11], [0, 0], [20, 20], [10, 10], [0.9, 0.8], [0, 1])[0].tolist() == [0, 1]
    # shifted along y by 5: inter = 20 * 5 = 100 again; by 6: 80 / 320 = 0.25, equal to a threshold of 0.25 -> kept (strict)
    assert O.merge_rect([0, 0], [0, 5], [20, 20], [10, 10], [0.9, 0.8], [0, 1])[0].tolist() == [0]
    assert O.merge_rect([0, 0], [0, 6], [20, 20], [10, 10], [0.9, 0.8], [0, 1], iou=0.25)[0].tolist() == [0, 1]
    # a 10 x 40 and a 40 x 10 rectangle inside a 40 x 40 one: 400 / 1600 = 0.25 each -> kept at 0.3, absorbed at 0.2
    # (the two small ones share a 10 x 10 patch only, 100 / 700)
    kept, nb = O.merge_rect([0, 15, 0], [0, 0, 15], [40, 10, 40], [40, 40, 10], [0.9, 0.8, 0.7], [0, 1, 2], iou=0.3)
    assert kept.tolist() == [0, 1, 2] and nb.tolist() == [0, 0, 0]
    kept, nb = O.merge_rect([0, 15, 0], [0, 0, 15], [40, 10, 40], [40, 40, 10], [0.9, 0.8, 0.7], [0, 1, 2], iou=0.2)
    assert kept.tolist() == [0] and nb.tolist() == [2]
    # touching rectangles do not overlap; an empty list stays empty
    assert O.merge_rect([0, 20], [0, 0], [20, 20], [10, 10], [0.5, 0.6], [0, 1], iou=0.0)[0].tolist() == [1, 0]
    assert O.merge_rect([], [], [], [], [], [])[0].tolist() == []


def test_rectangle_merge_against_exact_fractions():
    from fractions import Fraction
    rng = np.random.default_rng(43)
    n = 80
    bx, by = rng.integers(0, 150, n), rng.integers(0, 150, n)
    bw, bh = rng.integers(10, 90, n), rng.integers(10, 90, n)
    sc = rng.standard_normal(n).astype(np.float32)
    order = rng.permutation(n)
    for iou, mn in ((0.3, 1), (0.1, 3)):
        kept, nb = O.merge_rect(bx, by, bw, bh, sc, order, iou, mn)
        thr = Fraction(float(np.float32(iou)))
        seq = sorted(range(n), key=lambda i: (-float(sc[i]), int(order[i])))
        dead, want = set(), []
        for pos, a in enumerate(seq):
            if a in dead:
                continue
            cnt = 0
            for b in seq[pos + 1:]:
                if b in dead:
                    continue
                iw = min(int(bx[a] + bw[a]), int(bx[b] + bw[b])) - max(int(bx[a]), int(bx[b]))
                ih = min(int(by[a] + bh[a]), int(by[b] + bh[b])) - max(int(by[a]), int(by[b]))
                if iw <= 0 or ih <= 0:
                    continue
                inter = iw * ih
                uni = int(bw[a]) * int(bh[a]) + int(bw[b]) * int(bh[b]) - inter
                if Fraction(inter) > thr * uni:
                    dead.add(b)
                    cnt += 1
            if cnt + 1 >= mn:
                want.append((a, cnt))
        assert [(int(p), int(k)) for p, k in zip(kept, nb)] == want


def test_region_box_and_merge_of_a_unit_pass():
    """Box rule: the 27 x 31 window in frame pixels, rounded half up; score: the largest combined CNN_3 response."""
    n1 = I.paper_stage1()
    assert O.region_box(9, 7, 1.0, n1) == (36, 28, 27, 31)
    assert O.region_box(3, 2, 2.5, n1) == (30, 20, 68, 78)          # 67.5 and 77.5 round up
    assert O.region_box(1, 1, 1.5625, n1) == (6, 6, 42, 48)         # 6.25, 42.19, 48.44
    pyr = O.build_pyramid(I.make_frame(200, 160, 4), 12.0, 1.25)
    r3a, r3b = np.full((5, 5), -1.0), np.full((5, 5), -1.0)
    r3a[2, 3], r3b[0, 0] = 0.25, 0.75
    recs = [dict(index=10, level=0, i=9, j=7, face=True, r3=r3a), dict(index=11, level=0, i=10, j=7, face=True, r3=r3b),
            dict(index=12, level=0, i=11, j=7, face=False, r3=r3b), dict(index=40, level=0, i=30, j=20, face=True, r3=r3a)]
    det = O.select_merge(pyr, recs, n1, 0.3, 1)
    # windows (9, 7) and (10, 7) are 4 px apart: 23 x 31 of 27 x 31 in common -> merged, the one with 0.75 kept
    assert [(d["index"], d["neighbors"], d["score"]) for d in det] == [(11, 1, 0.75), (40, 0, 0.25)]
    assert (det[0]["x"], det[0]["y"], det[0]["w"], det[0]["h"]) == (40, 28, 27, 31)
