"""GPU parity of the selective unit in the paper's geometry: positions listed, response maps, counts K2 / K3 and the
decision of rule (2), against the oracle, region by region."""
import numpy as np
import pytest

import cnnc_inputs as I
from oracle import oracle as O

from parity import ATOL, BAND, RTOL, greedy_merge_rect_check

pytestmark = pytest.mark.gpu


def _select_case(frame, min_face, step, act, seed, q1, q2, t_nn, bias_sd=0.0, name="", rule=2, q3=None):
    import torch
    import paper_1508_01292_amd as P
    print("select case", name, frame.shape, "act", act, "q1", q1, flush=True)
    n1, n2, n3 = I.paper_stage1(act), I.paper_stage2(act), I.paper_stage3(act)
    w1, w2, w3 = (I.draw_scan_weights(n, seed + k, bias_sd=bias_sd) for k, n in enumerate((n1, n2, n3)))
    pyr = O.build_pyramid(frame, min_face, step)
    s1 = O.scan_scores(pyr, n1, w1)
    t1 = float(O.threshold_from_quantile(s1, q1))
    want_idx = np.nonzero(s1.astype(np.float32) > np.float32(t1))[0]
    # thresholds of the response maps: a quantile of CNN_2's responses over all listed regions
    ref = O.select_unit(frame, pyr, want_idx, n1, n2, w2, n3, w3, -1e30, -1e30, 1)
    t2 = float(np.float32(np.quantile(np.concatenate([r["r2"].ravel() for r in ref]), 1 - q2)))
    t3 = float(np.float32(np.quantile(np.concatenate([r["r3"].ravel() for r in ref]), 1 - (q2 if q3 is None else q3))))
    ref = O.select_unit(frame, pyr, want_idx, n1, n2, w2, n3, w3, t2, t3, t_nn, rule=rule)

    casc = I.default_cascade()
    ctx = P.Context(casc, I.draw_weights(casc, seed), frame.shape[1], frame.shape[0], 50000)
    ctx.set_params(min_face, step, (0.0, 0.0, 0.0))
    ctx.scan_set_weights(w1, act)
    ctx.select_set_weights(w2, w3, act)
    ft = torch.from_numpy(frame).cuda()
    ctx.build_pyramid(ft)
    ctx.scan_scoremap()
    if rule != 2:
        ctx.select_set_rule(rule)
    ctx.select_run(t1, t2, t3, t_nn)
    recs, m2, m3 = ctx.select_fetch(50000, maps=True)
    # positions: equal outside the band around t1
    got_idx = np.array([r.index for r in recs], np.int64)
    band1 = set(np.nonzero(np.abs(s1 - t1) <= BAND)[0].tolist())
    assert not ((set(got_idx.tolist()) ^ set(want_idx.tolist())) - band1)
    assert np.all(np.diff(got_idx) > 0)
    by_idx = {r["index"]: r for r in ref}
    n_cmp = n_face = n_banded = 0
    for r, a2, a3 in zip(recs, m2, m3):
        if r.index not in by_idx:
            continue
        w = by_idx[r.index]
        assert (r.level, r.i, r.j) == (w["level"], w["i"], w["j"])
        assert abs(r.response - s1[r.index]) <= ATOL + RTOL * abs(s1[r.index])
        assert np.all(np.abs(a2 - w["r2"]) <= ATOL + RTOL * np.abs(w["r2"])), "CNN_2 map of %d: %g" % (r.index, np.abs(a2 - w["r2"]).max())
        near2 = int((np.abs(w["r2"] - t2) <= BAND).sum())
        assert abs(r.k2 - w["k2"]) <= near2
        if near2 == 0 and (w["k2"] > 0 or rule == 3):
            assert np.all(np.abs(a3 - w["r3"]) <= ATOL + RTOL * np.abs(w["r3"])), "CNN_3 map of %d" % r.index
            near3 = int((np.abs(w["r3"] - t3) <= BAND).sum())
            assert abs(r.k3 - w["k3"]) <= near3
            if near3 == 0:
                assert bool(r.face) == w["face"]
                n_face += int(w["face"])
            else:
                n_banded += 1
        elif near2 == 0:
            assert r.k3 == 0 and not r.face and np.all(a3 == 0)       # CNN_3 not run
        else:
            n_banded += 1
        # the record's own consistency with rule (2)
        if rule == 3:
            assert bool(r.face) == (r.k2 >= t_nn or r.k3 >= t_nn)
        else:
            assert bool(r.face) == ((r.k2 >= t_nn and r.k3 > 0) or (r.k2 > 0 and r.k3 >= t_nn))
        n_cmp += 1
    # ---- merge of the accepted regions
    faces = [k for k, r in enumerate(recs) if r.face]
    box = np.array([O.region_box(recs[k].i, recs[k].j, pyr.scale[recs[k].level], n1) for k in faces], np.int64).reshape(-1, 4)
    sc = m3[faces].reshape(len(faces), 25).max(axis=1) if faces else np.zeros(0, np.float32)
    order = [recs[k].index for k in faces]
    ref_faces = [r for r in ref if r["face"]]
    ref_seq = sorted(ref_faces, key=lambda r: (-float(np.float32(r["r3"].max())), r["index"]))
    gpu_seq = sorted(range(len(faces)), key=lambda p: (-float(sc[p]), order[p]))
    same_input = [r["index"] for r in ref_seq] == [order[p] for p in gpu_seq]       # same regions in the same order
    for iou, mn in ((0.3, 1), (0.5, 2)):
        det = [d.as_dict() for d in ctx.select_merge(iou, mn, cap=50000)]
        valid = greedy_merge_rect_check(box[:, 0], box[:, 1], box[:, 2], box[:, 3], sc, order, iou, mn)
        assert [(d["index"], d["neighbors"]) for d in det] == [(order[p], k) for p, k in valid], (iou, mn)
        for d, (p, _) in zip(det, valid):
            assert (d["x"], d["y"], d["w"], d["h"]) == tuple(int(v) for v in box[p]) and d["level"] == recs[faces[p]].level
            assert d["score"] == sc[p]
        if same_input:
            want = O.select_merge(pyr, ref, n1, iou, mn)
            assert [(d["index"], d["neighbors"], d["x"], d["y"], d["w"], d["h"], d["level"]) for d in det] == \
                [(w["index"], w["neighbors"], w["x"], w["y"], w["w"], w["h"], w["level"]) for w in want], (iou, mn)
            assert all(abs(d["score"] - w["score"]) <= ATOL + RTOL * abs(w["score"]) for d, w in zip(det, want))
        # the whole path in one call, synchronous and enqueued on a stream: the same detections
        assert [d.as_dict() for d in ctx.detect_paper(ft, t1, t2, t3, t_nn, iou, mn, cap=50000)] == det
        side = torch.cuda.Stream()
        ctx.detect_paper_async(ft, t1, t2, t3, t_nn, iou, mn, stream=side)
        assert [d.as_dict() for d in ctx.fetch_paper(50000)] == det
        print("   merge at iou %.1f, min_neighbors %d: %d regions -> %d detections (%s)"
              % (iou, mn, len(faces), len(det), "equal to the oracle's" if same_input else "valid merge of the GPU's own list"),
              flush=True)
    ctx.close()
    print("   %d positions listed, %d compared, %d faces, %d with a response inside the band" % (len(recs), n_cmp, n_face, n_banded),
          flush=True)
    assert n_cmp >= len(want_idx) - len(band1)
    return recs, ref


@pytest.mark.parametrize("act", [I.ACT_RATIONAL, I.ACT_TANH])
def test_select_vga(act):
    c = I.CONFIGS[0]
    frame = I.make_frame(c["width"], c["height"], I.config_seed(0))
    recs, ref = _select_case(frame, c["min_face"], c["scale_step"], act, 40, 0.1, 0.3, 5,
                             bias_sd=0.0 if act == I.ACT_RATIONAL else 0.1, name="vga")
    assert len(ref) == 85
    assert any(r["face"] for r in ref) and not all(r["face"] for r in ref)


def test_select_weaker_rule_of_eq_3():
    """The same frame under eq. (3): every region eq. (2) accepts stays accepted, and some are added."""
    c = I.CONFIGS[0]
    frame = I.make_frame(c["width"], c["height"], I.config_seed(0))
    # CNN_3's threshold sits high in its responses, so that many regions have K2 >= T_nn and K3 = 0: there the rules differ
    args = (frame, c["min_face"], c["scale_step"], I.ACT_RATIONAL, 40, 0.1, 0.3, 4)
    _, ref3 = _select_case(*args, name="vga, rule 3", rule=3, q3=0.004)
    _, ref2 = _select_case(*args, name="vga, rule 2", rule=2, q3=0.004)
    f2, f3 = {r["index"] for r in ref2 if r["face"]}, {r["index"] for r in ref3 if r["face"]}
    assert f2 < f3


def test_select_ragged_frame_regions_cut_by_the_border():
    # small levels: most regions reach over the level edge, where the frame edge is repeated
    frame = I.make_frame(333, 251, 5)
    recs, ref = _select_case(frame, 12.0, 1.3, I.ACT_RATIONAL, 50, 0.03, 0.2, 3, bias_sd=0.1, name="333x251")
    assert any(r["i"] == 0 or r["j"] == 0 for r in ref)


def test_select_uhd_headline_frame():
    c = I.CONFIGS[2]
    frame = I.make_frame(c["width"], c["height"], I.config_seed(2))
    recs, ref = _select_case(frame, c["min_face"], c["scale_step"], I.ACT_RATIONAL, 60, 0.02, 0.25, 6, name="uhd")
    assert len(ref) == 965


def test_select_errors_and_degenerate_cases():
    import torch
    import paper_1508_01292_amd as P
    casc = I.default_cascade()
    n1, n2, n3 = I.paper_stage1(), I.paper_stage2(), I.paper_stage3()
    w1, w2, w3 = I.draw_scan_weights(n1, 1), I.draw_scan_weights(n2, 2), I.draw_scan_weights(n3, 3)
    frame = I.make_frame(160, 120, 8)
    ctx = P.Context(casc, I.draw_weights(casc, 1), 160, 120, 16)
    ctx.set_params(12.0, 1.25, (0.0, 0.0, 0.0))
    with pytest.raises(P.CnncError):
        ctx.select_run(0.0, 0.0, 0.0, 1)              # no weights
    with pytest.raises(P.CnncError):
        ctx.select_set_weights(w2[:-1], w3, 1)
    with pytest.raises(P.CnncError):
        ctx.select_set_weights(w2, w3, 4)
    with pytest.raises(P.CnncError):
        ctx.select_set_rule(1)
    ctx.select_set_weights(w2, w3, 1)
    with pytest.raises(P.CnncError):
        ctx.select_run(0.0, 0.0, 0.0, 1)              # no scan of this frame
    with pytest.raises(P.CnncError) as e:
        ctx.detect_paper(torch.from_numpy(frame).cuda(), 0.0, 0.0, 0.0, 1)     # whole path without the scan's weights
    assert e.value.code == -5
    with pytest.raises(P.CnncError) as e:
        ctx.fetch_paper()                             # nothing enqueued
    assert e.value.code == -5
    ctx.scan_set_weights(w1, 1)
    with pytest.raises(P.CnncError) as e:
        ctx.detect_paper(torch.from_numpy(frame).cuda(), 0.0, 0.0, 0.0, 0)     # T_nn < 1
    assert e.value.code == -1
    assert ctx.detect_paper(torch.from_numpy(frame).cuda(), 1e30, 0.0, 0.0, 1) == []
    ctx.build_pyramid(torch.from_numpy(frame).cuda())
    with pytest.raises(P.CnncError):
        ctx.select_fetch(16)                          # nothing run
    with pytest.raises(P.CnncError):
        ctx.select_merge()
    ctx.scan_scoremap()
    with pytest.raises(P.CnncError):
        ctx.select_run(float("nan"), 0.0, 0.0, 1)
    ctx.select_run(1e30, 0.0, 0.0, 1)                 # nothing passes T_1
    assert ctx.select_fetch(16) == []
    assert ctx.select_merge() == []
    with pytest.raises(P.CnncError):
        ctx.select_merge(iou=1.5)
    t_few = float(np.sort(ctx.get_scan_scoremap())[-9])   # eight positions (fewer with ties) lie above it
    ctx.select_run(t_few, 1e30, 1e30, 1)              # positions listed, none accepted
    assert 0 < len(ctx.select_fetch(16)) <= 8 and ctx.select_merge() == []
    ctx.select_run(t_few, -1e30, -1e30, 1)            # all of them accepted
    n_acc = len(ctx.select_fetch(16))
    det = ctx.select_merge(iou=0.0, min_neighbors=1)
    assert 0 < len(det) <= n_acc and sum(d.neighbors + 1 for d in det) == n_acc
    with pytest.raises(P.CnncError) as e:
        ctx.select_merge(iou=1.0, cap=0)              # nothing can be absorbed at iou 1: n_acc detections, no room
    assert e.value.code == -3
    ctx.select_run(-1e30, 0.0, 0.0, 1)                # everything passes: more than the capacity of 16
    with pytest.raises(P.CnncError) as e:
        ctx.select_fetch(16)
    assert e.value.code == -3
    with pytest.raises(P.CnncError) as e:
        ctx.select_merge()
    assert e.value.code == -3
    # a new pyramid invalidates the unit's results
    ctx.build_pyramid(torch.from_numpy(frame).cuda())
    with pytest.raises(P.CnncError):
        ctx.select_fetch(16)
    ctx.close()
