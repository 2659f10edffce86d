"""Comparison of the HIP path with the CPU oracle, step by step (helper for the GPU tests).

Bars (from the benchmark spec):
  * pyramid bytes, window indices and survivor sets: bit-exact, except that windows whose ORACLE
    score lies within BAND of a stage threshold may fall on either side;
  * scores: |gpu - oracle| <= ATOL + RTOL * |oracle| (fp32 kernels against the fp64 oracle).
"""
import numpy as np

from oracle import oracle as O

ATOL = 1e-4
RTOL = 1e-4
BAND = 1e-4


def close(gpu, ref):
    gpu = np.asarray(gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    return np.abs(gpu - ref) <= ATOL + RTOL * np.abs(ref)


def assert_scores(gpu, ref, what):
    ok = close(gpu, ref)
    if not ok.all():
        bad = np.nonzero(~ok)[0]
        i = bad[0]
        raise AssertionError("%s: %d of %d scores off, first at %d: gpu %.7f oracle %.7f (max abs diff %.3g)"
                             % (what, bad.size, ok.size, i, gpu[i], ref[i], np.abs(np.asarray(gpu, np.float64) - ref).max()))


def assert_survivors(gpu_idx, ref_scores_by_index, ref_candidates, thr, what):
    """gpu_idx: indices the GPU kept.  ref_candidates: all indices that entered the stage (oracle side),
    ref_scores_by_index: dict-like index -> oracle score.  Outside the band the sets must be equal.
    Returns the set of indices inside the band."""
    cand = np.asarray(ref_candidates, np.int64)
    sc = np.asarray([ref_scores_by_index[i] for i in cand], np.float64) if not isinstance(ref_scores_by_index, np.ndarray) \
        else ref_scores_by_index
    band = set(cand[np.abs(sc - float(thr)) <= BAND].tolist())
    want = set(cand[sc.astype(np.float32) > np.float32(thr)].tolist())
    got = set(int(g) for g in gpu_idx)
    assert np.all(np.diff(np.asarray(gpu_idx, np.int64)) > 0), what + ": survivor list not in ascending order"
    diff = (want ^ got) - band
    assert not diff, "%s: %d survivors differ outside the band, e.g. %s" % (what, len(diff), sorted(diff)[:5])
    return band


def boxes_of(pyr, idx):
    """Frame-pixel boxes of flat window indices (test-side restatement of the box rule)."""
    lvl, ys, xs = pyr.decode(idx)
    sc = np.asarray(pyr.scale, np.float64)[lvl]
    f = lambda v: np.floor(v + 0.5).astype(np.int64)
    return f(xs * sc), f(ys * sc), f(12 * sc), lvl


def greedy_merge_check(bx, by, bs, score, order, iou=0.3, min_neighbors=1):
    """Test-side greedy merge (numpy) used only as a validity check of the GPU's detections when several
    results are correct; returns [(position, neighbours)] in kept order."""
    n = len(bx)
    seq = sorted(range(n), key=lambda i: (-float(np.float32(score[i])), int(order[i])))
    bx, by, bs = (np.asarray(a, np.int64)[seq] for a in (bx, by, bs))
    dead = np.zeros(n, bool)
    thr = float(np.float32(iou))
    out = []
    for i in range(n):
        if dead[i]:
            continue
        j = np.arange(i + 1, n)
        iw = np.minimum(bx[i] + bs[i], bx[j] + bs[j]) - np.maximum(bx[i], bx[j])
        ih = np.minimum(by[i] + bs[i], by[j] + bs[j]) - np.maximum(by[i], by[j])
        inter = np.where((iw > 0) & (ih > 0), iw * ih, 0)
        uni = bs[i] ** 2 + bs[j] ** 2 - inter
        hit = (inter.astype(np.float64) > thr * uni.astype(np.float64)) & ~dead[j] & (inter > 0)
        dead[j[hit]] = True
        if hit.sum() + 1 >= min_neighbors:
            out.append((seq[i], int(hit.sum())))
    return out


def greedy_merge_rect_check(bx, by, bw, bh, score, order, iou=0.3, min_neighbors=1):
    """The same test-side check for rectangles (the regions the selective unit accepts)."""
    n = len(bx)
    seq = sorted(range(n), key=lambda i: (-float(np.float32(score[i])), int(order[i])))
    bx, by, bw, bh = (np.asarray(a, np.int64)[seq] for a in (bx, by, bw, bh))
    dead = np.zeros(n, bool)
    thr = float(np.float32(iou))
    out = []
    for i in range(n):
        if dead[i]:
            continue
        j = np.arange(i + 1, n)
        iw = np.minimum(bx[i] + bw[i], bx[j] + bw[j]) - np.maximum(bx[i], bx[j])
        ih = np.minimum(by[i] + bh[i], by[j] + bh[j]) - np.maximum(by[i], by[j])
        inter = np.where((iw > 0) & (ih > 0), iw * ih, 0)
        uni = bw[i] * bh[i] + bw[j] * bh[j] - inter
        hit = (inter.astype(np.float64) > thr * uni.astype(np.float64)) & ~dead[j] & (inter > 0)
        dead[j[hit]] = True
        if hit.sum() + 1 >= min_neighbors:
            out.append((seq[i], int(hit.sum())))
    return out


def run_gpu_steps(ctx, frame_t, thr, stream=None, det_cap=8192):
    """Run the path call by call and fetch every intermediate."""
    out = {}
    ctx.build_pyramid(frame_t, stream)
    out["pyramid"] = ctx.get_pyramid()
    ctx.stage1_scoremap(stream)
    out["score1"] = ctx.get_scoremap()
    ctx.compact_survivors(1, float(thr[0]), stream)
    out["idx1"], out["sc1"] = ctx.get_survivors(1, stream)
    ctx.eval_stage(2, stream)
    out["score2"] = ctx.get_stage_scores(2, stream)
    ctx.compact_survivors(2, float(thr[1]), stream)
    out["idx2"], out["sc2"] = ctx.get_survivors(2, stream)
    ctx.eval_stage(3, stream)
    out["score3"] = ctx.get_stage_scores(3, stream)
    ctx.compact_survivors(3, float(thr[2]), stream)
    out["idx3"], out["sc3"] = ctx.get_survivors(3, stream)
    out["det"] = [d.as_dict() for d in ctx.merge_detections(det_cap, stream)]
    return out


def compare_with_trace(g, tr: "O.Trace", frame, cascade, weights, iou=0.3, min_neighbors=1):
    """Element-by-element comparison of run_gpu_steps output with an oracle trace.  Where a band
    window makes the two paths take different survivors, downstream steps are compared on the
    windows both paths evaluated (the oracle evaluates extra windows on demand)."""
    pyr = tr.pyramid
    ref_pyr = np.concatenate([l.ravel() for l in pyr.levels])
    assert g["pyramid"].size == ref_pyr.size
    assert np.array_equal(g["pyramid"], ref_pyr), "pyramid bytes differ at %d positions" % int((g["pyramid"] != ref_pyr).sum())

    assert g["score1"].size == tr.score1.size
    assert_scores(g["score1"], tr.score1, "stage-1 score map")

    t1, t2, t3 = tr.thr
    band1 = assert_survivors(g["idx1"], tr.score1, np.arange(tr.score1.size), t1, "stage-1 survivors")
    assert np.array_equal(g["sc1"], g["score1"][g["idx1"]]), "compacted stage-1 scores are not the score map's"

    # stage 2 on the GPU's own list; oracle scores for exactly those windows
    ref2 = dict(zip(tr.idx1.tolist(), tr.score2.tolist()))
    extra = [i for i in g["idx1"].tolist() if i not in ref2]
    assert set(extra) <= band1
    if extra:
        ref2.update(zip(extra, O.eval_stage(frame, pyr, np.asarray(extra), cascade[1], weights[1]).tolist()))
    r2 = np.asarray([ref2[i] for i in g["idx1"].tolist()])
    assert_scores(g["score2"], r2, "stage-2 scores")
    band2 = assert_survivors(g["idx2"], r2, g["idx1"], t2, "stage-2 survivors")
    pos = np.searchsorted(g["idx1"], g["idx2"])
    assert np.array_equal(g["sc2"], g["score2"][pos]), "compacted stage-2 scores misaligned"

    ref3 = dict(zip(tr.idx2.tolist(), tr.score3.tolist()))
    extra = [i for i in g["idx2"].tolist() if i not in ref3]
    assert set(extra) <= (band1 | band2)
    if extra:
        ref3.update(zip(extra, O.eval_stage(frame, pyr, np.asarray(extra), cascade[2], weights[2]).tolist()))
    r3 = np.asarray([ref3[i] for i in g["idx2"].tolist()])
    assert_scores(g["score3"], r3, "stage-3 scores")
    band3 = assert_survivors(g["idx3"], r3, g["idx2"], t3, "stage-3 survivors")
    pos = np.searchsorted(g["idx2"], g["idx3"])
    assert np.array_equal(g["sc3"], g["score3"][pos]), "compacted stage-3 scores misaligned"

    # merge.  First bar: the detections equal the oracle's own (computed from the oracle's scores only).
    want = [(d["x"], d["y"], d["size"], d["level"], d["neighbors"], d["index"]) for d in tr.det]
    got = [(d["x"], d["y"], d["size"], d["level"], d["neighbors"], d["index"]) for d in g["det"]]
    exact = got == want
    if exact:
        assert_scores([d["score"] for d in g["det"]], [d["score"] for d in tr.det], "detection scores")
    else:
        # Several results can be correct when the two paths legitimately differ upstream: a window inside a
        # threshold band changes the accepted set, or two accepted windows whose oracle scores are closer than
        # the score tolerance swap places in the greedy order.  Only then (the accepted sets differ through a band
        # window, or the two descending-score orders of the same set really differ) is the result allowed to be
        # the greedy merge of what the GPU path accepted: the ORACLE's merge routine fed with the GPU's list and
        # fp32 scores, and the numpy restatement above as a second opinion.
        seq_ref = sorted(range(len(tr.idx3)), key=lambda p: (-float(np.float32(tr.score3_kept[p])), int(tr.idx3[p])))
        seq_gpu = sorted(range(len(g["idx3"])), key=lambda p: (-float(g["sc3"][p]), int(g["idx3"][p])))
        reordered = [int(tr.idx3[p]) for p in seq_ref] != [int(g["idx3"][p]) for p in seq_gpu]
        same_set = np.array_equal(np.asarray(tr.idx3, np.int64), np.asarray(g["idx3"], np.int64))
        assert ((band1 or band2 or band3) and not same_set) or (same_set and reordered), \
            "detections differ from the oracle's although the accepted windows and their order are the same"
        bx, by, bs, lvl = boxes_of(pyr, g["idx3"])
        kept, nb = O.merge(bx, by, bs, g["sc3"], g["idx3"], iou, min_neighbors)
        by_oracle = [(int(bx[p]), int(by[p]), int(bs[p]), int(lvl[p]), int(n), int(g["idx3"][p])) for p, n in zip(kept, nb)]
        assert got == by_oracle, "merged detections are not the oracle's merge of the windows the GPU accepted"
        valid = [(int(bx[p]), int(by[p]), int(bs[p]), int(lvl[p]), int(n), int(g["idx3"][p]))
                 for p, n in greedy_merge_check(bx, by, bs, g["sc3"], g["idx3"], iou, min_neighbors)]
        assert got == valid, "merged detections are not a greedy merge of the accepted windows"
    return dict(band=(len(band1), len(band2), len(band3)), merge_exact=exact)
