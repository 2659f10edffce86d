"""cnnc_compact_noalloc (the compaction for callers that cannot allocate) against cnnc_compact_survivors on the same
score maps: two calls in a row, the second with a smaller input, both forms of the kernels (with and without the
separate scan launch), truncation, the empty input and the size limit.  Results must be equal bit for bit."""
import ctypes as C

import numpy as np
import pytest

import cnnc_inputs as I

pytestmark = pytest.mark.gpu


def _existing_path(P, torch, ctx, frame, n_pass):
    """Score map (device pointer, length), a threshold that about n_pass values exceed, and the list
    cnnc_compact_survivors(1) makes of the map at that threshold."""
    ctx.build_pyramid(torch.from_numpy(frame).cuda())
    ctx.stage1_scoremap()
    s = ctx.get_scoremap()
    thr = float(np.partition(s, s.size - n_pass)[s.size - n_pass])
    ctx.compact_survivors(1, thr)
    idx, sc = ctx.get_survivors(1)
    p, n = C.c_void_p(0), C.c_int64(0)
    assert P.lib().cnnc_get_scoremap(ctx._h, C.byref(p), C.byref(n)) == 0
    return p.value, n.value, thr, idx, sc


def _noalloc(P, torch, d_vals, n, thr, cap, stream=None):
    oi = torch.full((max(cap, 1),), -1, dtype=torch.int32, device="cuda")
    osc = torch.full((max(cap, 1),), float("nan"), dtype=torch.float32, device="cuda")
    cnt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    rc = P.lib().cnnc_compact_noalloc(C.c_void_p(d_vals), C.c_int64(n), C.c_float(thr), C.c_void_p(oi.data_ptr()),
                                      C.c_void_p(osc.data_ptr()), C.c_int32(cap), C.c_void_p(cnt.data_ptr()),
                                      C.c_void_p(int(stream.cuda_stream)) if stream is not None else C.c_void_p(0))
    torch.cuda.synchronize()
    return rc, oi.cpu().numpy().view(np.uint32), osc.cpu().numpy(), int(cnt.item())


def test_noalloc_compaction_equals_the_context_path_twice_in_a_row():
    import torch

    import paper_1508_01292_amd as P
    casc = I.default_cascade()
    W = I.draw_weights(casc, 77)
    # first call: 8.4 M values (more than 4,096 workgroups: the form with the separate scan launch)
    w, h = 4400, 2100
    big = P.Context(casc, W, w, h, 300000)
    big.set_params(12.0, 2.0, (0.0, 0.0, 0.0))
    d_vals, n, thr, idx, sc = _existing_path(P, torch, big, I.make_frame(w, h, 77), 200000)
    assert n > 4096 * 2048 and 1000 < len(idx) < 300000
    print("case no-alloc, first call: %d values -> %d" % (n, len(idx)), flush=True)
    rc, gi, gs, cnt = _noalloc(P, torch, d_vals, n, thr, 300000)
    assert rc == 0 and cnt == len(idx)
    assert np.array_equal(gi[:cnt], idx) and np.array_equal(gs[:cnt], sc)
    # second call, smaller input (a few hundred workgroups: every scatter workgroup sums the counts before it);
    # the array still holds the first call's counts beyond this call's workgroups
    small = P.Context(casc, W, 640, 480, 100000)
    small.set_params(24.0, 1.25, (0.0, 0.0, 0.0))
    d2, n2, thr2, idx2, sc2 = _existing_path(P, torch, small, I.make_frame(640, 480, 5), 3000)
    assert 2048 < n2 < n // 8 and len(idx2) > 100
    print("case no-alloc, second call: %d values -> %d" % (n2, len(idx2)), flush=True)
    s = torch.cuda.Stream()
    rc, gi, gs, cnt = _noalloc(P, torch, d2, n2, thr2, 100000, stream=s)
    assert rc == 0 and cnt == len(idx2)
    assert np.array_equal(gi[:cnt], idx2) and np.array_equal(gs[:cnt], sc2)
    # a third, the large one again: nothing of the smaller call is left behind
    rc, gi, gs, cnt = _noalloc(P, torch, d_vals, n, thr, 300000)
    assert rc == 0 and cnt == len(idx) and np.array_equal(gi[:cnt], idx) and np.array_equal(gs[:cnt], sc)
    # truncation: the count is the untruncated one, the first `cap` entries are valid, nothing is written beyond them
    rc, gi, gs, cnt = _noalloc(P, torch, d2, n2, thr2, 50)
    assert rc == 0 and cnt == len(idx2) and np.array_equal(gi[:50], idx2[:50]) and np.array_equal(gs[:50], sc2[:50])
    # a prefix that ends inside a workgroup, nothing passing, the empty input
    rc, gi, gs, cnt = _noalloc(P, torch, d2, 5000, thr2, 100000)
    k = int(np.searchsorted(idx2, 5000))
    assert rc == 0 and cnt == k and np.array_equal(gi[:k], idx2[:k])
    rc, _, _, cnt = _noalloc(P, torch, d2, n2, 1e30, 100)
    assert rc == 0 and cnt == 0
    rc, _, _, cnt = _noalloc(P, torch, 0, 0, 0.0, 0)
    assert rc == 0 and cnt == 0
    # beyond the fixed scratch: refused, nothing launched (the count keeps its fill value)
    rc, _, _, cnt = _noalloc(P, torch, d_vals, (1 << 24) + 1, 0.0, 10)
    assert rc == -6 and cnt == -1
    one = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert P.lib().cnnc_compact_noalloc(C.c_void_p(d2), C.c_int64(-1), C.c_float(0), C.c_void_p(0), C.c_void_p(0),
                                        C.c_int32(0), C.c_void_p(one.data_ptr()), C.c_void_p(0)) == -1
    assert P.lib().cnnc_compact_noalloc(C.c_void_p(d2), C.c_int64(10), C.c_float(0), C.c_void_p(0), C.c_void_p(0),
                                        C.c_int32(0), C.c_void_p(0), C.c_void_p(0)) == -1
    big.close()
    small.close()
