"""Seeded sweep of the whole path over frame sizes, pyramid parameters, activations, survival quantiles and merge
parameters: every intermediate against the oracle, as in the fixed cases of test_gpu_parity.py."""
import numpy as np
import pytest

import cnnc_inputs as I
from oracle import oracle as O

from parity import compare_with_trace, run_gpu_steps

pytestmark = pytest.mark.gpu


def test_seeded_sweep_of_sizes_and_parameters():
    import torch
    import paper_1508_01292_amd as P
    rng = np.random.default_rng(1508)
    done = 0
    while done < 14:
        w, h = int(rng.integers(40, 480)), int(rng.integers(40, 360))
        min_face = float(rng.choice([12.0, 14.5, 20.0, 33.0, 60.0]))
        step = float(rng.choice([1.1, 1.2, 1.25, 1.41, 2.0]))
        act = int(rng.choice([I.ACT_RATIONAL, I.ACT_SCALED_TANH, I.ACT_TANH]))
        q1, q2 = float(rng.choice([0.005, 0.02, 0.1, 0.4])), float(rng.choice([0.05, 0.2, 0.6]))
        iou, mn = float(rng.choice([0.1, 0.3, 0.5, 0.8])), int(rng.choice([1, 2, 3]))
        seed = int(rng.integers(0, 10000))
        bias_sd = float(rng.choice([0.0, 0.1]))
        if min(w, h) / (min_face / 12.0) < 12:
            continue                                          # no pyramid level fits a window
        if O.pyramid_layout(w, h, min_face, step).score_off[-1] > 250000:
            continue                                          # keeps the oracle's share of the test short
        print("sweep case %d: %dx%d min_face %g step %g act %d quantiles %g / %g iou %g min_neighbors %d seed %d"
              % (done, w, h, min_face, step, act, q1, q2, iou, mn, seed), flush=True)
        casc = I.default_cascade(act)
        W = I.draw_weights(casc, seed, bias_sd=bias_sd)
        frame = I.make_frame(w, h, seed)
        tr = O.detect(frame, casc, W, min_face, step, quantiles=(q1, q2), iou=iou, min_neighbors=mn)
        ctx = P.Context(casc, W, w, h, len(tr.idx1) + 1000)
        ctx.set_params(min_face, step, tr.thr, merge_iou=iou, min_neighbors=mn)
        if done % 2:                                          # every other frame sits in a wider buffer (pitch > width)
            buf = torch.zeros((h, w + 13), dtype=torch.uint8, device="cuda")
            buf[:, :w] = torch.from_numpy(frame).cuda()
            ft = buf[:, :w]
        else:
            ft = torch.from_numpy(frame).cuda()
        g = run_gpu_steps(ctx, ft, tr.thr)
        info = compare_with_trace(g, tr, frame, casc, W, iou, mn)
        assert [d.as_dict() for d in ctx.detect(ft, 32768)] == g["det"]
        print("   windows %d -> %d -> %d -> %d -> %d detections; %s"
              % (tr.score1.size, len(g["idx1"]), len(g["idx2"]), len(g["idx3"]), len(g["det"]), info), flush=True)
        ctx.close()
        done += 1
