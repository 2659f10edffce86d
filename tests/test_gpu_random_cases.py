"""GPU parity on seeded random cases: frame size, pyramid parameters, activation, survival quantiles, merge parameters
and row pitch are drawn per case; every intermediate of the path is compared with the oracle through the same helpers
as the fixed cases (tests/parity.py), and the one-call path must return the same detections as the step-by-step calls."""
import numpy as np
import pytest

import cnnc_inputs as I
from oracle import oracle as O

from parity import compare_with_trace, run_gpu_steps

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("sweep_seed", [11, 12])
def test_random_cases_against_the_oracle(sweep_seed):
    import torch
    import paper_1508_01292_amd as P
    rng = np.random.default_rng(sweep_seed)
    done = 0
    while done < 8:
        w, h = int(rng.integers(40, 700)), int(rng.integers(40, 500))
        min_face = float(rng.choice([12.0, 14.5, 20.0, 33.0, 60.0]))
        step = float(rng.choice([1.1, 1.2, 1.25, 1.41, 2.0]))
        act = int(rng.choice([1, 2, 3]))
        q1, q2 = float(rng.choice([0.005, 0.02, 0.1, 0.5])), float(rng.choice([0.05, 0.2, 0.6]))
        iou, mn = float(rng.choice([0.1, 0.3, 0.5, 0.8])), int(rng.choice([1, 2, 3]))
        seed = int(rng.integers(0, 10000))
        padded = bool(rng.integers(0, 2))
        if min(w, h) / (min_face / 12.0) < 12:
            continue
        casc = I.default_cascade(act)
        W = I.draw_weights(casc, seed, bias_sd=float(rng.choice([0.0, 0.1])))
        frame = I.make_frame(w, h, seed)
        tr = O.detect(frame, casc, W, min_face, step, quantiles=(q1, q2), iou=iou, min_neighbors=mn)
        if len(tr.idx3) > 30000:                      # more accepted windows than the merge takes: covered elsewhere
            continue
        print("random case: %dx%d%s min_face %g step %g act %d q %g/%g iou %g min_neighbors %d seed %d"
              % (w, h, " padded rows" if padded else "", min_face, step, act, q1, q2, iou, mn, seed), flush=True)
        ctx = P.Context(casc, W, w, h, 400000)
        ctx.set_params(min_face, step, tr.thr, merge_iou=iou, min_neighbors=mn)
        if padded:                                    # row pitch larger than the width
            buf = torch.zeros((h, w + 13), dtype=torch.uint8, device="cuda")
            buf[:, :w] = torch.from_numpy(frame).cuda()
            ft = buf[:, :w]
        else:
            ft = torch.from_numpy(frame).cuda()
        g = run_gpu_steps(ctx, ft, tr.thr)
        compare_with_trace(g, tr, frame, casc, W, iou=iou, min_neighbors=mn)
        assert [d.as_dict() for d in ctx.detect(ft, 32768)] == g["det"]
        ctx.close()
        done += 1
