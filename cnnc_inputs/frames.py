"""Seeded synthetic grayscale frames shaped like the paper's video workloads.

The paper measures on video frames from VGA up to 4K UHD (Section 4.4).  Those
videos are not available, so frames are synthetic stand-ins: smooth noise plus
hard-edged bright / dark ellipses of face-like sizes.

Recipe (per frame, numpy `default_rng([seed, frame_index])`):
  1. i.i.d. N(0,1) field, separable Gaussian blur sigma = 2 px (reflect border),
  2. rescaled to mean 128, standard deviation 40,
  3. `n_ellipses` filled ellipses: full axes U(30,120) px each, centre uniform in
     the frame, angle U(0,pi), sign +-1 with probability 1/2, amplitude
     U(40,90) grey levels added inside the ellipse,
  4. clipped to [0,255] and rounded to uint8.
"""
from typing import Dict, List, Optional

import numpy as np
from scipy.ndimage import gaussian_filter1d

# Workload table: frame size, smallest face (px) mapped to the 12x12 stage-1
# window, pyramid scale step, frames in the stream.
CONFIGS: List[Dict] = [
    dict(name="vga", width=640, height=480, min_face=60, scale_step=1.25, frames=1),
    dict(name="fhd", width=1920, height=1080, min_face=60, scale_step=1.25, frames=1),
    dict(name="uhd", width=3840, height=2160, min_face=60, scale_step=1.25, frames=1),
    dict(name="uhd_small_faces", width=3840, height=2160, min_face=24, scale_step=1.2, frames=1),
    dict(name="fhd_stream", width=1920, height=1080, min_face=60, scale_step=1.25, frames=16),
]


def config_seed(config_index: int) -> int:
    return 1508 + config_index


def make_frame(width: int, height: int, seed: int, frame_index: int = 0,
               n_ellipses: Optional[int] = 20) -> np.ndarray:
    """One uint8 frame [height][width]; `n_ellipses=None` draws the count from U{0..200}."""
    rng = np.random.default_rng([seed, frame_index])
    img = rng.standard_normal((height, width))
    img = gaussian_filter1d(img, 2.0, axis=0, mode="reflect")
    img = gaussian_filter1d(img, 2.0, axis=1, mode="reflect")
    img = (img - img.mean()) / img.std() * 40.0 + 128.0
    if n_ellipses is None:
        n_ellipses = int(rng.integers(0, 201))
    for _ in range(n_ellipses):
        ax, ay = rng.uniform(30, 120, 2) / 2.0          # half axes
        cx, cy = rng.uniform(0, width), rng.uniform(0, height)
        ang = rng.uniform(0, np.pi)
        amp = rng.uniform(40, 90) * (1.0 if rng.random() < 0.5 else -1.0)
        r = int(np.ceil(max(ax, ay))) + 1
        x0, x1 = max(0, int(cx) - r), min(width, int(cx) + r + 1)
        y0, y1 = max(0, int(cy) - r), min(height, int(cy) + r + 1)
        if x0 >= x1 or y0 >= y1:
            continue
        yy, xx = np.mgrid[y0:y1, x0:x1]
        dx, dy = xx - cx, yy - cy
        u = dx * np.cos(ang) + dy * np.sin(ang)
        v = -dx * np.sin(ang) + dy * np.cos(ang)
        inside = (u / ax) ** 2 + (v / ay) ** 2 <= 1.0
        img[y0:y1, x0:x1][inside] += amp
    return np.clip(np.rint(img), 0, 255).astype(np.uint8)


def make_stream(config_index: int) -> List[np.ndarray]:
    """All frames of a workload; the multi-frame stream varies the ellipse count per frame."""
    c = CONFIGS[config_index]
    seed = config_seed(config_index)
    if c["frames"] == 1:
        return [make_frame(c["width"], c["height"], seed)]
    return [make_frame(c["width"], c["height"], seed, i, None) for i in range(c["frames"])]
