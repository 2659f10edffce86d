"""Seeded synthetic inputs for the compact CNN cascade hot path.

This package only *draws inputs*: frames, network weights and the description
of the three network shapes.  It contains none of the detector's arithmetic
(no pyramid, no convolution, no thresholding) and is the only code that both
the CPU oracle's tests and the HIP library's tests import.
"""
from .cascade import (ACT_NONE, ACT_RATIONAL, ACT_SCALED_TANH, ACT_TANH, CONV,
                      FC, POOL, Layer, RLayer, ScanNet, Stage, default_cascade,
                      draw_scan_weights, draw_weights, paper_stage1, paper_stage2, paper_stage3,
                      uniform_weights, REGION_W, REGION_H, REGION_MARGIN)
from .frames import CONFIGS, config_seed, make_frame, make_stream

__all__ = [
    "ACT_NONE", "ACT_RATIONAL", "ACT_SCALED_TANH", "ACT_TANH", "CONV", "FC",
    "POOL", "Layer", "Stage", "default_cascade", "draw_weights",
    "uniform_weights", "RLayer", "ScanNet", "paper_stage1", "paper_stage2", "paper_stage3", "REGION_W", "REGION_H", "REGION_MARGIN", "draw_scan_weights", "CONFIGS", "config_seed", "make_frame", "make_stream",
]
