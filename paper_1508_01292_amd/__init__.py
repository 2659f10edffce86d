"""MI355X-native hot path of the compact CNN cascade detector (arXiv 1508.01292).

The work is done by hand-written HIP kernels in libcnnc.so (C ABI: include/cnnc.h).  This
package is only the ctypes binding: it marshals arguments and never computes a step itself.
"""
from .binding import (CnncError, Context, Detection, Pipe, lib, library_path, cnnc_build_pyramid,
                      cnnc_compact_survivors, cnnc_create, cnnc_destroy, cnnc_detect, cnnc_detect_async,
                      cnnc_eval_stage, cnnc_fetch_detections, cnnc_merge_detections, cnnc_pyramid_layout,
                      cnnc_measure_peaks, cnnc_set_params, cnnc_stage1_scoremap, cnnc_scan_set_weights, cnnc_select_set_weights, cnnc_select_run, cnnc_select_set_rule, cnnc_select_fetch, cnnc_select_merge, Region, RegionDetection,
                      cnnc_stage1_survivors, cnnc_set_fused_stage1,
                      cnnc_scan_layout, cnnc_scan_scoremap, cnnc_get_scan_scoremap, EXPORTS, STEP_NAMES)

__all__ = ["CnncError", "Context", "Detection", "Pipe", "lib", "library_path", "EXPORTS", "STEP_NAMES",
           "cnnc_create", "cnnc_destroy", "cnnc_set_params", "cnnc_pyramid_layout", "cnnc_build_pyramid",
           "cnnc_stage1_scoremap", "cnnc_compact_survivors", "cnnc_eval_stage", "cnnc_merge_detections",
           "cnnc_detect", "cnnc_detect_async", "cnnc_fetch_detections", "cnnc_measure_peaks",
           "cnnc_stage1_survivors", "cnnc_set_fused_stage1", "cnnc_select_set_weights", "cnnc_select_run", "cnnc_select_fetch", "cnnc_select_set_rule", "cnnc_select_merge", "Region", "RegionDetection", "cnnc_scan_set_weights", "cnnc_scan_layout", "cnnc_scan_scoremap", "cnnc_get_scan_scoremap"]
