// Internal declarations of libcnnc: context, device-side tables and kernel launchers.
// Not part of the public interface (include/cnnc.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <string>
#include <vector>

#include "cnnc.h"

namespace cnnc {

// Network shapes the kernels are specialised for (Section 3.4 of the paper: code written per
// architecture instead of a generic layer stack).
constexpr int kWin = CNNC_WINDOW;          // stage-1 window
constexpr int kS1Params = 409;
constexpr int kS2In = 24, kS2Params = 9633;
constexpr int kS3In = 48, kS3Params = 122977;

// Offsets (in floats) of each layer's weights / biases inside a stage's blob.
namespace s1 { constexpr int W1 = 0, B1 = 36, W2 = 40, B2 = 328, W3 = 336, B3 = 408; }
// Stage 1 as its kernel reads it: the second convolution's kernels in the Winograd F(3,3) domain along their rows,
// U2[k][c][a][5 points] in place of w2[k][c][a][3 taps] (stage1_prepare_weights); everything else as in the blob.
namespace s1p { constexpr int W1 = 0, B1 = 36, U2 = 40, B2 = 520, W3 = 528, B3 = 600; }
constexpr int kS1Prepared = 601;
namespace s2 {
constexpr int W1 = 0, B1 = 200, W2 = 208, B2 = 1360, W3 = 1376, B3 = 9568, W4 = 9600, B4 = 9632;
}
namespace s3 {
constexpr int W1 = 0, B1 = 400, W2 = 416, B2 = 13216, W3 = 13248, B3 = 22464, W4 = 22496, B4 = 122848,
              W5 = 122912, B5 = 122976;
}

// One pyramid level as the kernels see it.
struct LevelDev {
    int32_t w, h;          // level size
    int32_t ow, oh;        // score-map size (w - 11, h - 11)
    int32_t pyr_off;       // first byte of the level in the pyramid buffer
    int32_t score_off;     // first flat window index of the level
    int32_t xmap_off;      // first entry of the level's column table in the tap table
    int32_t ymap_off;      // first entry of the level's row table
    int64_t scale_q16;     // round(scale * 65536)
    double scale;          // scale of the level (frame pixels per level pixel)
    int32_t word_off;      // first word of the level in the survivor bit mask (rows padded to 32 windows)
    int32_t words_per_row; // ceil(ow / 32)
};

// A frame may go through the stages in chunks of pyramid levels (asynchronous mode): at most this many.
constexpr int kMaxLevelChunks = 8;

// Small device-resident counters.
struct Counters {
    int32_t n[4];          // survivors of stage 1, 2, 3 and merged detections (untruncated counts)
    // end[s][k]: length of the stage-(s+1) survivor list once chunk k - 1 has been appended; end[s][0] stays 0, so
    // [end[s][k], end[s][k+1]) is the part of the list that chunk k added
    int32_t end[3][kMaxLevelChunks + 1];
};

// A range [*d_begin, *d_end) of a survivor list, both bounds living on the device.
struct ListRange {
    const int32_t *d_begin, *d_end;
};

// Completed steps of the current frame (cnnc_ctx::progress), for the call-order checks.
enum { DONE_PYR = 1, DONE_S1 = 2, DONE_C1 = 4, DONE_E2 = 8, DONE_C2 = 16, DONE_E3 = 32, DONE_C3 = 64, DONE_MERGE = 128 };

// One pyramid level as the scan of the paper-geometry first stage sees it.
// the scanning window of the paper's own geometry and its step, in level pixels (paper, Section 3.3)
constexpr int kScanWinW = 27, kScanWinH = 31, kScanStep = 4;

struct ScanLevel {
    int32_t w, h;          // level size
    int32_t ow, oh;        // responses per row / rows of responses (0 when the level is below 27 x 31)
    int32_t pyr_off;       // first byte of the level in the pyramid buffer
    int32_t out_off;       // first response of the level in the flat response map
};

struct StepTimer {
    std::vector<hipEvent_t> begin, end;   // recorded pairs not yet read
    std::vector<hipEvent_t> pool;         // events free for reuse
    double ms = 0;
    int calls = 0;
};

struct Stage1Literal;
struct ScanLiteral;
struct SelectLiteral;

}  // namespace cnnc

struct cnnc_ctx {
    int device = 0;
    int act = CNNC_ACT_RATIONAL;
    int max_w = 0, max_h = 0, max_surv = 0;
    cnnc_params params{};
    std::string err;

    // weights on the device: the caller's blobs
    float *d_wt[3] = {nullptr, nullptr, nullptr};
    // stages 2 / 3 on the matrix cores: weights re-ordered into MFMA operand fragments, and the
    // per-window activations handed from the convolution kernel to the fully connected kernel
    float *d_frag[2] = {nullptr, nullptr};
    float *d_feat[2] = {nullptr, nullptr};
    int eval_impl = 3;                        // stage 2 / 3 kernels: 3: matrix cores, stage-3 conv2 by Winograd F(4,5);
                                              // 2: the same with F(2,5); 1: matrix cores, direct sums only;
                                              // 0: direct convolution on the vector ALU

    // geometry of the current frame size / parameters
    bool layout_valid = false;
    int lay_w = 0, lay_h = 0;
    int n_levels = 0;
    std::vector<cnnc::LevelDev> levels;
    int64_t pyr_bytes = 0, n_windows = 0;
    int n_tiles_pyr = 0, n_tiles_s1 = 0;
    int layout_serial = 0;                    // bumped whenever the geometry tables are rebuilt

    // first stage in the paper's geometry (27 x 31 window, 4 pixel step): weights, tables and response map
    float *d_scan_wt = nullptr;
    cnnc::ScanLiteral *scan_literal = nullptr;   // the scan with its weights as instruction literals (or none)
    int scan_act = 0;
    cnnc::ScanLevel *d_scan_levels = nullptr;
    uint32_t *d_scan_tiles = nullptr;
    float *d_scan_map = nullptr;
    int64_t cap_scan_tiles = 0, cap_scan_map = 0, n_scan = 0;
    int n_scan_tiles = 0, scan_serial = -1;
    int scan_tile_request = 0, scan_tile_side = 0;   // responses per tile side: asked for (0 = chosen from the frame) and in use
    bool scan_done = false;

    // the selective unit in that geometry: networks, list of positions above T_1, per-region records and response maps
    float *d_sel_w2 = nullptr, *d_sel_w3 = nullptr;
    cnnc::SelectLiteral *sel_literal = nullptr;  // the unit with its first layers' weights as instruction literals (or none)
    float *d_sel_f2 = nullptr, *d_sel_f3 = nullptr;   // their second convolutions in matrix-operand lane order
    int sel_act = 0, sel_rule = 2;           // decision rule: eq. (2) or the weaker eq. (3)
    uint32_t *d_sel_idx = nullptr;
    float *d_sel_sc = nullptr;
    cnnc_region *d_sel_rec = nullptr;
    float *d_sel_maps = nullptr;             // [2][max_surv][25]
    int32_t *d_sel_cnt = nullptr, *h_sel_cnt = nullptr;   // [0] positions listed, [1] regions accepted, [2] merged detections
    float *d_sel_fsc = nullptr;              // [merge_cap] score of each accepted region
    uint32_t *d_sel_pick = nullptr;          // [merge_cap] its number in the list of regions
    cnnc_rdet *d_sel_det = nullptr;          // [merge_cap] merged detections of the unit
    cnnc_rdet *h_sel_det = nullptr;          // pinned: the first of them, copied back with the counters by the whole-path call
    bool paper_pending = false;              // a cnnc_detect_paper_async pass is enqueued
    bool sel_done = false;

    // device buffers that depend on the layout
    cnnc::LevelDev *d_levels = nullptr;
    uint32_t *d_taps = nullptr;      // column / row tap tables of all levels
    uint32_t *d_tiles_pyr = nullptr; // pyramid kernel: per level, the first level column / row of every frame tile
    int pyr_ntx = 0, pyr_nty = 0;    // frame tiles per row / column of tiles
    uint32_t *d_tiles_s1 = nullptr;  // (level, tile) table of the stage-1 kernel
    uint8_t *d_pyr = nullptr;
    float *d_score1 = nullptr;
    uint32_t *d_mask1 = nullptr;     // stage-1 survivor bits of the fused path, one word per 32 windows of a row
    int64_t cap_pyr = 0, cap_score1 = 0, cap_taps = 0, cap_tiles_pyr = 0, cap_tiles_s1 = 0, cap_mask1 = 0;
    int64_t n_words = 0;
    bool fused_stage1 = false;       // cnnc_detect uses cnnc_stage1_survivors instead of score map + compaction
    cnnc::Stage1Literal *s1_literal = nullptr;   // stage 1 with this context's weights as instruction literals (or none)
    bool use_literals = true;        // cnnc_set_literal_weights

    // survivor lists (capacity max_surv each)
    uint32_t *d_idx[3] = {nullptr, nullptr, nullptr};
    float *d_sc[3] = {nullptr, nullptr, nullptr};
    float *d_eval[2] = {nullptr, nullptr};   // scores of stage 2 / 3, aligned with the previous list
    int32_t *d_blockcnt[3] = {nullptr, nullptr, nullptr};   // compaction of stage 1 / 2 / 3: per-block counts and offsets
    int32_t cap_blocks = 0;
    cnnc::Counters *d_cnt = nullptr;
    cnnc::Counters *h_cnt = nullptr;         // pinned

    // merge
    int merge_cap = 0;
    void *d_merge_ws = nullptr;              // sorted boxes, flags
    cnnc_det *d_det = nullptr;
    cnnc_det *h_det = nullptr;               // pinned

    // current frame
    const uint8_t *d_frame = nullptr;
    int fw = 0, fh = 0, fpitch = 0;
    int progress = 0;                        // bit mask of completed steps for CNNC_E_STATE checks
    hipStream_t last_stream = nullptr;       // stream of the last enqueue; the default stream again once it has been waited for

    // asynchronous mode inside a frame: chunks of pyramid levels, stage 1 of a chunk on the caller's stream while the
    // later stages of earlier chunks run on a stream of the context, ordered by events only
    int async_chunks = 1;                    // 1: the whole frame on the caller's stream
    int n_chunks = 1;                        // chunks of the current layout (<= async_chunks, <= levels)
    int chunk_level[cnnc::kMaxLevelChunks + 1] = {0};   // first level of each chunk, then n_levels
    int chunk_tile[cnnc::kMaxLevelChunks + 1] = {0};    // first stage-1 tile of each chunk, then n_tiles_s1
    hipStream_t side = nullptr;
    hipEvent_t ev_s1[cnnc::kMaxLevelChunks] = {nullptr}, ev_done = nullptr;

    bool timing = false;
    cnnc::StepTimer timers[CNNC_T_COUNT];
};

namespace cnnc {

// blob (kS1Params floats, layout s1) -> what the stage-1 kernels read (kS1Prepared floats, layout s1p)
void stage1_prepare_weights(const float *blob, float *prepared);
// Stage 1 with a prepared weight set written into its code (k_stage1.hip); nullptr when that module does not load.
Stage1Literal *stage1_literal_create(const float *prepared);
void stage1_literal_destroy(Stage1Literal *s);

// Kernel launchers (one translation unit each).  All enqueue on `st` and return the launch status.
hipError_t launch_pyramid(const cnnc_ctx *c, hipStream_t st);
// Stage 1 over tiles [tile_begin, tile_end) of the (level, tile) table (levels are contiguous in it).
hipError_t launch_stage1(const cnnc_ctx *c, int tile_begin, int tile_end, hipStream_t st);
// Stage 1 that keeps only what passes `thr`: one bit per window in d_mask1 and the score of each passing window
// at its place in d_score1 (all other entries of d_score1 are left as they were).
hipError_t launch_stage1_emit(const cnnc_ctx *c, float thr, hipStream_t st);
// Ordered survivor list from d_mask1 / d_score1.
hipError_t launch_compact_mask(const cnnc_ctx *c, uint32_t *out_idx, float *out_sc, int32_t *d_count, hipStream_t st);
// One ordered compaction: the values above `thr` of a source, appended to an output list.
struct CompactJob {
    int slot;                     // which of the context's per-block count buffers to use (0..2: one per stage)
    const float *vals;            // source values
    const uint32_t *src_idx;      // index written for source element e: src_idx[e], or idx_base + e when nullptr
    uint32_t idx_base;
    const int32_t *d_begin, *d_end;   // source = elements [*d_begin, *d_end) clamped to max_surv; d_end == nullptr:
    int64_t n_literal;                // the first n_literal elements
    float thr;
    uint32_t *out_idx;            // output list (capacity max_surv) ...
    float *out_sc;
    const int32_t *d_base;        // ... which already holds *d_base entries (nullptr: none)
    int32_t *d_count, *d_count2;  // receive the new length of the list (d_count2 may be nullptr)
};
hipError_t launch_compact(const cnnc_ctx *c, const CompactJob &job, hipStream_t st);
// Stage 2 / 3 on the entries [*r.d_begin, *r.d_end) of the previous stage's survivor list.
hipError_t launch_eval2(const cnnc_ctx *c, ListRange r, hipStream_t st);
hipError_t launch_eval3(const cnnc_ctx *c, ListRange r, hipStream_t st);
hipError_t launch_eval3_mfma(cnnc_ctx *c, ListRange r, hipStream_t st);
hipError_t launch_eval2_mfma(cnnc_ctx *c, ListRange r, hipStream_t st);

// Brackets the launches made during its lifetime with a pair of events on the stream when the context's
// timing is on; the pair is read back by cnnc_get_timings.
struct ScopedTimer {
    cnnc_ctx *c;
    int step;
    hipStream_t st;
    hipEvent_t b = nullptr;
    ScopedTimer(cnnc_ctx *c_, int step_, hipStream_t st_);
    ~ScopedTimer();
};
// Host helpers shared by the translation units that hold entry points.
int fail(cnnc_ctx *c, int code, const std::string &msg);
int hip_fail(cnnc_ctx *c, hipError_t e, const char *what);
int compute_levels(const cnnc_ctx *c, int w, int h, std::vector<LevelDev> &lv, int64_t &pyr_bytes, int64_t &n_windows);
// Waits for the stream the context last enqueued on and forgets it: from then on the context holds no reference to a
// stream of the caller, who may destroy it.
inline hipError_t wait_last_stream(cnnc_ctx *c)
{
    const hipError_t e = hipStreamSynchronize(c->last_stream);
    c->last_stream = nullptr;
    return e;
}

void scan_release(cnnc_ctx *c);
void select_release(cnnc_ctx *c);
size_t eval2_frag_floats();
size_t eval2_feat_floats();
void eval2_make_fragments(const float *blob, float *frag);
size_t eval3_frag_floats();
size_t eval3_feat_floats();
int eval3_feat_rows(int max_surv);      // windows the stage-3 hand-over buffer holds
void eval3_make_fragments(const float *blob, float *frag);
int64_t eval3_mfma_per_crop(int impl);
int64_t eval2_mfma_per_crop(int impl);
hipError_t launch_merge(const cnnc_ctx *c, hipStream_t st);
size_t merge_workspace_bytes(int merge_cap);
hipError_t merge_init_workspace(const cnnc_ctx *c);
hipError_t launch_merge_regions(const cnnc_ctx *c, float iou, int min_neighbors, hipStream_t st);

constexpr int kCompactBlock = 256;
constexpr int kCompactPerBlock = 2048;   // values handled by one workgroup

// Stage-1 tile (outputs per workgroup) and pyramid tile.
constexpr int kS1TileW = 32, kS1TileH = 16;
constexpr int kPyrTileW = 128, kPyrTileH = 32;   // pyramid: FRAME pixels staged per workgroup

// tile table entry: level in the top 8 bits, tile row in the next 12, tile column in the low 12
inline uint32_t pack_tile(int level, int ty, int tx) { return (uint32_t(level) << 24) | (uint32_t(ty) << 12) | uint32_t(tx); }

}  // namespace cnnc
