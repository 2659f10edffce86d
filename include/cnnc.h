/*
 * cnnc - hot path of the compact CNN cascade detector (Kalinovskii & Spitsyn,
 * "Compact Convolutional Neural Network Cascade for Face Detection") for one
 * AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * The path, in the order of Section 3.3 of the paper:
 *   cnnc_build_pyramid      image pyramid of the frame             (Sections 2, 3.3)
 *   cnnc_stage1_scoremap    first CNN on every window of every     (Section 3.3, first
 *                           pyramid level, fully convolutional      paragraph; Section 3.4)
 *   cnnc_compact_survivors  windows whose response exceeds T_k     (Section 3.3)
 *   cnnc_eval_stage(k)      CNN_2 / CNN_3 on the surviving regions (Section 3.3, selective unit)
 *   cnnc_merge_detections   aggregation of accepted regions        (Section 3.3, last paragraph)
 *   cnnc_detect[_async]     all of the above on one frame; several contexts on several
 *                           streams overlap stages of different frames (Section 3.4,
 *                           asynchronous mode)
 *
 * Conventions
 *   - Every function returns CNNC_OK (0) or a negative CNNC_E_* code; nothing throws or aborts.
 *     cnnc_last_error() gives a text for the last failure on that context.
 *   - "device" pointers are HIP device memory on the context's GPU; "host" pointers are ordinary
 *     memory.  The caller owns the frame and the output arrays; the context owns everything else
 *     and only lends read-only device pointers through the cnnc_get_* calls (valid until the next
 *     call that changes the frame size or parameters, or cnnc_destroy).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued on
 *     it and not waited for, except where a function says it synchronises.  A context remembers the
 *     stream of its last enqueue until a call that waits for it (cnnc_merge_detections,
 *     cnnc_fetch_detections, cnnc_detect, cnnc_survivor_count on that stream, cnnc_select_fetch,
 *     cnnc_select_merge, cnnc_fetch_paper, cnnc_detect_paper); after such a call the stream may be destroyed.
 *   - Calls on one context must not overlap in time; use one context per stream / thread.
 *   - The flat window index g orders all stage-1 windows of a frame by (level, y, x):
 *     g = score_off[level] + y * (lvl_w[level] - 11) + x.
 *   - The three networks are the fixed shapes listed at cnnc_create; kernels are specialised for
 *     them (Section 3.4: no generic layer stack).
 */
#ifndef CNNC_H
#define CNNC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CNNC_OK          0
#define CNNC_E_INVAL    -1  /* bad argument (null pointer, size, stage index, unsupported network shape) */
#define CNNC_E_NOMEM    -2  /* host or device allocation failed */
#define CNNC_E_OVERFLOW -3  /* a survivor or detection list did not fit; contents up to the capacity are valid, and the
                               steps after a truncated list ran on the truncated list */
#define CNNC_E_HIP      -4  /* a HIP runtime call failed */
#define CNNC_E_STATE    -5  /* call out of order (e.g. score map before pyramid) */
#define CNNC_E_TOOBIG   -6  /* input larger than the fixed scratch of cnnc_compact_noalloc (CNNC_NOALLOC_MAX_VALUES) */

#define CNNC_WINDOW      12 /* side of the stage-1 window */
#define CNNC_MAX_LEVELS  64

enum { CNNC_CONV = 0, CNNC_POOL = 1, CNNC_FC = 2 };
/* Activations.  1 is the paper's: f(x) = 1.7159 * t(2x/3) with the rational t of eq. (1).
 * 2 is the same with the exact tanh; 3 is plain tanh(x); 0 is the identity (output layers). */
enum { CNNC_ACT_NONE = 0, CNNC_ACT_RATIONAL = 1, CNNC_ACT_SCALED_TANH = 2, CNNC_ACT_TANH = 3 };

typedef struct cnnc_ctx cnnc_ctx;

/* One layer.  CONV: k x k "valid" convolution, stride 1.  POOL: 2x2 max, stride 2 (Section 3.1).
 * FC: fully connected over a cin x k x k input map, features ordered [channel][row][col]. */
typedef struct {
    int32_t kind, cin, cout, k, act;
} cnnc_layer;

/* One network.  weights: host pointer, float32; for every CONV / FC layer in order:
 * w[cout][cin][k][k] then bias[cout].  Copied by cnnc_create. */
typedef struct {
    int32_t in_size;
    int32_t n_layers;
    const cnnc_layer *layers;
    const float *weights;
} cnnc_stage_desc;

/* Search parameters (Section 4.1: minSize, scaleFactor, T_1, T_2; Section 4.2: minNeighbors). */
typedef struct {
    double min_face;        /* smallest face side in frame pixels, >= 12; level-0 scale = min_face / 12 */
    double scale_step;      /* > 1; scale ratio between consecutive pyramid levels */
    float thr[3];           /* a window passes stage k iff its score > thr[k-1] (fp32, strict) */
    float merge_iou;        /* boxes with intersection-over-union above this are merged (0.3) */
    int32_t min_neighbors;  /* a merged box is reported iff it absorbed >= min_neighbors - 1 others */
} cnnc_params;

/* One detection in frame pixels.  index = flat window index g of the kept window. */
typedef struct {
    int32_t x, y, size;
    float score;            /* stage-3 score of the kept window */
    int32_t level;
    int32_t neighbors;      /* boxes it absorbed */
    int32_t index;
    int32_t reserved;
} cnnc_det;

/* Names of the timed steps for cnnc_get_timings. */
enum {
    CNNC_T_PYRAMID = 0, CNNC_T_STAGE1, CNNC_T_COMPACT1, CNNC_T_STAGE2, CNNC_T_COMPACT2,
    CNNC_T_STAGE3, CNNC_T_COMPACT3, CNNC_T_MERGE,
    /* the convolution kernel alone inside cnnc_eval_stage(2) / (3) (the step also runs a small fc kernel) */
    CNNC_T_STAGE2_CONV, CNNC_T_STAGE3_CONV,
    CNNC_T_SCAN,            /* cnnc_scan_scoremap */
    CNNC_T_SELECT,          /* cnnc_select_run */
    CNNC_T_COUNT
};

/* Create a context on the current HIP device.
 * stages[3]: the networks.  Supported shapes (anything else -> CNNC_E_INVAL):
 *   stage 1: 12x12 | conv3 1->4, pool, conv3 4->8, fc 8x3x3->1
 *   stage 2: 24x24 | conv5 1->8, pool, conv3 8->16, pool, fc 16x4x4->32, fc 32->1
 *   stage 3: 48x48 | conv5 1->16, pool, conv5 16->32, pool, conv3 32->32, fc 32x7x7->64, fc 64->1
 *   hidden layers all use one activation kind (1, 2 or 3), output layers kind 0.
 * max_w, max_h: largest frame accepted.  max_survivors (<= 2^20): capacity of every survivor list
 * (stage 1, 2 and 3) and of the merge input.  Allocates device memory (hipMalloc). */
int cnnc_create(cnnc_ctx **out, const cnnc_stage_desc stages[3], int max_w, int max_h, int max_survivors);
int cnnc_destroy(cnnc_ctx *ctx);

/* Set search parameters.  May reallocate pyramid buffers on the next frame. */
int cnnc_set_params(cnnc_ctx *ctx, const cnnc_params *p);

/* Host only, no GPU work.  Pyramid geometry for a w x h frame under the current parameters:
 * scale s_0 = min_face / 12, s_{l+1} = s_l * scale_step; level size floor(w / s_l + 1e-9) by
 * floor(h / s_l + 1e-9); levels end before the first with a side below 12.
 * Arrays (host, capacity CNNC_MAX_LEVELS; any may be NULL): lvl_w, lvl_h, lvl_scale,
 * pyr_off (byte offset of level l in the pyramid buffer, n_levels + 1 entries),
 * score_off (offset of level l in the flat window index, n_levels + 1 entries).
 * CNNC_E_INVAL if the frame exceeds max_w x max_h or has no level. */
int cnnc_pyramid_layout(cnnc_ctx *ctx, int w, int h, int *n_levels, int32_t *lvl_w, int32_t *lvl_h,
                        double *lvl_scale, int64_t *pyr_off, int64_t *score_off);

/* Resample every pyramid level from the frame (not level to level), bilinear with 8-bit weights:
 * sample position f = (i + 0.5) * s - 0.5 clamped to the frame, right/lower weight
 * q = round(frac * 256), pixel = (sum of the four pixel * weight products + 32768) >> 16.
 * d_frame: device, uint8 [h][pitch] (pitch >= w bytes).  Result: uint8 levels, row pitch = level width. */
int cnnc_build_pyramid(cnnc_ctx *ctx, const uint8_t *d_frame, int w, int h, int pitch, void *stream);

/* Score of every 12x12 window (stride 1, fully inside a level) of every level, fp32, in flat
 * window order.  Pixels enter the network as (p - 128) / 128.  Needs cnnc_build_pyramid first. */
int cnnc_stage1_scoremap(cnnc_ctx *ctx, void *stream);

/* cnnc_stage1_scoremap and cnnc_compact_survivors(1, thr) in one step that never writes the score map (the
 * paper's detector hands only the coordinates of windows above T_1 to the next unit, Section 3.3): the stage-1
 * kernel keeps one bit per window and the scores of the passing windows, and the ordered list is built from
 * those.  Leaves exactly the stage-1 survivor list of the two-call path (same order, same fp32 scores);
 * afterwards cnnc_get_scoremap reports CNNC_E_STATE.  Needs cnnc_build_pyramid first.
 * cnnc_set_fused_stage1(on): cnnc_detect / cnnc_detect_async take this step instead of the two calls. */
int cnnc_stage1_survivors(cnnc_ctx *ctx, float thr, void *stream);
int cnnc_set_fused_stage1(cnnc_ctx *ctx, int on);

/* stage = 1, 2 or 3: list the windows with score_stage > thr, in ascending flat index.
 * Stage 1 reads the score map; stage k > 1 reads the scores cnnc_eval_stage(k) left for the
 * survivors of stage k - 1.  The count stays on the device; lists longer than max_survivors are
 * truncated and reported by cnnc_survivor_count / cnnc_merge_detections as CNNC_E_OVERFLOW. */
int cnnc_compact_survivors(cnnc_ctx *ctx, int stage, float thr, void *stream);

/* The compaction of cnnc_compact_survivors for callers that cannot allocate device memory: code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  No context: the caller passes the input and
 * the outputs, and the per-workgroup counts the kernels need in between live in a fixed 32 KiB array inside the
 * library's device image (one copy per GPU, held until the process ends).  The call makes no hipMalloc / hipFree and
 * no allocating library call; it only launches kernels (no memset nodes), so it may be captured into a graph.
 *   d_values: device, n float32 (n >= 0).  Lists, in ascending order, the positions i with d_values[i] > thr (fp32,
 *   strict): d_index[k] = i, d_score[k] = d_values[i] for the first `cap` of them (device arrays of capacity cap),
 *   and *d_count (device) = their untruncated number.  Enqueued on `stream` of the current device, not waited for.
 *   Same kernels and same result, bit for bit, as cnnc_compact_survivors(1) on the same values.
 * CNNC_E_TOOBIG when n > CNNC_NOALLOC_MAX_VALUES (nothing is launched); CNNC_E_INVAL for null pointers, negative
 * sizes or a NaN threshold; CNNC_E_HIP when the array's address cannot be obtained or a launch fails.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or threads)
 * race and must be serialised by the caller.  Nothing in the array has to start at zero. */
#define CNNC_NOALLOC_MAX_VALUES (1 << 24)
int cnnc_compact_noalloc(const float *d_values, int64_t n, float thr, uint32_t *d_index, float *d_score, int32_t cap,
                         int32_t *d_count, void *stream);

/* k = 2 or 3: for every survivor of stage k - 1 cut its window rectangle
 * [x s, (x + 12) s) x [y s, (y + 12) s) from the frame given to cnnc_build_pyramid (which must
 * still be alive and unchanged), resample it to the network's input size (16.16 fixed point,
 * 8-bit weights) and run network k.  One fp32 score per survivor. */
int cnnc_eval_stage(cnnc_ctx *ctx, int k, void *stream);

/* Greedy merge of the stage-3 survivors: boxes X = round(x s), Y = round(y s), side = round(12 s);
 * in order of descending score (ties: ascending flat index) a box not yet absorbed is kept and
 * absorbs every later box with intersection > merge_iou * union.  Kept boxes with fewer than
 * min_neighbors - 1 absorbed boxes are dropped.  Synchronises the stream.
 * out: host array of capacity cap, kept order.  *n_out: number of kept boxes (may exceed cap ->
 * CNNC_E_OVERFLOW, first cap valid). */
int cnnc_merge_detections(cnnc_ctx *ctx, cnnc_det *out, int cap, int *n_out, void *stream);

/* The whole path on one frame with the context's thresholds.  cnnc_detect synchronises and
 * returns the detections; cnnc_detect_async only enqueues on `stream` and
 * cnnc_fetch_detections later waits for that work and returns its detections. */
int cnnc_detect(cnnc_ctx *ctx, const uint8_t *d_frame, int w, int h, int pitch, cnnc_det *out, int cap,
                int *n_out);
int cnnc_detect_async(cnnc_ctx *ctx, const uint8_t *d_frame, int w, int h, int pitch, void *stream);
int cnnc_fetch_detections(cnnc_ctx *ctx, cnnc_det *out, int cap, int *n_out);

/* Asynchronous mode inside a frame (Section 3.4: the first stage moves on to the next pyramid level while the regions
 * it has found are still being analysed).  chunks = 1 (default): cnnc_detect / cnnc_detect_async run every step on
 * the caller's stream.  chunks = 2..8: the pyramid levels are cut into that many runs of consecutive levels with
 * about equal numbers of windows (fewer when the frame has fewer levels); stage 1 and its compaction go chunk by
 * chunk on the caller's stream, stages 2 and 3 of a chunk start on a second stream as soon as that chunk's survivors
 * are listed, ordered by HIP events only; the merge follows the last chunk and the caller's stream then waits for it,
 * so the call keeps its contract (work enqueued, cnnc_fetch_detections waits).  Survivor lists and detections are
 * exactly those of chunks = 1.  The second stream belongs to the context (default priority; it exists while chunks > 1: the call that sets chunks > 1 creates it, the call that sets 1 waits for it and destroys it).  On one GPU whose later
 * stages already fill the chip the overlap buys less than the extra launches and cross-stream waits cost, so 1 is
 * the default; the mode is there for cascades whose first stage dominates, as in the paper.
 * Ignored (one stream) with cnnc_set_eval_impl(0) or cnnc_set_fused_stage1(1), and inside cnnc_pipe graphs. */
int cnnc_set_async_chunks(cnnc_ctx *ctx, int chunks);

/* Read-only device views for tests and callers that chain their own kernels. */
int cnnc_get_pyramid(cnnc_ctx *ctx, const uint8_t **d_pyramid, int64_t *n_bytes);
int cnnc_get_scoremap(cnnc_ctx *ctx, const float **d_scores, int64_t *n_windows);
/* stage = 1..3: d_index[i] = flat window index, d_score[i] = that stage's score, ascending index. */
int cnnc_get_survivors(cnnc_ctx *ctx, int stage, const uint32_t **d_index, const float **d_score);
/* Scores cnnc_eval_stage(k) produced, aligned with the survivor list of stage k - 1. */
int cnnc_get_stage_scores(cnnc_ctx *ctx, int k, const float **d_score);
/* Waits for `stream`, then returns the survivor count of a stage (CNNC_E_OVERFLOW if it was truncated;
 * *n then holds the untruncated count). */
int cnnc_survivor_count(cnnc_ctx *ctx, int stage, int *n, void *stream);

/* Per-step GPU time.  With timing on, every path call brackets its kernels with HIP events on the
 * caller's stream; cnnc_get_timings waits for them and returns milliseconds summed since the last
 * reset and the number of calls per step (host arrays of CNNC_T_COUNT entries), then resets. */
int cnnc_set_timing(cnnc_ctx *ctx, int on);
int cnnc_get_timings(cnnc_ctx *ctx, double *ms_sum, int32_t *calls);

/* Which kernels cnnc_eval_stage uses.  3 (default): implicit-GEMM kernels on the matrix cores (fp32 MFMA) with the
 * 5x5, 16 -> 32 convolution of stage 3 evaluated by the Winograd minimal-filtering algorithm F(4,5) along rows and its
 * 3x3, 32 -> 32 convolution by F(2,3), and the 3x3, 8 -> 16 convolution of stage 2 by F(4,3); 2: F(2,5) for the 5x5
 * convolution of stage 3, F(2,3) for its 3x3 one, direct sums in stage 2; 1: the matrix-core kernels with
 * direct sums only; 0: direct convolution on the vector ALU.  Same results within fp32 rounding (about 1e-6 on a
 * score); kept so that the choice stays measurable (the paper's Section 3.4 argues for code specialised per network
 * and processor). */
int cnnc_set_eval_impl(cnnc_ctx *ctx, int impl);

/* ---- First stage in the paper's own geometry -------------------------------------------------
 * Section 3.1: CNN_1 has no fully connected layer, convolution stride 1, pooling stride 2; Section 3.3: the
 * responses of its output layer correspond to a 27 x 31 (width x height) window moved over each pyramid
 * image with a 4 pixel step.  The layer shapes were printed only in the paper's Figure 1; built in here:
 *   conv 4x4 1->4, f, pool 2 | conv 3x3 4->11, f, pool 2 | conv 5x6 (w x h) 11->1 (linear)   = 806 parameters
 * (the paper states 797).  This scan is a second reader of the pyramid beside cnnc_stage1_scoremap; it does
 * not feed the later stages.
 *
 * cnnc_scan_set_weights: weights = host pointer to n_floats = 806 float32, per conv layer w[cout][cin][kh][kw]
 *   then bias[cout]; act = hidden activation kind (1, 2 or 3).  Copied to the device; synchronises.
 * cnnc_scan_layout: host only.  For a w x h frame under the current parameters: out_w[l] x out_h[l] responses on
 *   level l (0 x 0 when the level is smaller than the window), out_off[l] = first response of level l in the flat
 *   map, out_off[n_levels] = their total.  Arrays: host, capacity CNNC_MAX_LEVELS (+ 1 for out_off), may be NULL.
 * cnnc_scan_scoremap: needs cnnc_build_pyramid first (CNNC_E_STATE otherwise) and the weights.  Response (j, i)
 *   of level l is the network on the window whose corner is pixel (4 i, 4 j) of that level, pixels entering as
 *   (p - 128) / 128; fp32, flat order (level, row, column).  Enqueued on `stream`.
 * cnnc_get_scan_scoremap: device view of that map and its length.
 * cnnc_scan_set_tile: the scan kernel has two builds, a workgroup per 8 x 8 or per 16 x 16 tile of responses (the
 *   larger tile computes less of the border that neighbouring tiles compute again; the smaller one gives more workgroups
 *   on a small frame).  side = 0 (the default): chosen from the frame, 16 when that gives at least 128 tiles; 8 or 16:
 *   that build.  Both builds sum every response in the same order and give the same bits.  Anything else:
 *   CNNC_E_INVAL.  cnnc_scan_tile returns the side the last cnnc_scan_scoremap used (0 before the first). */
int cnnc_scan_set_weights(cnnc_ctx *ctx, const float *weights, int n_floats, int act);
int cnnc_scan_layout(cnnc_ctx *ctx, int w, int h, int *n_levels, int32_t *out_w, int32_t *out_h, int64_t *out_off);
int cnnc_scan_scoremap(cnnc_ctx *ctx, void *stream);
int cnnc_get_scan_scoremap(cnnc_ctx *ctx, const float **d_scores, int64_t *n);
int cnnc_scan_set_tile(cnnc_ctx *ctx, int side);
int cnnc_scan_tile(cnnc_ctx *ctx);

/* ---- The selective unit in the paper's geometry -----------------------------------------------
 * Section 3.3: a window position whose first-stage response exceeded T_1 is read from the original image together
 * with a neighbourhood and scaled to 51 x 55 pixels; its histogram is equalised; the region and its mirror image
 * (reflection about the vertical axis) go through CNN_2 and CNN_3, each giving a 5 x 5 response map; with K2, K3 the
 * numbers of responses above the threshold, rule (2) decides: face = (K2 >= T_nn and K3 > 0) or (K2 > 0 and
 * K3 >= T_nn); under that rule a region with K2 = 0 is not shown to CNN_3.
 * What the paper leaves open is fixed as follows: neighbourhood = 12 level pixels on every side of the 27 x 31 window;
 * region samples in 16.16 fixed point with 8-bit weights, rounded to uint8; equalisation v -> round((cdf(v) - c0) * 255
 * / (n - c0)) with c0 the cdf of the smallest value present (a constant region is left alone); networks
 * conv 4x4 1->c1, f, pool 2 | conv 3x3 c1->c2, f, pool 2 | conv 7x8 (w x h) c2->1 on a 35 x 39 window at step 4, with
 * (c1, c2) = (4, 19) for CNN_2 (1836 parameters; the paper: 1819) and (5, 28) for CNN_3 (2942; the paper: 2923); a
 * window's response is the mean of response (v, u) of the region and response (v, 4 - u) of the mirror image.
 *
 * cnnc_select_set_weights: host blobs (per conv layer w[cout][cin][kh][kw] then bias[cout]), n2 = 1836, n3 = 2942,
 *   act = hidden activation kind; copied; synchronises; allocates the unit's buffers on first use.
 * cnnc_select_set_rule: rule = 2 (default) is eq. (2) above; rule = 3 the weaker rule of Section 4.3, eq. (3):
 *   face = K2 >= T_nn or K3 >= T_nn (more recall, less precision).  CNN_3's count alone can accept a region there, so
 *   under rule 3 CNN_3 runs on every listed region, whatever K2 is.
 *   Applies to later cnnc_select_run calls; CNNC_E_INVAL for another value.
 * cnnc_select_run: needs cnnc_scan_scoremap of the current frame (CNNC_E_STATE otherwise), whose frame must still be
 *   alive.  Lists the positions with response > t1 in ascending flat order and runs the unit on each; K2 counts
 *   responses > t2, K3 responses > t3 (fp32, strict).  Enqueued on `stream`.
 * cnnc_select_fetch: waits, then returns one record per listed position, in that order (out: host, capacity cap;
 *   *n_out = their number, CNNC_E_OVERFLOW rules as for detections).  maps2 / maps3: optional host arrays of
 *   cap x 25 floats receiving the combined response maps (row-major 5 x 5; maps3 is zero where CNN_3 was not run). */
typedef struct {
    int32_t index;          /* flat index of the position in the response map of cnnc_scan_scoremap */
    int32_t level, i, j;    /* pyramid level, column and row of the position (window corner = pixel (4 i, 4 j)) */
    int32_t k2, k3;         /* responses above the threshold in the 5 x 5 maps of CNN_2 and CNN_3 */
    int32_t face;           /* decision by rule (2), or rule (3) when selected */
    float response;         /* first-stage response of the position */
} cnnc_region;
int cnnc_select_set_weights(cnnc_ctx *ctx, const float *w2, int n2, const float *w3, int n3, int act);
int cnnc_select_set_rule(cnnc_ctx *ctx, int rule);
int cnnc_select_run(cnnc_ctx *ctx, float t1, float t2, float t3, int t_nn, void *stream);
int cnnc_select_fetch(cnnc_ctx *ctx, cnnc_region *out, int cap, int *n_out, float *maps2, float *maps3);

/* Merging of the regions the unit accepted (Section 3.3: non-maximum suppression aggregates the found regions;
 * Section 4.2: minNeighbors), by the greedy rule of cnnc_merge_detections on rectangles.  What the paper leaves open:
 * an accepted region (face != 0) enters as its 27 x 31 window in frame pixels, x = round(4 i s), y = round(4 j s),
 * w = round(27 s), h = round(31 s) with s the scale of its level, and with the largest of its 25 combined CNN_3
 * responses as score (ties: ascending flat position).  A kept rectangle absorbs every later one whose intersection
 * exceeds iou * union; kept rectangles with neighbors + 1 < min_neighbors are dropped.
 * Needs cnnc_select_run of the current frame (CNNC_E_STATE otherwise).  Enqueued on `stream`, then waits.
 * out: host array of capacity cap, kept order; *n_out = number of detections.  CNNC_E_OVERFLOW when the accepted
 * regions exceed the merge capacity (min(max_survivors, 32768)) or the detections exceed cap (first cap are valid).
 * Uses the merge workspace of the context: do not overlap with cnnc_merge_detections / cnnc_detect of the same context. */
typedef struct {
    int32_t x, y, w, h;     /* frame pixels */
    float score;            /* largest combined CNN_3 response of the region */
    int32_t level;          /* pyramid level of the region */
    int32_t neighbors;      /* regions it absorbed */
    int32_t index;          /* flat index of its position in the response map of cnnc_scan_scoremap */
} cnnc_rdet;
int cnnc_select_merge(cnnc_ctx *ctx, float iou, int min_neighbors, cnnc_rdet *out, int cap, int *n_out, void *stream);

/* The whole path in the paper's geometry on one frame (Section 3.3, in its order): cnnc_build_pyramid,
 * cnnc_scan_scoremap, cnnc_select_run, and the merge of cnnc_select_merge, with counts staying on the device between
 * the steps.  Needs cnnc_scan_set_weights and cnnc_select_set_weights (CNNC_E_STATE otherwise); the rule is the one set
 * by cnnc_select_set_rule; pyramid parameters are the context's (cnnc_set_params: min_face maps to the 12-pixel base
 * of the pyramid as for the other path).  cnnc_detect_paper synchronises and returns the detections (host array `out`
 * of capacity cap, kept order; *n_out = their number; CNNC_E_OVERFLOW rules as for cnnc_select_merge);
 * cnnc_detect_paper_async only enqueues on `stream`, and cnnc_fetch_paper later waits for that work and returns its
 * detections.  The frame must stay alive and unchanged until then.  Uses the context's merge workspace. */
typedef struct {
    float t1, t2, t3;       /* thresholds of the scan and of the two response maps (fp32, strict) */
    int32_t t_nn;           /* T_nn of the decision rule, >= 1 */
    float merge_iou;        /* 0.3 */
    int32_t min_neighbors;  /* >= 1 */
} cnnc_paper_params;
int cnnc_detect_paper(cnnc_ctx *ctx, const uint8_t *d_frame, int w, int h, int pitch, const cnnc_paper_params *p,
                      cnnc_rdet *out, int cap, int *n_out);
int cnnc_detect_paper_async(cnnc_ctx *ctx, const uint8_t *d_frame, int w, int h, int pitch, const cnnc_paper_params *p,
                            void *stream);
int cnnc_fetch_paper(cnnc_ctx *ctx, cnnc_rdet *out, int cap, int *n_out);

/* ---- Frame ingest from host memory ------------------------------------------------------------
 * The paper's detector is fed video (Section 4.2) and overlaps its stages (Section 3.4, asynchronous mode).
 * A pipe is a ring of `depth` slots (1..16), each a pinned host frame (w * h bytes, row pitch w) and a device frame,
 * feeding min(depth, 3) lanes, each a context with a HIP stream of its own (not synchronising with the default stream);
 * the host-to-device copies are enqueued on the device's default stream, whose hardware queue no lane shares (work the
 * caller puts on the default stream delays them, nothing else).  Up to `depth` frames are in flight: at most one per lane is being processed (or keeps its results in
 * the lane's context until fetched), the others are copied in and start when a fetch frees a lane.  So with
 * depth = lanes + 1 the copy of the next frame is hidden behind the kernels of the others (more compute streams than
 * three share hardware queues on this GPU and lower the throughput).  use_graph != 0: from a lane's second frame on,
 * a frame's kernels + read-back run as one captured HIP graph launch (one graph per slot and lane; the copy in front of
 * it stays a plain asynchronous copy, which the DMA engine carries out).  All frames of a pipe have the size given at
 * creation.  One thread per pipe.  Memory: min(depth, 3) contexts plus depth device and pinned frames.
 *
 * cnnc_pipe_frame_buffer: the pinned buffer the next submit will send (that of the free slot that has been free
 *   longest), for producers that write frames in place; valid until the next submit or fetch.  CNNC_E_STATE when
 *   every slot is in flight.
 * cnnc_pipe_submit: h_frame = NULL or the pointer from cnnc_pipe_frame_buffer: send the buffer as it is; any other
 *   host pointer: its w x h bytes (row pitch `pitch`) are copied into the buffer first.  Enqueues and returns a
 *   ticket; CNNC_E_STATE when every slot is in flight.
 * cnnc_pipe_submit_device: the same for a frame that is in device memory already (w x h bytes, row pitch `pitch`):
 *   nothing is copied.  The frame must be complete when the call is made (written by work the caller has waited
 *   for) and stay unchanged until its ticket is fetched; it takes a slot like any other frame.  With use_graph the path
 *   is captured per (frame address, pitch, lane) and replayed whenever that address comes again (48 such graphs are
 *   kept; frames at further addresses run without one).
 * cnnc_pipe_fetch: waits for the frame with that ticket and returns its detections like cnnc_detect
 *   (CNNC_E_OVERFLOW rules included); frees the slot and starts the frame that has waited longest for a lane.  Tickets
 *   may be fetched in any order: if the frame still waits for a lane, the results of frames submitted earlier are taken
 *   out of their lanes into host memory (and handed out when their tickets are fetched) until it has run.
 * cnnc_pipe_set_params: for every lane; CNNC_E_STATE while frames are in flight.
 * cnnc_pipe_set_paper: from now on submit runs the path in the paper's geometry (cnnc_detect_paper_async: pyramid,
 *   27x31 scan, selective unit, merge; Section 3.3) instead of the cascade of cnnc_detect_async.  Arguments as for
 *   cnnc_scan_set_weights, cnnc_select_set_weights, cnnc_select_set_rule and cnnc_detect_paper, applied to every
 *   lane; the host arrays are copied.  CNNC_E_STATE while frames are in flight.  Results then come through
 *   cnnc_pipe_fetch_paper (as cnnc_fetch_paper; cnnc_pipe_fetch answers CNNC_E_STATE on such a pipe and
 *   cnnc_pipe_fetch_paper on any other). */
typedef struct cnnc_pipe cnnc_pipe;
int cnnc_pipe_create(cnnc_pipe **out, const cnnc_stage_desc stages[3], int w, int h, int max_survivors, int depth,
                     int use_graph);
int cnnc_pipe_destroy(cnnc_pipe *pipe);
int cnnc_pipe_set_params(cnnc_pipe *pipe, const cnnc_params *p);
int cnnc_pipe_frame_buffer(cnnc_pipe *pipe, uint8_t **h_frame);
int cnnc_pipe_submit(cnnc_pipe *pipe, const uint8_t *h_frame, int pitch, int64_t *ticket);
int cnnc_pipe_submit_device(cnnc_pipe *pipe, const uint8_t *d_frame, int pitch, int64_t *ticket);
int cnnc_pipe_fetch(cnnc_pipe *pipe, int64_t ticket, cnnc_det *out, int cap, int *n_out);
int cnnc_pipe_set_paper(cnnc_pipe *pipe, const float *scan_weights, int n_scan, int scan_act, const float *w2, int n2,
                        const float *w3, int n3, int select_act, int rule, const cnnc_paper_params *p);
int cnnc_pipe_fetch_paper(cnnc_pipe *pipe, int64_t ticket, cnnc_rdet *out, int cap, int *n_out);
const char *cnnc_pipe_last_error(const cnnc_pipe *pipe);

/* Weights as instruction literals (Section 3.4: the code is written for the network it runs).  The kernels whose weights
 * are the same for every lane of a wave (stage 1; with cnnc_scan_set_weights the 27x31 scan; with
 * cnnc_select_set_weights the first layers of CNN_2 and CNN_3 in the selective unit) exist in a second build in which
 * those weights are 32-bit literals of the multiply-add instructions instead of values loaded from memory (such
 * instructions issue at up to twice the rate on this GPU).  cnnc_create and the two set_weights calls write the
 * context's weights into a copy of that code and load it; the calls that run those kernels then use it.  Results are
 * bit-identical to the kernels that read their weights from memory.  cnnc_set_literal_weights(ctx, 0) switches to
 * those, 1 (default) back; cnnc_literal_weights returns 1 when the literal build of stage 1 is in use, 0 when it is
 * switched off or could not be loaded at creation (the context then works as with 0).  Host only. */
int cnnc_set_literal_weights(cnnc_ctx *ctx, int on);
int cnnc_literal_weights(const cnnc_ctx *ctx);

/* Measurement aid: how many 16x16x4 fp32 matrix instructions (1024 multiply-adds each) the convolution kernel of
 * cnnc_eval_stage(k), k = 2 or 3, issues per crop under the current cnnc_set_eval_impl choice, padded tiles and the
 * Winograd forms included (0 for the vector-ALU kernels).  Lets a benchmark report the executed matrix work beside
 * the algorithmic work of the layer definitions.  Host only. */
int cnnc_executed_mfma(const cnnc_ctx *ctx, int k, int64_t *per_crop);

/* Measurement aid for benchmarks: what this GPU sustains on three synthetic probes (dense fp32 MFMA loop,
 * fp32 FMA loop on the vector ALU, 1 GiB device-to-device copy counted as read + write).  Runs on the
 * current device's default stream, allocates and frees 2 GiB, synchronises.  Outputs are host pointers. */
int cnnc_measure_peaks(double *mfma_f32_tflops, double *valu_f32_tflops, double *hbm_copy_gbs);

/* Measurement aids behind two design choices (weights as literals; the lane orders of LDS reads).  Both run small probe
 * kernels on the current device's default stream and synchronise; outputs are host pointers.
 * cnnc_measure_issue_rates: ns per wave instruction and SIMD, four waves per SIMD issuing the same instruction back to
 *   back on independent registers, into ns[0 .. min(n, 4)): [0] v_fmac_f32 with vector-register operands, [1] with one
 *   operand in a scalar register, [2] with a 32-bit literal operand, [3] v_rcp_f32.
 * cnnc_measure_lds_read: ns per wave instruction and compute unit of ds_read_b32 / _b64 / _b128 (width = 1, 2, 4
 *   dwords) when lane l reads at dword address addr[l] of the workgroup's LDS (addr[l] < 0: lane inactive; otherwise a
 *   multiple of width and at most 8704; CNNC_E_INVAL else), sixteen waves per compute unit issuing such reads back to back. */
int cnnc_measure_issue_rates(double *ns, int n);
int cnnc_measure_lds_read(const int32_t *addr, int width, double *ns_per_instruction);

/* For bindings: sizes in bytes of cnnc_layer, cnnc_stage_desc, cnnc_params, cnnc_det, cnnc_region, the value of
 * CNNC_T_COUNT, and the size of cnnc_rdet, in that order, into out[0 .. n) (host; at most seven are written).
 * Returns how many exist (7). */
int cnnc_abi_sizes(int32_t *out, int n);

const char *cnnc_last_error(const cnnc_ctx *ctx);
const char *cnnc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CNNC_H */
