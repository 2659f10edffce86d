/*
 * CPU oracle for the compact CNN cascade detector hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, definition-level
 * implementation that the HIP library is checked against.  It shares no code,
 * header, table or helper with the HIP library, and nothing in the product
 * path may call it.  Only the tests, the smoke check and the benchmark's
 * "cpu_baseline" leg load it.
 *
 * Everything floating point is computed in double (weights are given as
 * float32 and widened).  Everything that decides an integer (pyramid pixels,
 * crop samples, survivor sets, box merging) is integer arithmetic or an fp32
 * comparison, stated at each function.
 *
 * What follows the paper and what is a reading of a point the paper leaves
 * open is said at each function: "paper" cites a section / equation of
 * Kalinovskii & Spitsyn, "reading" marks a choice made for this build.
 *
 * Parity pins (tests/test_oracle_*.py): eq. (1) error bound, closed forms on
 * constant windows, hand-computed one-hot windows, library convolution,
 * per-window definition vs dense evaluation, translation equivariance,
 * threshold monotonicity, exact special cases of the resampling, merge
 * special cases; for the first stage in the paper's own geometry (end of
 * this file): library convolution on windows and whole levels, a
 * hand-computed one-hot window, definition vs single pass, translation by
 * one step; for the selective unit in that geometry: exact special cases and
 * library bilinear for the region, closed forms of histogram equalisation,
 * library convolution for the mirrored response maps, the truth tables of
 * eq. (2) and eq. (3), and the merge of the accepted rectangles against the square merge
 * and a brute force in exact fractions.  The choice of the readings
 * themselves (resampling convention, crop rectangle, merge rule; in the
 * paper's geometry the layer shapes, the width of the neighbourhood, the
 * equalisation rule, how the mirror image's responses are combined, and the
 * box and the score an accepted region enters the merge with) cannot be
 * pinned to the authors' detector: parity unpinned for those choices.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_CONV = 0, ORC_POOL = 1, ORC_FC = 2 };
enum { ORC_ACT_NONE = 0, ORC_ACT_RATIONAL = 1, ORC_ACT_SCALED_TANH = 2, ORC_ACT_TANH = 3 };

typedef struct {
    int32_t kind; /* ORC_CONV, ORC_POOL, ORC_FC */
    int32_t cin, cout;
    int32_t k;   /* kernel side; FC: side of its input map */
    int32_t act; /* ORC_ACT_* applied to the output */
} orc_layer;

/* Threads the parallel loops below will use (for reporting timings), and a   */
/* way to set that number (the benchmark reports one-thread and all-core      */
/* timings of the same routines).                                             */
void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------ */
/* Activation.  Paper, Section 3.1, eq. (1): f(x) = 1.7159 tanh(2x/3) with   */
/* tanh(y) ~ sgn(y) (1 - 1/(1 + |y| + y^2 + 1.41645 y^4)).                   */
/* Kinds 2 and 3 are the same scaled form with the exact tanh, and the plain */
/* tanh(x), kept so that any reading of the benchmark's "+ tanh" can be run. */
/* ------------------------------------------------------------------------ */
double orc_rational_tanh(double y)
{
    double a = fabs(y), y2 = y * y;
    double t = 1.0 - 1.0 / (1.0 + a + y2 + 1.41645 * (y2 * y2));
    return y < 0 ? -t : t;
}

double orc_activation(double x, int act)
{
    switch (act) {
    case ORC_ACT_RATIONAL:    return 1.7159 * orc_rational_tanh(x * (2.0 / 3.0));
    case ORC_ACT_SCALED_TANH: return 1.7159 * tanh(x * (2.0 / 3.0));
    case ORC_ACT_TANH:        return tanh(x);
    default:                  return x;
    }
}

/* ------------------------------------------------------------------------ */
/* Image pyramid.  Paper, Sections 2 and 3.3: the only pre-processing is the */
/* pyramid, parameterised by minSize and scaleFactor (Section 4.1).          */
/* Reading: scale of level 0 is min_face/12 (a min_face-pixel face fills the */
/* 12x12 stage-1 window); each next scale is the previous times the step     */
/* (repeated multiplication); level size is floor(W/s + 1e-9) (the epsilon   */
/* keeps exact quotients such as 3840/2.4 from rounding down); levels stop   */
/* at the first one with a side below the stage-1 window.                    */
/* Returns the number of levels (<= cap), or -1 for bad arguments.           */
/* ------------------------------------------------------------------------ */
int orc_pyramid_layout(int w, int h, double min_face, double step, int window, int cap,
                       int32_t *lvl_w, int32_t *lvl_h, double *lvl_scale)
{
    if (w <= 0 || h <= 0 || !(min_face >= window) || !(step > 1.0)) return -1;
    double s = min_face / (double)window;
    int n = 0;
    while (n < cap) {
        int lw = (int)floor((double)w / s + 1e-9);
        int lh = (int)floor((double)h / s + 1e-9);
        if (lw < window || lh < window) break;
        lvl_w[n] = lw; lvl_h[n] = lh; lvl_scale[n] = s;
        ++n;
        s = s * step;
    }
    return n;
}

/* One axis of the bilinear map.  Reading: pixel-centre alignment,            */
/* f = (i + 0.5) s - 0.5 clamped to [0, n_in-1]; i0 = floor(f);               */
/* weight of the right/lower neighbour quantised to 1/256:                    */
/* q = round((f - i0) * 256) in [0,256].                                      */
static void axis_map(int n_out, int n_in, double s, int32_t *i0, int32_t *i1, int32_t *q)
{
    for (int i = 0; i < n_out; ++i) {
        double f = ((double)i + 0.5) * s - 0.5;
        if (f < 0.0) f = 0.0;
        if (f > (double)(n_in - 1)) f = (double)(n_in - 1);
        int a = (int)floor(f);
        i0[i] = a;
        i1[i] = a + 1 < n_in ? a + 1 : n_in - 1;
        q[i] = (int32_t)floor((f - (double)a) * 256.0 + 0.5);
    }
}

/* Bilinear resampling of one pyramid level straight from the frame (not     */
/* level to level).  Reading: integer blend with 8-bit weights,               */
/* out = (sum of four pixel*weight products + 32768) >> 16, result uint8.     */
void orc_resample_level(const uint8_t *frame, int w, int h, int pitch, double s,
                        int lw, int lh, uint8_t *out)
{
    int32_t *x0 = malloc(sizeof(int32_t) * 3 * (size_t)lw), *x1 = x0 + lw, *qx = x1 + lw;
    int32_t *y0 = malloc(sizeof(int32_t) * 3 * (size_t)lh), *y1 = y0 + lh, *qy = y1 + lh;
    axis_map(lw, w, s, x0, x1, qx);
    axis_map(lh, h, s, y0, y1, qy);
    for (int y = 0; y < lh; ++y) {
        const uint8_t *r0 = frame + (size_t)y0[y] * pitch, *r1 = frame + (size_t)y1[y] * pitch;
        uint32_t wy = (uint32_t)qy[y];
        for (int x = 0; x < lw; ++x) {
            uint32_t wx = (uint32_t)qx[x];
            uint32_t acc = r0[x0[x]] * (256u - wx) * (256u - wy) + r0[x1[x]] * wx * (256u - wy)
                         + r1[x0[x]] * (256u - wx) * wy + r1[x1[x]] * wx * wy;
            out[(size_t)y * lw + x] = (uint8_t)((acc + 32768u) >> 16);
        }
    }
    free(x0); free(y0);
}

/* ------------------------------------------------------------------------ */
/* One network on one window, as a plain stack of layers.                    */
/* Paper, Section 3.1: convolution stride 1 ("valid", no padding), pooling    */
/* stride 2 (2x2 max), the activation after hidden layers.  A fully           */
/* connected layer is the convolution whose kernel covers its whole input,    */
/* features ordered [channel][row][col].                                      */
/* in: in_size x in_size doubles (one channel).  out: the last layer's cout   */
/* values.  Returns 0, or -1 if the layer list does not fit the input.        */
/* ------------------------------------------------------------------------ */
static size_t layer_params(const orc_layer *l)
{
    return l->kind == ORC_POOL ? 0 : (size_t)l->cout * l->cin * l->k * l->k + (size_t)l->cout;
}

int orc_net_forward(const orc_layer *layers, int n_layers, const float *weights, int in_size,
                    const double *in, double *out)
{
    int c = 1, s = in_size;
    size_t cap = (size_t)in_size * in_size;
    for (int i = 0, cc = 1, ss = in_size; i < n_layers; ++i) { /* largest intermediate map */
        const orc_layer *l = &layers[i];
        if (l->kind == ORC_POOL) ss /= 2; else { ss = ss - l->k + 1; cc = l->cout; }
        if (ss < 1) return -1;
        if ((size_t)cc * ss * ss > cap) cap = (size_t)cc * ss * ss;
    }
    double *cur = malloc(sizeof(double) * cap), *nxt = malloc(sizeof(double) * cap);
    memcpy(cur, in, sizeof(double) * (size_t)in_size * in_size);
    const float *wp = weights;
    int rc = 0;
    for (int i = 0; i < n_layers && rc == 0; ++i) {
        const orc_layer *l = &layers[i];
        if (l->cin != c) { rc = -1; break; }
        if (l->kind == ORC_POOL) {
            if (s % 2) { rc = -1; break; }
            int o = s / 2;
            for (int ch = 0; ch < c; ++ch)
                for (int y = 0; y < o; ++y)
                    for (int x = 0; x < o; ++x) {
                        const double *p = cur + ((size_t)ch * s + 2 * y) * s + 2 * x;
                        double m = p[0];
                        if (p[1] > m) m = p[1];
                        if (p[s] > m) m = p[s];
                        if (p[s + 1] > m) m = p[s + 1];
                        nxt[((size_t)ch * o + y) * o + x] = m;
                    }
            s = o;
        } else {
            int k = l->k, o = s - k + 1;
            if (l->kind == ORC_FC && o != 1) { rc = -1; break; }
            const float *bias = wp + (size_t)l->cout * l->cin * k * k;
            for (int oc = 0; oc < l->cout; ++oc)
                for (int y = 0; y < o; ++y)
                    for (int x = 0; x < o; ++x) {
                        double acc = (double)bias[oc];
                        for (int ic = 0; ic < c; ++ic)
                            for (int a = 0; a < k; ++a)
                                for (int b = 0; b < k; ++b)
                                    acc += (double)wp[(((size_t)oc * c + ic) * k + a) * k + b]
                                         * cur[((size_t)ic * s + y + a) * s + x + b];
                        nxt[((size_t)oc * o + y) * o + x] = orc_activation(acc, l->act);
                    }
            wp += layer_params(l);
            c = l->cout; s = o;
        }
        double *t = cur; cur = nxt; nxt = t;
    }
    if (rc == 0) memcpy(out, cur, sizeof(double) * (size_t)c * s * s);
    free(cur); free(nxt);
    return rc;
}

/* Pixel to network input.  Reading: x = (p - 128) / 128.                    */
static double normalise(double p) { return (p - 128.0) * (1.0 / 128.0); }

/* ------------------------------------------------------------------------ */
/* Stage 1 by its definition (paper, Section 3.3: the first CNN scans every  */
/* pyramid image; one response per window position).  Reading: stride 1,      */
/* only windows that lie fully inside the level.                              */
/* scores: (lh - in_size + 1) x (lw - in_size + 1), row-major.                */
/* ------------------------------------------------------------------------ */
int orc_stage1_windows(const uint8_t *level, int lw, int lh, const orc_layer *layers, int n_layers,
                       const float *weights, int in_size, double *scores)
{
    int ow = lw - in_size + 1, oh = lh - in_size + 1, rc = 0;
    if (ow < 1 || oh < 1) return -1;
#pragma omp parallel for schedule(dynamic)
    for (int y = 0; y < oh; ++y) {
        double *win = malloc(sizeof(double) * (size_t)in_size * in_size);
        for (int x = 0; x < ow; ++x) {
            for (int a = 0; a < in_size; ++a)
                for (int b = 0; b < in_size; ++b)
                    win[a * in_size + b] = normalise((double)level[(size_t)(y + a) * lw + x + b]);
            double r;
            if (orc_net_forward(layers, n_layers, weights, in_size, win, &r) != 0) {
#pragma omp atomic write
                rc = -1;
            }
            scores[(size_t)y * ow + x] = r;
        }
        free(win);
    }
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Stage 1 as one fully convolutional pass over the level: the same numbers   */
/* as orc_stage1_windows, reorganised.  Each stride-2 pool becomes a          */
/* stride-1 max over taps `d` apart and doubles the tap spacing `d` of every  */
/* later layer.  Used for the large workloads; checked against the            */
/* definition on small images.                                                */
/* ------------------------------------------------------------------------ */
int orc_stage1_dense(const uint8_t *level, int lw, int lh, const orc_layer *layers, int n_layers,
                     const float *weights, int in_size, double *scores)
{
    int ow = lw - in_size + 1, oh = lh - in_size + 1;
    if (ow < 1 || oh < 1) return -1;
    int c = 1, W = lw, H = lh, d = 1;
    double *cur = malloc(sizeof(double) * (size_t)lw * lh);
    for (size_t i = 0; i < (size_t)lw * lh; ++i) cur[i] = normalise((double)level[i]);
    const float *wp = weights;
    for (int i = 0; i < n_layers; ++i) {
        const orc_layer *l = &layers[i];
        int oc_n = l->kind == ORC_POOL ? c : l->cout;
        int span = l->kind == ORC_POOL ? d : (l->k - 1) * d;
        int OW = W - span, OH = H - span;
        double *nxt = malloc(sizeof(double) * (size_t)oc_n * OW * OH);
        if (l->kind == ORC_POOL) {
#pragma omp parallel for collapse(2)
            for (int ch = 0; ch < c; ++ch)
                for (int y = 0; y < OH; ++y)
                    for (int x = 0; x < OW; ++x) {
                        const double *p = cur + ((size_t)ch * H + y) * W + x;
                        double m = p[0];
                        if (p[d] > m) m = p[d];
                        if (p[(size_t)d * W] > m) m = p[(size_t)d * W];
                        if (p[(size_t)d * W + d] > m) m = p[(size_t)d * W + d];
                        nxt[((size_t)ch * OH + y) * OW + x] = m;
                    }
            d *= 2;
        } else {
            int k = l->k;
            const float *bias = wp + (size_t)l->cout * l->cin * k * k;
#pragma omp parallel for collapse(2)
            for (int oc = 0; oc < l->cout; ++oc)
                for (int y = 0; y < OH; ++y)
                    for (int x = 0; x < OW; ++x) {
                        double acc = (double)bias[oc];
                        for (int ic = 0; ic < c; ++ic)
                            for (int a = 0; a < k; ++a)
                                for (int b = 0; b < k; ++b)
                                    acc += (double)wp[(((size_t)oc * c + ic) * k + a) * k + b]
                                         * cur[((size_t)ic * H + y + (size_t)a * d) * W + x + (size_t)b * d];
                        nxt[((size_t)oc * OH + y) * OW + x] = orc_activation(acc, l->act);
                    }
            wp += layer_params(l);
            c = l->cout;
        }
        free(cur); cur = nxt; W = OW; H = OH;
    }
    int rc = (c == 1 && W == ow && H == oh) ? 0 : -1;
    if (rc == 0) memcpy(scores, cur, sizeof(double) * (size_t)ow * oh);
    free(cur);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Survivors of a stage (paper, Section 3.3: windows whose response exceeded  */
/* the threshold go on).  The comparison is strict and done in fp32, the      */
/* precision the paper's implementations compute in (Section 3.4).            */
/* idx receives the positions i with score[i] > thr in ascending order.       */
/* Returns the count (may exceed cap; only the first cap are written).        */
/* ------------------------------------------------------------------------ */
int64_t orc_survivors(const double *scores, int64_t n, float thr, int64_t cap, int64_t *idx)
{
    int64_t m = 0;
    for (int64_t i = 0; i < n; ++i)
        if ((float)scores[i] > thr) { if (m < cap) idx[m] = i; ++m; }
    return m;
}

/* ------------------------------------------------------------------------ */
/* Crop for stages 2 and 3 (paper, Section 3.3: the region is read from the   */
/* original grayscale image and scaled to the network's input size).          */
/* Reading: the region is the surviving window's own rectangle                */
/* [x s, (x+12) s) x [y s, (y+12) s) in frame pixels, no extra neighbourhood, */
/* resampled bilinearly to n x n in 16.16 fixed point:                        */
/*   S = round(s * 65536); P_i = x S + ((2i+1) * window * S) / (2n) - 32768   */
/*   clamped to [0, (W-1) * 65536]; i0 = P_i >> 16; weight of the right       */
/*   neighbour q = ((P_i & 0xFFFF) + 128) >> 8 in [0,256].                    */
/* The blended value sum / 65536 (sum < 2^24, exact in fp32) is normalised    */
/* like pyramid pixels.  out: n x n doubles.                                  */
/* ------------------------------------------------------------------------ */
static void crop_axis(int64_t origin, int64_t S, int window, int n, int n_in,
                      int32_t *i0, int32_t *i1, int32_t *q)
{
    for (int i = 0; i < n; ++i) {
        int64_t P = origin * S + ((int64_t)(2 * i + 1) * window * S) / (2 * n) - 32768;
        int64_t hi = (int64_t)(n_in - 1) * 65536;
        if (P < 0) P = 0;
        if (P > hi) P = hi;
        int32_t a = (int32_t)(P >> 16);
        i0[i] = a;
        i1[i] = a + 1 < n_in ? a + 1 : n_in - 1;
        q[i] = (int32_t)(((P & 0xFFFF) + 128) >> 8);
    }
}

void orc_crop(const uint8_t *frame, int w, int h, int pitch, int x, int y, double s, int window,
              int n, double *out)
{
    int64_t S = (int64_t)floor(s * 65536.0 + 0.5);
    int32_t *x0 = malloc(sizeof(int32_t) * 6 * (size_t)n);
    int32_t *x1 = x0 + n, *qx = x1 + n, *y0 = qx + n, *y1 = y0 + n, *qy = y1 + n;
    crop_axis(x, S, window, n, w, x0, x1, qx);
    crop_axis(y, S, window, n, h, y0, y1, qy);
    for (int i = 0; i < n; ++i) {
        const uint8_t *r0 = frame + (size_t)y0[i] * pitch, *r1 = frame + (size_t)y1[i] * pitch;
        uint32_t wy = (uint32_t)qy[i];
        for (int j = 0; j < n; ++j) {
            uint32_t wx = (uint32_t)qx[j];
            uint32_t acc = r0[x0[j]] * (256u - wx) * (256u - wy) + r0[x1[j]] * wx * (256u - wy)
                         + r1[x0[j]] * (256u - wx) * wy + r1[x1[j]] * wx * wy;
            out[i * n + j] = normalise((double)acc / 65536.0);
        }
    }
    free(x0);
}

/* Stage 2 / 3: the network on the crop of each listed window.               */
/* xs, ys: window corner in level coordinates; scales: that level's scale.   */
int orc_eval_crops(const uint8_t *frame, int w, int h, int pitch, const int32_t *xs, const int32_t *ys,
                   const double *scales, int64_t count, int window, const orc_layer *layers,
                   int n_layers, const float *weights, int in_size, double *scores)
{
    int rc = 0;
#pragma omp parallel for schedule(dynamic)
    for (int64_t i = 0; i < count; ++i) {
        double *crop = malloc(sizeof(double) * (size_t)in_size * in_size);
        orc_crop(frame, w, h, pitch, xs[i], ys[i], scales[i], window, in_size, crop);
        if (orc_net_forward(layers, n_layers, weights, in_size, crop, &scores[i]) != 0) {
#pragma omp atomic write
            rc = -1;
        }
        free(crop);
    }
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Window (level coordinates) to box in frame pixels.  Reading:               */
/* X = round(x s), Y = round(y s), side = round(window * s).                  */
/* ------------------------------------------------------------------------ */
void orc_window_box(int x, int y, double s, int window, int32_t *bx, int32_t *by, int32_t *bsize)
{
    *bx = (int32_t)floor((double)x * s + 0.5);
    *by = (int32_t)floor((double)y * s + 0.5);
    *bsize = (int32_t)floor((double)window * s + 0.5);
}

/* ------------------------------------------------------------------------ */
/* Merging of accepted windows (paper, Section 3.3: non-maximum suppression   */
/* aggregates the found regions; Section 4.2: minNeighbors).                  */
/* Reading: greedy.  Boxes are ordered by score (fp32) descending, ties by    */
/* ascending `order` key.  The best box not yet suppressed is kept and        */
/* suppresses every later, not yet suppressed box whose intersection over     */
/* union with it exceeds `iou` (strict; areas are integers and the test       */
/* inter > iou * union is evaluated exactly in double with iou an fp32        */
/* value).  `neighbors` of a kept box = how many it suppressed.  Kept boxes   */
/* with neighbors + 1 < min_neighbors are dropped.                            */
/* out_index[j] = input position of the j-th kept box (in kept order),        */
/* out_neighbors[j] its neighbour count.  Returns the number kept.            */
/* ------------------------------------------------------------------------ */
typedef struct { float score; int64_t order; int32_t pos; } merge_key;

static int merge_cmp(const void *a, const void *b)
{
    const merge_key *p = a, *q = b;
    if (p->score > q->score) return -1;
    if (p->score < q->score) return 1;
    return (p->order > q->order) - (p->order < q->order);
}

int32_t orc_merge(const int32_t *bx, const int32_t *by, const int32_t *bsize, const float *score,
                  const int64_t *order, int32_t n, float iou, int32_t min_neighbors,
                  int32_t *out_index, int32_t *out_neighbors)
{
    merge_key *key = malloc(sizeof(merge_key) * (size_t)(n > 0 ? n : 1));
    uint8_t *dead = calloc((size_t)(n > 0 ? n : 1), 1);
    for (int32_t i = 0; i < n; ++i) { key[i].score = score[i]; key[i].order = order[i]; key[i].pos = i; }
    qsort(key, (size_t)n, sizeof(merge_key), merge_cmp);
    int32_t kept = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (dead[i]) continue;
        int32_t p = key[i].pos, nb = 0;
        int64_t ax0 = bx[p], ay0 = by[p], ax1 = ax0 + bsize[p], ay1 = ay0 + bsize[p];
        int64_t aa = (int64_t)bsize[p] * bsize[p];
        for (int32_t j = i + 1; j < n; ++j) {
            if (dead[j]) continue;
            int32_t r = key[j].pos;
            int64_t cx0 = bx[r], cy0 = by[r], cx1 = cx0 + bsize[r], cy1 = cy0 + bsize[r];
            int64_t iw = (ax1 < cx1 ? ax1 : cx1) - (ax0 > cx0 ? ax0 : cx0);
            int64_t ih = (ay1 < cy1 ? ay1 : cy1) - (ay0 > cy0 ? ay0 : cy0);
            if (iw <= 0 || ih <= 0) continue;
            int64_t inter = iw * ih, uni = aa + (int64_t)bsize[r] * bsize[r] - inter;
            if ((double)inter > (double)iou * (double)uni) { dead[j] = 1; ++nb; }
        }
        if (nb + 1 >= min_neighbors) { out_index[kept] = p; out_neighbors[kept] = nb; ++kept; }
    }
    free(key); free(dead);
    return kept;
}

/* ======================================================================== */
/* First stage in the paper's own geometry (paper, Section 3.1: no fully     */
/* connected layer, convolution stride 1, pooling stride 2; Section 3.3: the */
/* output responses correspond to a 27 x 31 scanning window moved with a     */
/* 4 pixel step).  The layer shapes were printed only in the paper's         */
/* Figure 1; the shapes are therefore passed in, with rectangular kernels,   */
/* and any list conv / pool / conv / pool / conv whose last kernel covers    */
/* the remaining map of one window fits.                                      */
/* ======================================================================== */
typedef struct {
    int32_t kind;    /* ORC_CONV or ORC_POOL */
    int32_t cin, cout;
    int32_t kw, kh;  /* kernel width and height (POOL: 2, 2) */
    int32_t act;
} orc_rlayer;

static size_t rlayer_params(const orc_rlayer *l)
{
    return l->kind == ORC_POOL ? 0 : (size_t)l->cout * l->cin * l->kw * l->kh + (size_t)l->cout;
}

/* One window by the definition of the network: in is in_h rows of in_w       */
/* doubles; weights per conv layer [cout][cin][kh][kw] then bias[cout].       */
/* The last layer must leave a 1 x 1 map; out receives its cout values.       */
int orc_rnet_forward(const orc_rlayer *layers, int n_layers, const float *weights, int in_w, int in_h,
                     const double *in, double *out)
{
    int c = 1, w = in_w, h = in_h;
    size_t cap = (size_t)in_w * in_h;
    for (int i = 0, cc = 1, ww = in_w, hh = in_h; i < n_layers; ++i) {
        const orc_rlayer *l = &layers[i];
        if (l->kind == ORC_POOL) { ww /= 2; hh /= 2; } else { ww -= l->kw - 1; hh -= l->kh - 1; cc = l->cout; }
        if (ww < 1 || hh < 1) return -1;
        if ((size_t)cc * ww * hh > cap) cap = (size_t)cc * ww * hh;
    }
    double *cur = malloc(sizeof(double) * cap), *nxt = malloc(sizeof(double) * cap);
    memcpy(cur, in, sizeof(double) * (size_t)in_w * in_h);
    const float *wp = weights;
    int rc = 0;
    for (int i = 0; i < n_layers && rc == 0; ++i) {
        const orc_rlayer *l = &layers[i];
        if (l->cin != c) { rc = -1; break; }
        if (l->kind == ORC_POOL) {
            if (w % 2 || h % 2) { rc = -1; break; }
            int ow = w / 2, oh = h / 2;
            for (int ch = 0; ch < c; ++ch)
                for (int y = 0; y < oh; ++y)
                    for (int x = 0; x < ow; ++x) {
                        const double *p = cur + ((size_t)ch * h + 2 * y) * w + 2 * x;
                        double m = p[0];
                        if (p[1] > m) m = p[1];
                        if (p[w] > m) m = p[w];
                        if (p[w + 1] > m) m = p[w + 1];
                        nxt[((size_t)ch * oh + y) * ow + x] = m;
                    }
            w = ow; h = oh;
        } else {
            int ow = w - l->kw + 1, oh = h - l->kh + 1;
            const float *bias = wp + (size_t)l->cout * c * l->kw * l->kh;
            for (int oc = 0; oc < l->cout; ++oc)
                for (int y = 0; y < oh; ++y)
                    for (int x = 0; x < ow; ++x) {
                        double acc = (double)bias[oc];
                        for (int ic = 0; ic < c; ++ic)
                            for (int a = 0; a < l->kh; ++a)
                                for (int b = 0; b < l->kw; ++b)
                                    acc += (double)wp[(((size_t)oc * c + ic) * l->kh + a) * l->kw + b]
                                         * cur[((size_t)ic * h + y + a) * w + x + b];
                        nxt[((size_t)oc * oh + y) * ow + x] = orc_activation(acc, l->act);
                    }
            wp += rlayer_params(l);
            c = l->cout; w = ow; h = oh;
        }
        double *t = cur; cur = nxt; nxt = t;
    }
    if (rc == 0 && (w != 1 || h != 1)) rc = -1;
    if (rc == 0) memcpy(out, cur, sizeof(double) * (size_t)c);
    free(cur); free(nxt);
    return rc;
}

/* The scan by its definition: the window of win_w x win_h pixels is cut at   */
/* every position (step * i, step * j) that keeps it inside the level and     */
/* run through the network on its own.                                        */
/* scores: ((lh - win_h) / step + 1) rows of ((lw - win_w) / step + 1).       */
int orc_scan_windows(const uint8_t *level, int lw, int lh, const orc_rlayer *layers, int n_layers,
                     const float *weights, int win_w, int win_h, int step, double *scores)
{
    if (lw < win_w || lh < win_h || step < 1) return -1;
    int ow = (lw - win_w) / step + 1, oh = (lh - win_h) / step + 1, rc = 0;
#pragma omp parallel for schedule(dynamic)
    for (int j = 0; j < oh; ++j) {
        double *win = malloc(sizeof(double) * (size_t)win_w * win_h);
        for (int i = 0; i < ow; ++i) {
            for (int a = 0; a < win_h; ++a)
                for (int b = 0; b < win_w; ++b)
                    win[a * win_w + b] = normalise((double)level[(size_t)(step * j + a) * lw + step * i + b]);
            double r = 0.0;
            if (orc_rnet_forward(layers, n_layers, weights, win_w, win_h, win, &r) != 0) {
#pragma omp atomic write
                rc = -1;
            }
            scores[(size_t)j * ow + i] = r;
        }
        free(win);
    }
    return rc;
}

/* The same scan as one pass of the layers over the whole level (paper,       */
/* Section 3.3: the network scans the image, its output layer holds the       */
/* responses of all window positions): convolutions at stride 1, pools at     */
/* stride 2 anchored at the level's corner (a trailing odd row or column is   */
/* dropped).  The step between windows is 2^(number of pools).                */
int orc_scan_fcn(const uint8_t *level, int lw, int lh, const orc_rlayer *layers, int n_layers,
                 const float *weights, int win_w, int win_h, double *scores)
{
    int step = 1;
    for (int i = 0; i < n_layers; ++i) if (layers[i].kind == ORC_POOL) step *= 2;
    if (lw < win_w || lh < win_h) return -1;
    int ow = (lw - win_w) / step + 1, oh = (lh - win_h) / step + 1;
    int c = 1, W = lw, H = lh;
    double *cur = malloc(sizeof(double) * (size_t)lw * lh);
    for (size_t i = 0; i < (size_t)lw * lh; ++i) cur[i] = normalise((double)level[i]);
    const float *wp = weights;
    for (int i = 0; i < n_layers; ++i) {
        const orc_rlayer *l = &layers[i];
        int OW, OH, oc_n;
        if (l->kind == ORC_POOL) { OW = W / 2; OH = H / 2; oc_n = c; }
        else { OW = W - l->kw + 1; OH = H - l->kh + 1; oc_n = l->cout; }
        if (OW < 1 || OH < 1) { free(cur); return -1; }
        double *nxt = malloc(sizeof(double) * (size_t)oc_n * OW * OH);
        if (l->kind == ORC_POOL) {
#pragma omp parallel for collapse(2)
            for (int ch = 0; ch < c; ++ch)
                for (int y = 0; y < OH; ++y)
                    for (int x = 0; x < OW; ++x) {
                        const double *p = cur + ((size_t)ch * H + 2 * y) * W + 2 * x;
                        double m = p[0];
                        if (p[1] > m) m = p[1];
                        if (p[W] > m) m = p[W];
                        if (p[W + 1] > m) m = p[W + 1];
                        nxt[((size_t)ch * OH + y) * OW + x] = m;
                    }
        } else {
            const float *bias = wp + (size_t)l->cout * c * l->kw * l->kh;
#pragma omp parallel for collapse(2)
            for (int oc = 0; oc < l->cout; ++oc)
                for (int y = 0; y < OH; ++y)
                    for (int x = 0; x < OW; ++x) {
                        double acc = (double)bias[oc];
                        for (int ic = 0; ic < c; ++ic)
                            for (int a = 0; a < l->kh; ++a)
                                for (int b = 0; b < l->kw; ++b)
                                    acc += (double)wp[(((size_t)oc * c + ic) * l->kh + a) * l->kw + b]
                                         * cur[((size_t)ic * H + y + a) * W + x + b];
                        nxt[((size_t)oc * OH + y) * OW + x] = orc_activation(acc, l->act);
                    }
            wp += rlayer_params(l);
            c = l->cout;
        }
        free(cur); cur = nxt; W = OW; H = OH;
    }
    int rc = (c == 1 && W >= ow && H >= oh) ? 0 : -1;   /* equal when the window is the net's receptive field */
    if (rc == 0)
        for (int y = 0; y < oh; ++y) memcpy(scores + (size_t)y * ow, cur + (size_t)y * W, sizeof(double) * (size_t)ow);
    free(cur);
    return rc;
}

/* ======================================================================== */
/* The selective unit in the paper's geometry (paper, Section 3.3, second to */
/* fourth paragraph, eq. (2)).                                                */
/* ======================================================================== */

/* Region of rw x rh level pixels whose corner is (x0, y0) in level           */
/* coordinates (may lie outside the level: the frame edge is repeated), read  */
/* from the original frame.  Paper: the analysed region is read from the      */
/* original image together with a neighbourhood and scaled to 51 x 55.        */
/* Reading: sample i sits at frame position (x0 + i + 0.5) s - 0.5 in 16.16   */
/* fixed point with S = round(s * 65536), weights of 8 bits, and the pixel    */
/* is rounded to uint8 (it feeds a histogram).                                */
void orc_region(const uint8_t *frame, int w, int h, int pitch, int x0, int y0, double s, int rw, int rh,
                uint8_t *out)
{
    const int64_t S = (int64_t)floor(s * 65536.0 + 0.5);
    int32_t *xi = malloc(sizeof(int32_t) * 2 * (size_t)(rw + rh));
    int32_t *xq = xi + rw, *yi = xq + rw, *yq = yi + rh;
    for (int k = 0; k < rw + rh; ++k) {
        const int is_y = k >= rw, i = is_y ? k - rw : k, n_in = is_y ? h : w;
        int64_t P = (int64_t)(is_y ? y0 : x0) * S + ((int64_t)(2 * i + 1) * S) / 2 - 32768;
        const int64_t hi = (int64_t)(n_in - 1) << 16;
        if (P < 0) P = 0;
        if (P > hi) P = hi;
        (is_y ? yi : xi)[i] = (int32_t)(P >> 16);
        (is_y ? yq : xq)[i] = (int32_t)(((P & 0xFFFF) + 128) >> 8);
    }
    for (int r = 0; r < rh; ++r)
        for (int c = 0; c < rw; ++c) {
            const int xa = xi[c], xb = xa + 1 < w ? xa + 1 : w - 1, ya = yi[r], yb = ya + 1 < h ? ya + 1 : h - 1;
            const uint32_t qx = (uint32_t)xq[c], qy = (uint32_t)yq[r];
            const uint32_t sum = frame[(size_t)ya * pitch + xa] * (256u - qx) * (256u - qy) + frame[(size_t)ya * pitch + xb] * qx * (256u - qy)
                               + frame[(size_t)yb * pitch + xa] * (256u - qx) * qy + frame[(size_t)yb * pitch + xb] * qx * qy;
            out[(size_t)r * rw + c] = (uint8_t)((sum + 32768u) >> 16);
        }
    free(xi);
}

/* Histogram equalisation of n uint8 values in place (paper, Section 3.3:     */
/* the region's histogram is equalised).  The textbook rule: with cdf(v) =    */
/* number of pixels <= v and c0 = cdf of the smallest value present,          */
/* v -> round((cdf(v) - c0) * 255 / (n - c0)); a constant region (n == c0)    */
/* is left as it is.  Integer arithmetic, ties of the rounding go up.         */
void orc_histeq(uint8_t *img, int n)
{
    int64_t hist[256] = {0}, cdf = 0, c0 = -1;
    uint8_t lut[256];
    for (int i = 0; i < n; ++i) ++hist[img[i]];
    for (int v = 0; v < 256; ++v) {
        cdf += hist[v];
        if (c0 < 0 && hist[v] > 0) c0 = cdf;
        lut[v] = (uint8_t)v;
        if (c0 >= 0 && n > c0) lut[v] = (uint8_t)((2 * (cdf - c0) * 255 + (n - c0)) / (2 * (n - c0)));
    }
    for (int i = 0; i < n; ++i) img[i] = lut[img[i]];
}

/* One region through the unit.  The equalised region and its mirror image    */
/* (reflection about the vertical axis) go through CNN_2; response (v, u) of  */
/* the region and response (v, nw - 1 - u) of the mirror belong to the same   */
/* window.  Reading (the paper does not say how the two are combined): their  */
/* mean.  K2 = number of combined responses > t2 (fp32, strict).  If K2 = 0   */
/* the analysis stops (paper: "further analysis of the region stops"), else   */
/* CNN_3 gives K3 the same way with t3, and eq. (2) decides:                  */
/*   face = (K2 >= t_nn and K3 > 0) or (K2 > 0 and K3 >= t_nn).               */
/* rule = 3 selects the weaker rule of Section 4.3, eq. (3):                  */
/*   face = K2 >= t_nn or K3 >= t_nn.                                         */
/* There CNN_3's count alone can accept a region, so no outcome of CNN_2      */
/* "disagrees with the rule" (the stop of Section 3.3 is stated for rule      */
/* (2), under which K2 = 0 already decides): CNN_3 runs on every region.      */
/* r2, r3: the combined response maps (nh x nw doubles each; r3 is zero when  */
/* CNN_3 was not run).  Returns 0, -1 if a network does not fit the region.   */
int orc_select_region(const uint8_t *region, int rw, int rh,
                      const orc_rlayer *l2, int n2, const float *w2, const orc_rlayer *l3, int n3, const float *w3,
                      int win_w, int win_h, float t2, float t3, int t_nn, int rule,
                      int32_t *k2, int32_t *k3, int32_t *face, double *r2, double *r3)
{
    int step = 1;
    for (int i = 0; i < n2; ++i) if (l2[i].kind == ORC_POOL) step *= 2;
    const int nw = (rw - win_w) / step + 1, nh = (rh - win_h) / step + 1;
    uint8_t *mir = malloc((size_t)rw * rh);
    double *a = malloc(sizeof(double) * 2 * (size_t)nw * nh), *b = a + (size_t)nw * nh;
    for (int y = 0; y < rh; ++y)
        for (int x = 0; x < rw; ++x) mir[(size_t)y * rw + x] = region[(size_t)y * rw + (rw - 1 - x)];
    int rc = 0;
    *k2 = *k3 = *face = 0;
    for (int i = 0; i < nw * nh; ++i) r2[i] = r3[i] = 0.0;
    if (orc_scan_fcn(region, rw, rh, l2, n2, w2, win_w, win_h, a) || orc_scan_fcn(mir, rw, rh, l2, n2, w2, win_w, win_h, b)) rc = -1;
    if (rc == 0) {
        for (int v = 0; v < nh; ++v)
            for (int u = 0; u < nw; ++u) {
                r2[v * nw + u] = 0.5 * (a[v * nw + u] + b[v * nw + (nw - 1 - u)]);
                if ((float)r2[v * nw + u] > t2) ++*k2;
            }
        if (*k2 > 0 || rule == 3) {
            if (orc_scan_fcn(region, rw, rh, l3, n3, w3, win_w, win_h, a) || orc_scan_fcn(mir, rw, rh, l3, n3, w3, win_w, win_h, b)) rc = -1;
            if (rc == 0)
                for (int v = 0; v < nh; ++v)
                    for (int u = 0; u < nw; ++u) {
                        r3[v * nw + u] = 0.5 * (a[v * nw + u] + b[v * nw + (nw - 1 - u)]);
                        if ((float)r3[v * nw + u] > t3) ++*k3;
                    }
        }
        if (rule == 3) *face = *k2 >= t_nn || *k3 >= t_nn;
        else *face = (*k2 >= t_nn && *k3 > 0) || (*k2 > 0 && *k3 >= t_nn);
    }
    free(mir); free(a);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Merging of the regions the selective unit accepted (paper, Section 3.3:    */
/* non-maximum suppression aggregates the found regions; Section 4.2:         */
/* minNeighbors).  The greedy rule of orc_merge for rectangles bw x bh: order */
/* by score (fp32) descending, ties by ascending `order`; the best rectangle  */
/* not yet suppressed is kept and suppresses every later one with             */
/* inter > iou * union (integer areas, exact in double, strict).              */
/* Reading (the paper gives neither): an accepted region enters as its 27x31  */
/* window in frame pixels (orc_region_box) with the largest combined CNN_3    */
/* response of its map as score.                                              */
/* ------------------------------------------------------------------------ */
void orc_region_box(int i, int j, double s, int step, int win_w, int win_h,
                    int32_t *bx, int32_t *by, int32_t *bw, int32_t *bh)
{
    *bx = (int32_t)floor((double)(step * i) * s + 0.5);
    *by = (int32_t)floor((double)(step * j) * s + 0.5);
    *bw = (int32_t)floor((double)win_w * s + 0.5);
    *bh = (int32_t)floor((double)win_h * s + 0.5);
}

int32_t orc_merge_rect(const int32_t *bx, const int32_t *by, const int32_t *bw, const int32_t *bh, const float *score,
                       const int64_t *order, int32_t n, float iou, int32_t min_neighbors,
                       int32_t *out_index, int32_t *out_neighbors)
{
    merge_key *key = malloc(sizeof(merge_key) * (size_t)(n > 0 ? n : 1));
    uint8_t *dead = calloc((size_t)(n > 0 ? n : 1), 1);
    for (int32_t i = 0; i < n; ++i) { key[i].score = score[i]; key[i].order = order[i]; key[i].pos = i; }
    qsort(key, (size_t)n, sizeof(merge_key), merge_cmp);
    int32_t kept = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (dead[i]) continue;
        const int32_t p = key[i].pos;
        int32_t nb = 0;
        for (int32_t j = i + 1; j < n; ++j) {
            if (dead[j]) continue;
            const int32_t r = key[j].pos;
            const int64_t right = (int64_t)bx[p] + bw[p] < (int64_t)bx[r] + bw[r] ? (int64_t)bx[p] + bw[p] : (int64_t)bx[r] + bw[r];
            const int64_t left = bx[p] > bx[r] ? bx[p] : bx[r];
            const int64_t bottom = (int64_t)by[p] + bh[p] < (int64_t)by[r] + bh[r] ? (int64_t)by[p] + bh[p] : (int64_t)by[r] + bh[r];
            const int64_t top = by[p] > by[r] ? by[p] : by[r];
            if (right <= left || bottom <= top) continue;
            const int64_t inter = (right - left) * (bottom - top);
            const int64_t uni = (int64_t)bw[p] * bh[p] + (int64_t)bw[r] * bh[r] - inter;
            if ((double)inter > (double)iou * (double)uni) { dead[j] = 1; ++nb; }
        }
        if (nb + 1 >= min_neighbors) { out_index[kept] = p; out_neighbors[kept] = nb; ++kept; }
    }
    free(key); free(dead);
    return kept;
}
