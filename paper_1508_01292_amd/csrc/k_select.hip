// The selective unit in the paper's geometry (paper, Section 3.3): host side, and the kernel around the workgroup
// routine of select_body.h.  Two builds of that routine: select_kernel reads the first layers' weights of CNN_2 and CNN_3
// from memory; the code object of k_select_lit.hip carries them as instruction literals, filled in by
// cnnc_select_set_weights (literal_weights.h), and is used whenever its module loads.
#include <vector>

#include <string.h>

#include "literal_weights.h"
#include "select_body.h"

#include "select_lit_image.inc"      // written by the build: kSelectLitImage, kSelectLitPatch

namespace cnnc {

using namespace selbody;

template <int ACT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))
void select_kernel(const uint8_t *__restrict__ frame, int fw, int fh, int pitch, const LevelDev *__restrict__ levels,
                   const ScanLevel *__restrict__ slev, int n_levels, const uint32_t *__restrict__ idx,
                   const float *__restrict__ resp, const int32_t *__restrict__ d_n, int n_max,
                   const float *__restrict__ w2, const float *__restrict__ w3, const float *__restrict__ f2,
                   const float *__restrict__ f3, float t2, float t3, int t_nn, int rule,
                   cnnc_region *__restrict__ rec, float *__restrict__ maps2, float *__restrict__ maps3)
{
    select_regions<ACT>(frame, fw, fh, pitch, levels, slev, n_levels, idx, resp, d_n, n_max, w2, w3, w2, w3, f2, f3, t2, t3, t_nn,
                        rule, rec, maps2, maps3);
}

struct SelectLiteral {
    LiteralModule *mod = nullptr;
    hipFunction_t fn[3] = {nullptr, nullptr, nullptr};       // [activation - 1]
};

namespace {
void select_literal_destroy(SelectLiteral *s)
{
    if (!s) return;
    literal_release(s->mod);
    delete s;
}

// w2, w3: the networks' blobs; their first layers (weights, then biases) are what becomes literal
SelectLiteral *select_literal_create(const float *w2, const float *w3)
{
    static const LiteralImage img = {kSelectLitImage, sizeof(kSelectLitImage), kSelectLitPatch,
                                     sizeof(kSelectLitPatch) / sizeof(kSelectLitPatch[0]), kFirstLayers};
    float first[kFirstLayers];
    memcpy(first, w2, sizeof(float) * kFirst2);
    memcpy(first + kFirst2, w3, sizeof(float) * kFirst3);
    LiteralModule *m = literal_acquire(img, first);
    if (!m) return nullptr;
    SelectLiteral *s = new SelectLiteral();
    s->mod = m;
    static const char *const names[3] = {"cnnc_select_lit_act1", "cnnc_select_lit_act2", "cnnc_select_lit_act3"};
    for (int a = 0; a < 3; ++a)
        if (!(s->fn[a] = literal_function(m, names[a]))) {
            select_literal_destroy(s);
            return nullptr;
        }
    return s;
}
}  // namespace

namespace {
constexpr int kPaperFastDets = 2048;      // detections of the whole-path call that come back with the counters

// B operand of a network's second convolution in lane order: [n tile][k step][lane], lane (g = lane / 16, j = lane % 16)
// holds the weight of tap k = 4 step + g (k = 9 c + 3 a + b) for map n = 16 tile + j; zero beyond K and C2.  Behind it
// the weights of the output convolution as [c2][8 kernel rows][8] (a row's seven, then a zero), for 16-byte loads.
size_t fragment_floats(int c1, int c2) { return (size_t)2 * conv2_steps(c1) * 64 + (size_t)c2 * kK3H * kOutRowPad; }

void conv2_fragments(const float *blob, int c1, int c2, std::vector<float> &f)
{
    const int K = c1 * 9, KS = conv2_steps(c1), W2 = c1 * 17, W3 = W2 + c2 * K + c2;
    f.assign(fragment_floats(c1, c2), 0.0f);
    for (int k = 0; k < c2; ++k)
        for (int a = 0; a < kK3H; ++a)
            for (int b = 0; b < kK3W; ++b)
                f[(size_t)2 * KS * 64 + ((size_t)k * kK3H + a) * kOutRowPad + b] = blob[W3 + (k * kK3H + a) * kK3W + b];
    for (int nt = 0; nt < 2; ++nt)
        for (int st = 0; st < KS; ++st)
            for (int lane = 0; lane < 64; ++lane) {
                const int k = 4 * st + (lane >> 4), n = 16 * nt + (lane & 15);
                if (k < K && n < c2) f[((size_t)nt * KS + st) * 64 + lane] = blob[W2 + n * K + k];
            }
}
}  // namespace

void select_release(cnnc_ctx *c)
{
    select_literal_destroy(c->sel_literal);
    c->sel_literal = nullptr;
    (void)hipFree(c->d_sel_f2); (void)hipFree(c->d_sel_f3);
    c->d_sel_f2 = c->d_sel_f3 = nullptr;
    (void)hipFree(c->d_sel_w2); (void)hipFree(c->d_sel_w3); (void)hipFree(c->d_sel_idx); (void)hipFree(c->d_sel_sc);
    (void)hipFree(c->d_sel_rec); (void)hipFree(c->d_sel_maps); (void)hipFree(c->d_sel_cnt);
    (void)hipFree(c->d_sel_fsc); (void)hipFree(c->d_sel_pick); (void)hipFree(c->d_sel_det);
    c->d_sel_fsc = nullptr; c->d_sel_pick = nullptr; c->d_sel_det = nullptr;
    if (c->h_sel_cnt) (void)hipHostFree(c->h_sel_cnt);
    if (c->h_sel_det) (void)hipHostFree(c->h_sel_det);
    c->h_sel_det = nullptr;
    c->d_sel_w2 = c->d_sel_w3 = nullptr; c->d_sel_idx = nullptr; c->d_sel_sc = nullptr; c->d_sel_rec = nullptr;
    c->d_sel_maps = nullptr; c->d_sel_cnt = nullptr; c->h_sel_cnt = nullptr;
}

}  // namespace cnnc

using namespace cnnc;

#define HIP_TRY(c, expr)                                         \
    do {                                                         \
        hipError_t e_ = (expr);                                  \
        if (e_ != hipSuccess) return hip_fail((c), e_, #expr);   \
    } while (0)

extern "C" {

int cnnc_select_set_weights(cnnc_ctx *c, const float *w2, int n2, const float *w3, int n3, int act)
{
    if (!c) return CNNC_E_INVAL;
    if (!w2 || !w3 || n2 != kNet2Params || n3 != kNet3Params)
        return fail(c, CNNC_E_INVAL, "the selective unit's networks have 1836 and 2942 parameters");
    if (act < CNNC_ACT_RATIONAL || act > CNNC_ACT_TANH) return fail(c, CNNC_E_INVAL, "activation kind must be 1, 2 or 3");
    HIP_TRY(c, wait_last_stream(c));
    if (!c->d_sel_w2) {
        const size_t cap = (size_t)c->max_surv;
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_w2, sizeof(float) * kNet2Params));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_w3, sizeof(float) * kNet3Params));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_f2, sizeof(float) * fragment_floats(kNet2C1, kNet2C2)));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_f3, sizeof(float) * fragment_floats(kNet3C1, kNet3C2)));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_idx, sizeof(uint32_t) * cap));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_sc, sizeof(float) * cap));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_rec, sizeof(cnnc_region) * cap));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_maps, sizeof(float) * 2 * kMap * cap));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_cnt, sizeof(int32_t) * 4));
        HIP_TRY(c, hipHostMalloc((void **)&c->h_sel_cnt, sizeof(int32_t) * 4, hipHostMallocDefault));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_fsc, sizeof(float) * (size_t)c->merge_cap));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_pick, sizeof(uint32_t) * (size_t)c->merge_cap));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_det, sizeof(cnnc_rdet) * (size_t)c->merge_cap));
        HIP_TRY(c, hipHostMalloc((void **)&c->h_sel_det, sizeof(cnnc_rdet) * (size_t)kPaperFastDets, hipHostMallocDefault));
    }
    HIP_TRY(c, hipMemcpy(c->d_sel_w2, w2, sizeof(float) * kNet2Params, hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemcpy(c->d_sel_w3, w3, sizeof(float) * kNet3Params, hipMemcpyHostToDevice));
    std::vector<float> f;
    conv2_fragments(w2, kNet2C1, kNet2C2, f);
    HIP_TRY(c, hipMemcpy(c->d_sel_f2, f.data(), sizeof(float) * f.size(), hipMemcpyHostToDevice));
    conv2_fragments(w3, kNet3C1, kNet3C2, f);
    HIP_TRY(c, hipMemcpy(c->d_sel_f3, f.data(), sizeof(float) * f.size(), hipMemcpyHostToDevice));
    select_literal_destroy(c->sel_literal);
    c->sel_literal = select_literal_create(w2, w3);              // optional: without it the first layers read their weights from memory
    c->sel_act = act;
    c->sel_done = false;
    return CNNC_OK;
}

int cnnc_select_set_rule(cnnc_ctx *c, int rule)
{
    if (!c) return CNNC_E_INVAL;
    if (rule != 2 && rule != 3) return fail(c, CNNC_E_INVAL, "decision rule must be 2 or 3");
    c->sel_rule = rule;
    return CNNC_OK;
}

int cnnc_select_run(cnnc_ctx *c, float t1, float t2, float t3, int t_nn, void *stream)
{
    if (!c) return CNNC_E_INVAL;
    if (t1 != t1 || t2 != t2 || t3 != t3) return fail(c, CNNC_E_INVAL, "a threshold is NaN");
    if (!c->d_sel_w2) return fail(c, CNNC_E_STATE, "cnnc_select_set_weights has not been called");
    if (!c->scan_done) return fail(c, CNNC_E_STATE, "the selective unit needs cnnc_scan_scoremap of this frame");
    if ((c->n_scan + kCompactPerBlock - 1) / kCompactPerBlock + 1 > c->cap_blocks)
        return fail(c, CNNC_E_INVAL, "response map larger than the compaction workspace");
    hipStream_t st = (hipStream_t)stream;
    c->last_stream = st;
    ScopedTimer tm(c, CNNC_T_SELECT, st);
    {
        CompactJob job{};
        job.slot = 0; job.vals = c->d_scan_map; job.n_literal = c->n_scan; job.thr = t1;
        job.out_idx = c->d_sel_idx; job.out_sc = c->d_sel_sc; job.d_count = c->d_sel_cnt;
        HIP_TRY(c, launch_compact(c, job, st));
    }
    dim3 grid(256 * 4), block(kThreads);
    float *m2 = c->d_sel_maps, *m3 = c->d_sel_maps + (size_t)kMap * c->max_surv;
    if (c->sel_literal && c->use_literals) {
        const uint8_t *frame = c->d_frame;
        int fw = c->fw, fh = c->fh, fpitch = c->fpitch, n_levels = c->n_levels, n_max = c->max_surv, rule = c->sel_rule;
        const LevelDev *levels = c->d_levels;
        const ScanLevel *slev = c->d_scan_levels;
        const uint32_t *idx = c->d_sel_idx;
        const float *resp = c->d_sel_sc, *w2 = c->d_sel_w2, *w3 = c->d_sel_w3, *f2 = c->d_sel_f2, *f3 = c->d_sel_f3;
        const int32_t *d_n = c->d_sel_cnt;
        cnnc_region *rec = c->d_sel_rec;
        void *args[] = {&frame, &fw, &fh, &fpitch, &levels, &slev, &n_levels, &idx, &resp, &d_n, &n_max, &w2, &w3, &f2, &f3,
                        &t2, &t3, &t_nn, &rule, &rec, &m2, &m3};
        HIP_TRY(c, hipModuleLaunchKernel(c->sel_literal->fn[c->sel_act - 1], grid.x, 1, 1, kThreads, 1, 1, 0, st, args, nullptr));
        c->sel_done = true;
        return CNNC_OK;
    }
#define CNNC_SEL(ACT)                                                                                             \
    hipLaunchKernelGGL(select_kernel<ACT>, grid, block, 0, st, c->d_frame, c->fw, c->fh, c->fpitch, c->d_levels,  \
                       c->d_scan_levels, c->n_levels, c->d_sel_idx, c->d_sel_sc, c->d_sel_cnt, c->max_surv,       \
                       c->d_sel_w2, c->d_sel_w3, c->d_sel_f2, c->d_sel_f3, t2, t3, t_nn, c->sel_rule, c->d_sel_rec, m2, m3)
    switch (c->sel_act) {
    case CNNC_ACT_RATIONAL: CNNC_SEL(CNNC_ACT_RATIONAL); break;
    case CNNC_ACT_SCALED_TANH: CNNC_SEL(CNNC_ACT_SCALED_TANH); break;
    default: CNNC_SEL(CNNC_ACT_TANH); break;
    }
#undef CNNC_SEL
    HIP_TRY(c, hipGetLastError());
    c->sel_done = true;
    return CNNC_OK;
}

int cnnc_select_fetch(cnnc_ctx *c, cnnc_region *out, int cap, int *n_out, float *maps2, float *maps3)
{
    if (!c) return CNNC_E_INVAL;
    if (!n_out || cap < 0 || (!out && cap > 0)) return fail(c, CNNC_E_INVAL, "null output");
    if (!c->sel_done) return fail(c, CNNC_E_STATE, "cnnc_select_run has not been called for this frame");
    HIP_TRY(c, hipMemcpyAsync(c->h_sel_cnt, c->d_sel_cnt, sizeof(int32_t), hipMemcpyDeviceToHost, c->last_stream));
    HIP_TRY(c, wait_last_stream(c));
    const int total = *c->h_sel_cnt;
    *n_out = total;
    const int have = std::min(total, c->max_surv), m = std::min(have, cap);
    if (m > 0) {
        HIP_TRY(c, hipMemcpy(out, c->d_sel_rec, sizeof(cnnc_region) * (size_t)m, hipMemcpyDeviceToHost));
        if (maps2) HIP_TRY(c, hipMemcpy(maps2, c->d_sel_maps, sizeof(float) * kMap * (size_t)m, hipMemcpyDeviceToHost));
        if (maps3)
            HIP_TRY(c, hipMemcpy(maps3, c->d_sel_maps + (size_t)kMap * c->max_surv, sizeof(float) * kMap * (size_t)m, hipMemcpyDeviceToHost));
    }
    if (total > c->max_surv) return fail(c, CNNC_E_OVERFLOW, "more positions passed T_1 than the context's survivor capacity");
    if (total > cap) return fail(c, CNNC_E_OVERFLOW, "output array too small");
    return CNNC_OK;
}

int cnnc_select_merge(cnnc_ctx *c, float iou, int min_neighbors, cnnc_rdet *out, int cap, int *n_out, void *stream)
{
    if (!c) return CNNC_E_INVAL;
    if (!n_out || cap < 0 || (!out && cap > 0)) return fail(c, CNNC_E_INVAL, "null output");
    if (!(iou >= 0.0f && iou <= 1.0f) || min_neighbors < 1) return fail(c, CNNC_E_INVAL, "iou outside [0, 1] or min_neighbors < 1");
    if (!c->sel_done) return fail(c, CNNC_E_STATE, "cnnc_select_run has not been called for this frame");
    hipStream_t st = (hipStream_t)stream;
    c->last_stream = st;
    HIP_TRY(c, launch_merge_regions(c, iou, min_neighbors, st));
    HIP_TRY(c, hipMemcpyAsync(c->h_sel_cnt, c->d_sel_cnt, sizeof(int32_t) * 3, hipMemcpyDeviceToHost, st));
    HIP_TRY(c, wait_last_stream(c));
    *n_out = 0;
    if (c->h_sel_cnt[0] > c->max_surv) return fail(c, CNNC_E_OVERFLOW, "more positions passed T_1 than the context's survivor capacity");
    if (c->h_sel_cnt[1] > c->merge_cap) return fail(c, CNNC_E_OVERFLOW, "more regions accepted than the merge can take");
    const int total = c->h_sel_cnt[2], m = std::min(total, cap);
    *n_out = total;
    if (m > 0) HIP_TRY(c, hipMemcpy(out, c->d_sel_det, sizeof(cnnc_rdet) * (size_t)m, hipMemcpyDeviceToHost));
    if (total > cap) return fail(c, CNNC_E_OVERFLOW, "output array too small");
    return CNNC_OK;
}

// ---- the whole path in the paper's geometry: pyramid, scan, selective unit, merge (Section 3.3) ----------------
static int paper_fetch(cnnc_ctx *c, cnnc_rdet *out, int cap, int *n_out)
{
    HIP_TRY(c, wait_last_stream(c));
    *n_out = 0;
    if (c->h_sel_cnt[0] > c->max_surv) return fail(c, CNNC_E_OVERFLOW, "more positions passed T_1 than the context's survivor capacity");
    if (c->h_sel_cnt[1] > c->merge_cap) return fail(c, CNNC_E_OVERFLOW, "more regions accepted than the merge can take");
    const int total = c->h_sel_cnt[2], m = std::min(total, cap);
    *n_out = total;
    if (m > 0) memcpy(out, c->h_sel_det, sizeof(cnnc_rdet) * (size_t)std::min(m, kPaperFastDets));
    if (m > kPaperFastDets)      // the enqueued copy only brought the first kPaperFastDets
        HIP_TRY(c, hipMemcpy(out + kPaperFastDets, c->d_sel_det + kPaperFastDets, sizeof(cnnc_rdet) * (size_t)(m - kPaperFastDets),
                             hipMemcpyDeviceToHost));
    if (total > cap) return fail(c, CNNC_E_OVERFLOW, "output array too small");
    return CNNC_OK;
}

int cnnc_detect_paper_async(cnnc_ctx *c, const uint8_t *d_frame, int w, int h, int pitch, const cnnc_paper_params *p, void *stream)
{
    if (!c) return CNNC_E_INVAL;
    if (!p) return fail(c, CNNC_E_INVAL, "null parameters");
    if (!(p->merge_iou >= 0.0f && p->merge_iou <= 1.0f) || p->min_neighbors < 1 || p->t_nn < 1)
        return fail(c, CNNC_E_INVAL, "iou outside [0, 1], min_neighbors < 1 or t_nn < 1");
    if (!c->d_scan_wt || !c->d_sel_w2) return fail(c, CNNC_E_STATE, "cnnc_scan_set_weights / cnnc_select_set_weights have not been called");
    int rc;
    c->paper_pending = false;
    if ((rc = cnnc_build_pyramid(c, d_frame, w, h, pitch, stream))) return rc;
    if ((rc = cnnc_scan_scoremap(c, stream))) return rc;
    if ((rc = cnnc_select_run(c, p->t1, p->t2, p->t3, p->t_nn, stream))) return rc;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(c, launch_merge_regions(c, p->merge_iou, p->min_neighbors, st));
    HIP_TRY(c, hipMemcpyAsync(c->h_sel_cnt, c->d_sel_cnt, sizeof(int32_t) * 3, hipMemcpyDeviceToHost, st));
    HIP_TRY(c, hipMemcpyAsync(c->h_sel_det, c->d_sel_det, sizeof(cnnc_rdet) * (size_t)std::min(c->merge_cap, kPaperFastDets),
                              hipMemcpyDeviceToHost, st));
    c->paper_pending = true;
    return CNNC_OK;
}

int cnnc_fetch_paper(cnnc_ctx *c, cnnc_rdet *out, int cap, int *n_out)
{
    if (!c) return CNNC_E_INVAL;
    if (!n_out || cap < 0 || (!out && cap > 0)) return fail(c, CNNC_E_INVAL, "null output");
    if (!c->paper_pending) return fail(c, CNNC_E_STATE, "no cnnc_detect_paper_async pass was enqueued");
    return paper_fetch(c, out, cap, n_out);
}

int cnnc_detect_paper(cnnc_ctx *c, const uint8_t *d_frame, int w, int h, int pitch, const cnnc_paper_params *p, cnnc_rdet *out,
                      int cap, int *n_out)
{
    if (!c) return CNNC_E_INVAL;
    if (!n_out || cap < 0 || (!out && cap > 0)) return fail(c, CNNC_E_INVAL, "null output");
    const int rc = cnnc_detect_paper_async(c, d_frame, w, h, pitch, p, nullptr);
    if (rc) return rc;
    return paper_fetch(c, out, cap, n_out);
}

}  // extern "C"
