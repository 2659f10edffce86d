// Host side of libcnnc: context, geometry tables, buffer management and the C entry points.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "cnnc_internal.h"

using namespace cnnc;

namespace cnnc {
int fail(cnnc_ctx *c, int code, const std::string &msg)
{
    if (c) c->err = msg;
    return code;
}

int hip_fail(cnnc_ctx *c, hipError_t e, const char *what)
{
    return fail(c, e == hipErrorOutOfMemory ? CNNC_E_NOMEM : CNNC_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}
}  // namespace cnnc

namespace {

constexpr int kFastDets = 2048;   // detections copied to the host together with the counters

#define HIP_TRY(c, expr)                                         \
    do {                                                         \
        hipError_t e_ = (expr);                                  \
        if (e_ != hipSuccess) return hip_fail((c), e_, #expr);   \
    } while (0)

struct LayerSpec { int kind, cin, cout, k; bool hidden; };

const LayerSpec kStage1[] = {{CNNC_CONV, 1, 4, 3, true}, {CNNC_POOL, 4, 4, 2, false}, {CNNC_CONV, 4, 8, 3, true},
                             {CNNC_FC, 8, 1, 3, false}};
const LayerSpec kStage2[] = {{CNNC_CONV, 1, 8, 5, true}, {CNNC_POOL, 8, 8, 2, false}, {CNNC_CONV, 8, 16, 3, true},
                             {CNNC_POOL, 16, 16, 2, false}, {CNNC_FC, 16, 32, 4, true}, {CNNC_FC, 32, 1, 1, false}};
const LayerSpec kStage3[] = {{CNNC_CONV, 1, 16, 5, true}, {CNNC_POOL, 16, 16, 2, false}, {CNNC_CONV, 16, 32, 5, true},
                             {CNNC_POOL, 32, 32, 2, false}, {CNNC_CONV, 32, 32, 3, true}, {CNNC_FC, 32, 64, 7, true},
                             {CNNC_FC, 64, 1, 1, false}};

// The descriptor must name one of the built-in shapes; returns the hidden activation or -1.
int check_stage(const cnnc_stage_desc &d, const LayerSpec *spec, int n_spec, int in_size)
{
    if (d.in_size != in_size || d.n_layers != n_spec || !d.layers || !d.weights) return -1;
    int act = 0;
    for (int i = 0; i < n_spec; ++i) {
        const cnnc_layer &l = d.layers[i];
        if (l.kind != spec[i].kind || l.cin != spec[i].cin || l.cout != spec[i].cout || l.k != spec[i].k) return -1;
        if (spec[i].hidden) {
            if (l.act < CNNC_ACT_RATIONAL || l.act > CNNC_ACT_TANH) return -1;
            if (act && l.act != act) return -1;
            act = l.act;
        } else if (l.act != CNNC_ACT_NONE) {
            return -1;
        }
    }
    return act;
}

template <typename T>
int ensure(cnnc_ctx *c, T *&ptr, int64_t &cap, int64_t need)
{
    if (need <= cap) return CNNC_OK;
    if (ptr) { HIP_TRY(c, hipFree(ptr)); ptr = nullptr; cap = 0; }
    HIP_TRY(c, hipMalloc((void **)&ptr, sizeof(T) * (size_t)need));
    cap = need;
    return CNNC_OK;
}

// One axis of the pyramid's bilinear map; entry = (left index << 9) | weight of the right neighbour.
void axis_taps(int n_out, int n_in, double s, uint32_t *out)
{
    for (int i = 0; i < n_out; ++i) {
        double f = ((double)i + 0.5) * s - 0.5;
        if (f < 0.0) f = 0.0;
        if (f > (double)(n_in - 1)) f = (double)(n_in - 1);
        const int a = (int)floor(f);
        const int q = (int)floor((f - (double)a) * 256.0 + 0.5);
        out[i] = ((uint32_t)a << 9) | (uint32_t)q;
    }
}

}  // namespace

namespace cnnc {
// Pyramid geometry for a frame size under the current parameters (host arithmetic only).
int compute_levels(const cnnc_ctx *c, int w, int h, std::vector<LevelDev> &lv, int64_t &pyr_bytes, int64_t &n_windows)
{
    lv.clear();
    double s = c->params.min_face / (double)kWin;
    int64_t poff = 0, soff = 0, toff = 0, woff = 0;
    while ((int)lv.size() < CNNC_MAX_LEVELS) {
        const int lw = (int)floor((double)w / s + 1e-9), lh = (int)floor((double)h / s + 1e-9);
        if (lw < kWin || lh < kWin) break;
        LevelDev L{};
        L.w = lw; L.h = lh; L.ow = lw - kWin + 1; L.oh = lh - kWin + 1;
        L.pyr_off = (int32_t)poff; L.score_off = (int32_t)soff;
        L.xmap_off = (int32_t)toff; L.ymap_off = (int32_t)(toff + lw);
        L.scale_q16 = (int64_t)floor(s * 65536.0 + 0.5);
        L.scale = s;
        L.word_off = (int32_t)woff; L.words_per_row = (L.ow + 31) / 32;
        woff += (int64_t)L.words_per_row * L.oh;
        lv.push_back(L);
        poff += (int64_t)lw * lh; soff += (int64_t)L.ow * L.oh; toff += lw + lh;
        if (poff > INT32_MAX || soff > INT32_MAX) return CNNC_E_INVAL;
        s = s * c->params.scale_step;
    }
    pyr_bytes = poff; n_windows = soff;
    return lv.empty() ? CNNC_E_INVAL : CNNC_OK;
}

}  // namespace cnnc

namespace {

int prepare_layout(cnnc_ctx *c, int w, int h)
{
    if (c->layout_valid && c->lay_w == w && c->lay_h == h) return CNNC_OK;
    if (w < kWin || h < kWin || w > c->max_w || h > c->max_h) return fail(c, CNNC_E_INVAL, "frame size outside [12, max]");
    std::vector<LevelDev> lv;
    int64_t pyr_bytes = 0, n_windows = 0;
    if (compute_levels(c, w, h, lv, pyr_bytes, n_windows) != CNNC_OK)
        return fail(c, CNNC_E_INVAL, "frame has no pyramid level at these parameters");

    const int pyr_ntx = (w + kPyrTileW - 1) / kPyrTileW, pyr_nty = (h + kPyrTileH - 1) / kPyrTileH;
    std::vector<uint32_t> taps, tiles_pyr, tiles_s1;
    std::vector<int> s1_tile_of_level(lv.size() + 1, 0);
    for (size_t l = 0; l < lv.size(); ++l) {
        const LevelDev &L = lv[l];
        s1_tile_of_level[l] = (int)tiles_s1.size();
        const size_t base = taps.size();
        taps.resize(base + L.w + L.h);
        axis_taps(L.w, w, L.scale, taps.data() + base);
        axis_taps(L.h, h, L.scale, taps.data() + base + L.w);
        // which level columns / rows each frame tile produces: those whose left / upper source pixel lies in it
        for (int axis = 0; axis < 2; ++axis) {
            const uint32_t *tp = taps.data() + base + (axis ? L.w : 0);
            const int n = axis ? L.h : L.w, nt = axis ? pyr_nty : pyr_ntx, T = axis ? kPyrTileH : kPyrTileW;
            int i = 0;
            for (int t = 0; t <= nt; ++t) {
                while (i < n && (int)(tp[i] >> 9) < t * T) ++i;
                tiles_pyr.push_back((uint32_t)i);
            }
        }
        // Stage-1 tiles of the level, in an order that follows the hardware's hand-out of workgroups: consecutive
        // workgroups go to the eight XCDs in turn, each with an L2 of its own, so the table positions that fall to
        // one XCD get a run of tiles that are neighbours in the level and share their halo lines in that L2.
        {
            std::vector<uint32_t> row_major;
            for (int ty = 0; ty * kS1TileH < L.oh; ++ty)
                for (int tx = 0; tx * kS1TileW < L.ow; ++tx) row_major.push_back(pack_tile((int)l, ty, tx));
            const size_t first = tiles_s1.size(), m = row_major.size();
            tiles_s1.resize(first + m);
            size_t next = 0;
            for (size_t xcd = 0; xcd < 8; ++xcd)
                for (size_t p = 0; p < m; ++p)
                    if (((first + p) & 7) == xcd) tiles_s1[first + p] = row_major[next++];
        }
    }

    s1_tile_of_level[lv.size()] = (int)tiles_s1.size();
    // Chunks of the asynchronous mode: consecutive levels, cut where the running number of windows passes k / K of all
    {
        const int K = std::max(1, std::min(std::min(c->async_chunks, kMaxLevelChunks), (int)lv.size()));
        int k = 0;
        c->chunk_level[0] = 0;
        for (size_t l = 1; l < lv.size() && k + 1 < K; ++l)
            if ((int64_t)lv[l].score_off * K >= (int64_t)(k + 1) * n_windows) c->chunk_level[++k] = (int)l;
        c->n_chunks = k + 1;
        c->chunk_level[c->n_chunks] = (int)lv.size();
        for (int q = 0; q <= c->n_chunks; ++q) c->chunk_tile[q] = s1_tile_of_level[c->chunk_level[q]];
    }

    // buffers may be in use by work still queued on the last stream
    HIP_TRY(c, wait_last_stream(c));
    int rc;
    int64_t cap_levels = c->d_levels ? CNNC_MAX_LEVELS : 0;
    if ((rc = ensure(c, c->d_levels, cap_levels, CNNC_MAX_LEVELS))) return rc;
    if ((rc = ensure(c, c->d_taps, c->cap_taps, (int64_t)taps.size()))) return rc;
    if ((rc = ensure(c, c->d_tiles_pyr, c->cap_tiles_pyr, (int64_t)tiles_pyr.size()))) return rc;
    if ((rc = ensure(c, c->d_tiles_s1, c->cap_tiles_s1, (int64_t)tiles_s1.size()))) return rc;
    if ((rc = ensure(c, c->d_pyr, c->cap_pyr, pyr_bytes))) return rc;
    if ((rc = ensure(c, c->d_score1, c->cap_score1, n_windows))) return rc;
    const int64_t n_words = (int64_t)lv.back().word_off + (int64_t)lv.back().words_per_row * lv.back().oh;
    if ((rc = ensure(c, c->d_mask1, c->cap_mask1, n_words))) return rc;
    const int64_t nblocks = std::max<int64_t>(std::max<int64_t>((n_windows + kCompactPerBlock - 1) / kCompactPerBlock,
                                                                (c->max_surv + kCompactPerBlock - 1) / kCompactPerBlock),
                                              (n_words + kCompactBlock - 1) / kCompactBlock) + 1;
    for (int k = 0; k < 3; ++k) {            // one per stage: their compactions may run on different streams
        int64_t cap_blocks = c->cap_blocks;
        if ((rc = ensure(c, c->d_blockcnt[k], cap_blocks, nblocks))) return rc;
        if (k == 2) c->cap_blocks = (int32_t)cap_blocks;
    }

    HIP_TRY(c, hipMemcpy(c->d_levels, lv.data(), sizeof(LevelDev) * lv.size(), hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemcpy(c->d_taps, taps.data(), sizeof(uint32_t) * taps.size(), hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemcpy(c->d_tiles_pyr, tiles_pyr.data(), sizeof(uint32_t) * tiles_pyr.size(), hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemcpy(c->d_tiles_s1, tiles_s1.data(), sizeof(uint32_t) * tiles_s1.size(), hipMemcpyHostToDevice));

    c->levels = lv;
    c->n_levels = (int)lv.size();
    c->pyr_bytes = pyr_bytes; c->n_windows = n_windows; c->n_words = n_words;
    c->n_tiles_pyr = (int)tiles_pyr.size(); c->n_tiles_s1 = (int)tiles_s1.size();
    c->pyr_ntx = pyr_ntx; c->pyr_nty = pyr_nty;
    c->lay_w = w; c->lay_h = h; c->layout_valid = true;
    ++c->layout_serial;
    return CNNC_OK;
}

// ---- per-step timing with events on the caller's stream ---------------------------------------
hipEvent_t take_event(StepTimer &t)
{
    hipEvent_t e = nullptr;
    if (!t.pool.empty()) { e = t.pool.back(); t.pool.pop_back(); return e; }
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

using Timed = cnnc::ScopedTimer;

int fetch(cnnc_ctx *c, cnnc_det *out, int cap, int *n_out)
{
    HIP_TRY(c, wait_last_stream(c));
    const Counters &k = *c->h_cnt;
    // The detections made from the (possibly truncated) lists are handed over in every case; an overflow is reported
    // after the copy, so that "contents up to the capacity are valid" holds for this call too.
    const int n = k.n[3];
    if (n_out) *n_out = n;
    const int m = std::min(std::min(n, cap), c->merge_cap);
    if (m > kFastDets)   // the enqueued copy only brought the first kFastDets
        HIP_TRY(c, hipMemcpy(c->h_det + kFastDets, c->d_det + kFastDets, sizeof(cnnc_det) * (size_t)(m - kFastDets),
                             hipMemcpyDeviceToHost));
    if (m > 0) memcpy(out, c->h_det, sizeof(cnnc_det) * (size_t)m);
    for (int s = 0; s < 3; ++s)
        if (k.n[s] > c->max_surv)
            return fail(c, CNNC_E_OVERFLOW, "survivor list of stage " + std::to_string(s + 1) + " needs " +
                                                std::to_string(k.n[s]) + " entries; detections come from the truncated list");
    if (k.n[2] > c->merge_cap)
        return fail(c, CNNC_E_OVERFLOW, "merge input of " + std::to_string(k.n[2]) + " windows exceeds its capacity; "
                                        "detections come from the first " + std::to_string(c->merge_cap));
    return n > cap ? fail(c, CNNC_E_OVERFLOW, "detection array too small") : CNNC_OK;
}

// Enqueue the copy of the counters and of the detections to pinned host memory.
int enqueue_readback(cnnc_ctx *c, hipStream_t st)
{
    HIP_TRY(c, hipMemcpyAsync(c->h_cnt, c->d_cnt, sizeof(Counters), hipMemcpyDeviceToHost, st));
    HIP_TRY(c, hipMemcpyAsync(c->h_det, c->d_det, sizeof(cnnc_det) * (size_t)std::min(c->merge_cap, kFastDets),
                              hipMemcpyDeviceToHost, st));
    return CNNC_OK;
}

}  // namespace

namespace cnnc {
ScopedTimer::ScopedTimer(cnnc_ctx *c_, int step_, hipStream_t st_) : c(c_), step(step_), st(st_)
{
    if (c->timing && (b = take_event(c->timers[step]))) (void)hipEventRecord(b, st);
}
ScopedTimer::~ScopedTimer()
{
    if (!b) return;
    StepTimer &t = c->timers[step];
    hipEvent_t e = take_event(t);
    if (!e) { t.pool.push_back(b); return; }
    (void)hipEventRecord(e, st);
    t.begin.push_back(b); t.end.push_back(e);
}
}  // namespace cnnc

// ------------------------------------------------------------------------------------------------
extern "C" {

const char *cnnc_version(void) { return "cnnc 0.1 (gfx950)"; }

int cnnc_abi_sizes(int32_t *out, int n)
{
    const int32_t v[7] = {(int32_t)sizeof(cnnc_layer), (int32_t)sizeof(cnnc_stage_desc), (int32_t)sizeof(cnnc_params),
                          (int32_t)sizeof(cnnc_det), (int32_t)sizeof(cnnc_region), (int32_t)CNNC_T_COUNT,
                          (int32_t)sizeof(cnnc_rdet)};
    for (int i = 0; out && i < n && i < 7; ++i) out[i] = v[i];
    return 7;
}

const char *cnnc_last_error(const cnnc_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int cnnc_create(cnnc_ctx **out, const cnnc_stage_desc stages[3], int max_w, int max_h, int max_survivors)
{
    if (!out) return CNNC_E_INVAL;
    *out = nullptr;
    if (!stages || max_w < kWin || max_h < kWin || max_w > 16384 || max_h > 16384 || max_survivors < 1 ||
        max_survivors > (1 << 20))
        return CNNC_E_INVAL;
    const int a1 = check_stage(stages[0], kStage1, 4, 12);
    const int a2 = check_stage(stages[1], kStage2, 6, kS2In);
    const int a3 = check_stage(stages[2], kStage3, 7, kS3In);
    if (a1 < 1 || a2 != a1 || a3 != a1) return CNNC_E_INVAL;

    cnnc_ctx *c = new (std::nothrow) cnnc_ctx();
    if (!c) return CNNC_E_NOMEM;
    c->act = a1;
    c->max_w = max_w; c->max_h = max_h; c->max_surv = max_survivors;
    c->merge_cap = std::min(max_survivors, 32768);
    c->params.min_face = 60; c->params.scale_step = 1.25;
    c->params.thr[0] = c->params.thr[1] = c->params.thr[2] = 0.0f;
    c->params.merge_iou = 0.3f; c->params.min_neighbors = 1;

    auto bail = [&](int rc) { cnnc_destroy(c); return rc; };
    if (hipGetDevice(&c->device) != hipSuccess) return bail(CNNC_E_HIP);
    const int n_params[3] = {kS1Params, kS2Params, kS3Params};
    for (int s = 1; s < 3; ++s) {
        if (hipMalloc((void **)&c->d_wt[s], sizeof(float) * n_params[s]) != hipSuccess) return bail(CNNC_E_NOMEM);
        if (hipMemcpy(c->d_wt[s], stages[s].weights, sizeof(float) * n_params[s], hipMemcpyHostToDevice) != hipSuccess)
            return bail(CNNC_E_HIP);
    }
    {
        std::vector<float> prepared(kS1Prepared);
        stage1_prepare_weights(stages[0].weights, prepared.data());
        if (hipMalloc((void **)&c->d_wt[0], sizeof(float) * kS1Prepared) != hipSuccess) return bail(CNNC_E_NOMEM);
        if (hipMemcpy(c->d_wt[0], prepared.data(), sizeof(float) * kS1Prepared, hipMemcpyHostToDevice) != hipSuccess)
            return bail(CNNC_E_HIP);
        c->s1_literal = stage1_literal_create(prepared.data());  // optional: without it stage 1 reads its weights from memory
    }
    {
        std::vector<float> frag(eval2_frag_floats());
        eval2_make_fragments(stages[1].weights, frag.data());
        if (hipMalloc((void **)&c->d_frag[0], sizeof(float) * frag.size()) != hipSuccess) return bail(CNNC_E_NOMEM);
        if (hipMemcpy(c->d_frag[0], frag.data(), sizeof(float) * frag.size(), hipMemcpyHostToDevice) != hipSuccess)
            return bail(CNNC_E_HIP);
        if (hipMalloc((void **)&c->d_feat[0], sizeof(float) * eval2_feat_floats() * (size_t)max_survivors) != hipSuccess)
            return bail(CNNC_E_NOMEM);
    }
    {
        std::vector<float> frag(eval3_frag_floats());
        eval3_make_fragments(stages[2].weights, frag.data());
        if (hipMalloc((void **)&c->d_frag[1], sizeof(float) * frag.size()) != hipSuccess) return bail(CNNC_E_NOMEM);
        if (hipMemcpy(c->d_frag[1], frag.data(), sizeof(float) * frag.size(), hipMemcpyHostToDevice) != hipSuccess)
            return bail(CNNC_E_HIP);
        if (hipMalloc((void **)&c->d_feat[1], sizeof(float) * eval3_feat_floats() * (size_t)eval3_feat_rows(max_survivors)) != hipSuccess)
            return bail(CNNC_E_NOMEM);
    }
    for (int s = 0; s < 3; ++s) {
        if (hipMalloc((void **)&c->d_idx[s], sizeof(uint32_t) * (size_t)max_survivors) != hipSuccess) return bail(CNNC_E_NOMEM);
        if (hipMalloc((void **)&c->d_sc[s], sizeof(float) * (size_t)max_survivors) != hipSuccess) return bail(CNNC_E_NOMEM);
    }
    for (int s = 0; s < 2; ++s)
        if (hipMalloc((void **)&c->d_eval[s], sizeof(float) * (size_t)max_survivors) != hipSuccess) return bail(CNNC_E_NOMEM);
    for (int k = 0; k < kMaxLevelChunks; ++k)
        if (hipEventCreateWithFlags(&c->ev_s1[k], hipEventDisableTiming) != hipSuccess) return bail(CNNC_E_HIP);
    if (hipEventCreateWithFlags(&c->ev_done, hipEventDisableTiming) != hipSuccess) return bail(CNNC_E_HIP);
    if (hipMalloc((void **)&c->d_cnt, sizeof(Counters)) != hipSuccess) return bail(CNNC_E_NOMEM);
    if (hipMemset(c->d_cnt, 0, sizeof(Counters)) != hipSuccess) return bail(CNNC_E_HIP);
    if (hipHostMalloc((void **)&c->h_cnt, sizeof(Counters), hipHostMallocDefault) != hipSuccess) return bail(CNNC_E_NOMEM);
    memset(c->h_cnt, 0, sizeof(Counters));
    if (hipMalloc(&c->d_merge_ws, merge_workspace_bytes(c->merge_cap)) != hipSuccess) return bail(CNNC_E_NOMEM);
    if (merge_init_workspace(c) != hipSuccess) return bail(CNNC_E_HIP);
    if (hipMalloc((void **)&c->d_det, sizeof(cnnc_det) * (size_t)c->merge_cap) != hipSuccess) return bail(CNNC_E_NOMEM);
    if (hipHostMalloc((void **)&c->h_det, sizeof(cnnc_det) * (size_t)c->merge_cap, hipHostMallocDefault) != hipSuccess)
        return bail(CNNC_E_NOMEM);
    *out = c;
    return CNNC_OK;
}

int cnnc_destroy(cnnc_ctx *c)
{
    if (!c) return CNNC_E_INVAL;
    (void)hipDeviceSynchronize();
    for (int s = 0; s < 3; ++s) { (void)hipFree(c->d_wt[s]); (void)hipFree(c->d_idx[s]); (void)hipFree(c->d_sc[s]); }
    for (int s = 0; s < 2; ++s) { (void)hipFree(c->d_eval[s]); (void)hipFree(c->d_frag[s]); (void)hipFree(c->d_feat[s]); }
    stage1_literal_destroy(c->s1_literal);
    c->s1_literal = nullptr;
    scan_release(c);
    select_release(c);
    (void)hipFree(c->d_levels); (void)hipFree(c->d_taps); (void)hipFree(c->d_tiles_pyr); (void)hipFree(c->d_tiles_s1);
    (void)hipFree(c->d_pyr); (void)hipFree(c->d_score1); (void)hipFree(c->d_mask1); (void)hipFree(c->d_cnt);
    for (int k = 0; k < 3; ++k) (void)hipFree(c->d_blockcnt[k]);
    (void)hipFree(c->d_merge_ws); (void)hipFree(c->d_det);
    if (c->h_cnt) (void)hipHostFree(c->h_cnt);
    if (c->h_det) (void)hipHostFree(c->h_det);
    if (c->side) (void)hipStreamDestroy(c->side);
    for (int k = 0; k < kMaxLevelChunks; ++k)
        if (c->ev_s1[k]) (void)hipEventDestroy(c->ev_s1[k]);
    if (c->ev_done) (void)hipEventDestroy(c->ev_done);
    for (auto &t : c->timers) {
        for (auto e : t.begin) (void)hipEventDestroy(e);
        for (auto e : t.end) (void)hipEventDestroy(e);
        for (auto e : t.pool) (void)hipEventDestroy(e);
    }
    delete c;
    return CNNC_OK;
}

int cnnc_set_params(cnnc_ctx *c, const cnnc_params *p)
{
    if (!c) return CNNC_E_INVAL;
    if (!p) return fail(c, CNNC_E_INVAL, "null parameters");
    if (!(p->min_face >= kWin) || !(p->scale_step > 1.0) || !(p->merge_iou >= 0.0f) || !(p->merge_iou <= 1.0f) ||
        p->min_neighbors < 1)
        return fail(c, CNNC_E_INVAL, "parameter out of range");
    for (float t : p->thr)
        if (t != t) return fail(c, CNNC_E_INVAL, "threshold is NaN");
    if (p->min_face != c->params.min_face || p->scale_step != c->params.scale_step) { c->layout_valid = false; c->progress = 0; }
    c->params = *p;
    return CNNC_OK;
}

int cnnc_pyramid_layout(cnnc_ctx *c, int w, int h, int *n_levels, int32_t *lvl_w, int32_t *lvl_h, double *lvl_scale,
                        int64_t *pyr_off, int64_t *score_off)
{
    if (!c) return CNNC_E_INVAL;
    if (w < kWin || h < kWin || w > c->max_w || h > c->max_h) return fail(c, CNNC_E_INVAL, "frame size outside [12, max]");
    std::vector<LevelDev> lv;
    int64_t pb = 0, nw = 0;
    if (compute_levels(c, w, h, lv, pb, nw) != CNNC_OK) return fail(c, CNNC_E_INVAL, "frame has no pyramid level");
    if (n_levels) *n_levels = (int)lv.size();
    for (size_t l = 0; l < lv.size(); ++l) {
        if (lvl_w) lvl_w[l] = lv[l].w;
        if (lvl_h) lvl_h[l] = lv[l].h;
        if (lvl_scale) lvl_scale[l] = lv[l].scale;
        if (pyr_off) pyr_off[l] = lv[l].pyr_off;
        if (score_off) score_off[l] = lv[l].score_off;
    }
    if (pyr_off) pyr_off[lv.size()] = pb;
    if (score_off) score_off[lv.size()] = nw;
    return CNNC_OK;
}

int cnnc_build_pyramid(cnnc_ctx *c, const uint8_t *d_frame, int w, int h, int pitch, void *stream)
{
    if (!c) return CNNC_E_INVAL;
    if (!d_frame || pitch < w) return fail(c, CNNC_E_INVAL, "null frame or pitch < width");
    int rc = prepare_layout(c, w, h);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    c->d_frame = d_frame; c->fw = w; c->fh = h; c->fpitch = pitch;
    c->last_stream = st;
    c->progress = 0;
    c->scan_done = false;
    c->sel_done = false;
    {
        Timed t(c, CNNC_T_PYRAMID, st);
        HIP_TRY(c, launch_pyramid(c, st));
    }
    c->progress = DONE_PYR;
    return CNNC_OK;
}

int cnnc_stage1_scoremap(cnnc_ctx *c, void *stream)
{
    if (!c) return CNNC_E_INVAL;
    if (!(c->progress & DONE_PYR)) return fail(c, CNNC_E_STATE, "stage 1 needs a pyramid");
    hipStream_t st = (hipStream_t)stream;
    c->last_stream = st;
    {
        Timed t(c, CNNC_T_STAGE1, st);
        HIP_TRY(c, launch_stage1(c, 0, c->n_tiles_s1, st));
    }
    c->progress = DONE_PYR | DONE_S1;
    return CNNC_OK;
}

int cnnc_stage1_survivors(cnnc_ctx *c, float thr, void *stream)
{
    if (!c) return CNNC_E_INVAL;
    if (thr != thr) return fail(c, CNNC_E_INVAL, "threshold is NaN");
    if (!(c->progress & DONE_PYR)) return fail(c, CNNC_E_STATE, "stage 1 needs a pyramid");
    hipStream_t st = (hipStream_t)stream;
    c->last_stream = st;
    {
        Timed t(c, CNNC_T_STAGE1, st);
        HIP_TRY(c, launch_stage1_emit(c, thr, st));
    }
    {
        Timed t(c, CNNC_T_COMPACT1, st);
        HIP_TRY(c, launch_compact_mask(c, c->d_idx[0], c->d_sc[0], &c->d_cnt->n[0], st));
    }
    c->progress = DONE_PYR | DONE_C1;      // no score map: cnnc_get_scoremap reports CNNC_E_STATE
    return CNNC_OK;
}

int cnnc_set_literal_weights(cnnc_ctx *c, int on)
{
    if (!c) return CNNC_E_INVAL;
    c->use_literals = on != 0;
    return CNNC_OK;
}

int cnnc_literal_weights(const cnnc_ctx *c) { return c && c->use_literals && c->s1_literal ? 1 : 0; }

int cnnc_set_fused_stage1(cnnc_ctx *c, int on)
{
    if (!c) return CNNC_E_INVAL;
    c->fused_stage1 = on != 0;
    return CNNC_OK;
}

int cnnc_compact_survivors(cnnc_ctx *c, int stage, float thr, void *stream)
{
    if (!c) return CNNC_E_INVAL;
    if (stage < 1 || stage > 3) return fail(c, CNNC_E_INVAL, "stage must be 1, 2 or 3");
    if (thr != thr) return fail(c, CNNC_E_INVAL, "threshold is NaN");
    const int need[3] = {DONE_S1, DONE_E2, DONE_E3};
    if (!(c->progress & need[stage - 1])) return fail(c, CNNC_E_STATE, "compaction needs that stage's scores");
    hipStream_t st = (hipStream_t)stream;
    c->last_stream = st;
    {
        Timed t(c, CNNC_T_COMPACT1 + 2 * (stage - 1), st);
        CompactJob job{};
        job.slot = stage - 1; job.thr = thr;
        job.out_idx = c->d_idx[stage - 1]; job.out_sc = c->d_sc[stage - 1]; job.d_count = &c->d_cnt->n[stage - 1];
        if (stage == 1) {
            job.vals = c->d_score1; job.n_literal = c->n_windows;
        } else {
            job.vals = c->d_eval[stage - 2]; job.src_idx = c->d_idx[stage - 2];
            job.d_begin = &c->d_cnt->end[stage - 2][0]; job.d_end = &c->d_cnt->n[stage - 2];     // end[.][0] is always 0
        }
        HIP_TRY(c, launch_compact(c, job, st));
    }
    const int done[3] = {DONE_C1, DONE_C2, DONE_C3};
    const int keep[3] = {DONE_PYR | DONE_S1, DONE_PYR | DONE_S1 | DONE_C1 | DONE_E2,
                         DONE_PYR | DONE_S1 | DONE_C1 | DONE_E2 | DONE_C2 | DONE_E3};
    c->progress = (c->progress & keep[stage - 1]) | done[stage - 1];
    return CNNC_OK;
}

int cnnc_eval_stage(cnnc_ctx *c, int k, void *stream)
{
    if (!c) return CNNC_E_INVAL;
    if (k != 2 && k != 3) return fail(c, CNNC_E_INVAL, "stage must be 2 or 3");
    if (!(c->progress & (k == 2 ? DONE_C1 : DONE_C2))) return fail(c, CNNC_E_STATE, "evaluation needs the previous stage's survivors");
    hipStream_t st = (hipStream_t)stream;
    c->last_stream = st;
    {
        Timed t(c, k == 2 ? CNNC_T_STAGE2 : CNNC_T_STAGE3, st);
        const ListRange all{&c->d_cnt->end[k - 2][0], &c->d_cnt->n[k - 2]};                      // end[.][0] is always 0
        if (k == 2) HIP_TRY(c, c->eval_impl ? launch_eval2_mfma(c, all, st) : launch_eval2(c, all, st));
        else HIP_TRY(c, c->eval_impl ? launch_eval3_mfma(c, all, st) : launch_eval3(c, all, st));
    }
    const int keep = k == 2 ? (DONE_PYR | DONE_S1 | DONE_C1) : (DONE_PYR | DONE_S1 | DONE_C1 | DONE_E2 | DONE_C2);
    c->progress = (c->progress & keep) | (k == 2 ? DONE_E2 : DONE_E3);
    return CNNC_OK;
}

static int merge_enqueue(cnnc_ctx *c, hipStream_t st)
{
    if (!(c->progress & DONE_C3)) return fail(c, CNNC_E_STATE, "merging needs the stage-3 survivors");
    c->last_stream = st;
    {
        Timed t(c, CNNC_T_MERGE, st);
        HIP_TRY(c, launch_merge(c, st));
    }
    c->progress |= DONE_MERGE;
    return enqueue_readback(c, st);
}

int cnnc_merge_detections(cnnc_ctx *c, cnnc_det *out, int cap, int *n_out, void *stream)
{
    if (!c) return CNNC_E_INVAL;
    if ((!out && cap > 0) || cap < 0 || !n_out) return fail(c, CNNC_E_INVAL, "null output");
    int rc = merge_enqueue(c, (hipStream_t)stream);
    if (rc) return rc;
    return fetch(c, out, cap, n_out);
}

// The path in chunks of pyramid levels (paper, Section 3.4, asynchronous mode: the first stage moves on to the next
// level while the regions it has found are still being analysed).  Stage 1 and its compaction run chunk by chunk on
// the caller's stream and append to the stage-1 list; stages 2 and 3 of a chunk wait only for that chunk's event and
// run on the context's own stream; the lists grow in chunk order, so they are exactly the lists of the one-stream
// path.  No host wait anywhere: the caller's stream finally waits for the event behind the merge.  (A third stream
// for stage 3 was measured: every extra cross-stream dependency costs more than the overlap it buys.)
static int detect_chunked(cnnc_ctx *c, hipStream_t sa)
{
    Counters *k = c->d_cnt;
    const hipStream_t sb = c->side, sc = c->side;       // stages 2 and 3 share the context's stream (see below)
    const int K = c->n_chunks;
    for (int q = 0; q < K; ++q) {
        const bool last = q + 1 == K;
        const LevelDev &L0 = c->levels[c->chunk_level[q]];
        const int64_t off = L0.score_off;
        const int64_t len = (last ? c->n_windows : (int64_t)c->levels[c->chunk_level[q + 1]].score_off) - off;
        {
            Timed t(c, CNNC_T_STAGE1, sa);
            HIP_TRY(c, launch_stage1(c, c->chunk_tile[q], c->chunk_tile[q + 1], sa));
        }
        {
            Timed t(c, CNNC_T_COMPACT1, sa);
            CompactJob job{};
            job.slot = 0; job.vals = c->d_score1 + off; job.idx_base = (uint32_t)off; job.n_literal = len;
            job.thr = c->params.thr[0]; job.out_idx = c->d_idx[0]; job.out_sc = c->d_sc[0];
            job.d_base = &k->end[0][q]; job.d_count = &k->end[0][q + 1]; job.d_count2 = last ? &k->n[0] : nullptr;
            HIP_TRY(c, launch_compact(c, job, sa));
        }
        HIP_TRY(c, hipEventRecord(c->ev_s1[q], sa));
        HIP_TRY(c, hipStreamWaitEvent(sb, c->ev_s1[q], 0));
        const ListRange r1{&k->end[0][q], &k->end[0][q + 1]};
        {
            Timed t(c, CNNC_T_STAGE2, sb);
            HIP_TRY(c, launch_eval2_mfma(c, r1, sb));
        }
        {
            Timed t(c, CNNC_T_COMPACT2, sb);
            CompactJob job{};
            job.slot = 1; job.vals = c->d_eval[0]; job.src_idx = c->d_idx[0]; job.d_begin = r1.d_begin; job.d_end = r1.d_end;
            job.thr = c->params.thr[1]; job.out_idx = c->d_idx[1]; job.out_sc = c->d_sc[1];
            job.d_base = &k->end[1][q]; job.d_count = &k->end[1][q + 1]; job.d_count2 = last ? &k->n[1] : nullptr;
            HIP_TRY(c, launch_compact(c, job, sb));
        }
        const ListRange r2{&k->end[1][q], &k->end[1][q + 1]};
        {
            Timed t(c, CNNC_T_STAGE3, sc);
            HIP_TRY(c, launch_eval3_mfma(c, r2, sc));
        }
        {
            Timed t(c, CNNC_T_COMPACT3, sc);
            CompactJob job{};
            job.slot = 2; job.vals = c->d_eval[1]; job.src_idx = c->d_idx[1]; job.d_begin = r2.d_begin; job.d_end = r2.d_end;
            job.thr = c->params.thr[2]; job.out_idx = c->d_idx[2]; job.out_sc = c->d_sc[2];
            job.d_base = &k->end[2][q]; job.d_count = &k->end[2][q + 1]; job.d_count2 = last ? &k->n[2] : nullptr;
            HIP_TRY(c, launch_compact(c, job, sc));
        }
    }
    c->progress = DONE_PYR | DONE_S1 | DONE_C1 | DONE_E2 | DONE_C2 | DONE_E3 | DONE_C3;
    {
        Timed t(c, CNNC_T_MERGE, sc);
        HIP_TRY(c, launch_merge(c, sc));
    }
    c->progress |= DONE_MERGE;
    int rc = enqueue_readback(c, sc);
    if (rc) return rc;
    HIP_TRY(c, hipEventRecord(c->ev_done, sc));
    HIP_TRY(c, hipStreamWaitEvent(sa, c->ev_done, 0));
    c->last_stream = sa;
    return CNNC_OK;
}

int cnnc_set_async_chunks(cnnc_ctx *c, int chunks)
{
    if (!c) return CNNC_E_INVAL;
    if (chunks < 1 || chunks > kMaxLevelChunks) return fail(c, CNNC_E_INVAL, "chunks must be 1..8");
    if (chunks == c->async_chunks) return CNNC_OK;
    // The second stream exists only while it is used: a process has few hardware queues, and every stream that is alive
    // keeps its share of them whether it carries work or not.
    HIP_TRY(c, wait_last_stream(c));
    if (chunks > 1 && !c->side) HIP_TRY(c, hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking));
    if (chunks == 1 && c->side) {
        HIP_TRY(c, hipStreamSynchronize(c->side));
        HIP_TRY(c, hipStreamDestroy(c->side));
        c->side = nullptr;
    }
    c->async_chunks = chunks;
    c->layout_valid = false;
    c->progress = 0;
    return CNNC_OK;
}

int cnnc_detect_async(cnnc_ctx *c, const uint8_t *d_frame, int w, int h, int pitch, void *stream)
{
    int rc;
    if ((rc = cnnc_build_pyramid(c, d_frame, w, h, pitch, stream))) return rc;
    if (c->n_chunks > 1 && c->eval_impl != 0 && !c->fused_stage1) return detect_chunked(c, (hipStream_t)stream);
    if (c->fused_stage1) {
        if ((rc = cnnc_stage1_survivors(c, c->params.thr[0], stream))) return rc;
    } else {
        if ((rc = cnnc_stage1_scoremap(c, stream))) return rc;
        if ((rc = cnnc_compact_survivors(c, 1, c->params.thr[0], stream))) return rc;
    }
    if ((rc = cnnc_eval_stage(c, 2, stream))) return rc;
    if ((rc = cnnc_compact_survivors(c, 2, c->params.thr[1], stream))) return rc;
    if ((rc = cnnc_eval_stage(c, 3, stream))) return rc;
    if ((rc = cnnc_compact_survivors(c, 3, c->params.thr[2], stream))) return rc;
    return merge_enqueue(c, (hipStream_t)stream);
}

int cnnc_fetch_detections(cnnc_ctx *c, cnnc_det *out, int cap, int *n_out)
{
    if (!c) return CNNC_E_INVAL;
    if ((!out && cap > 0) || cap < 0 || !n_out) return fail(c, CNNC_E_INVAL, "null output");
    if (!(c->progress & DONE_MERGE)) return fail(c, CNNC_E_STATE, "no detection pass was enqueued");
    return fetch(c, out, cap, n_out);
}

int cnnc_detect(cnnc_ctx *c, const uint8_t *d_frame, int w, int h, int pitch, cnnc_det *out, int cap, int *n_out)
{
    if (!c) return CNNC_E_INVAL;
    if ((!out && cap > 0) || cap < 0 || !n_out) return fail(c, CNNC_E_INVAL, "null output");
    int rc = cnnc_detect_async(c, d_frame, w, h, pitch, nullptr);
    if (rc) return rc;
    return fetch(c, out, cap, n_out);
}

int cnnc_get_pyramid(cnnc_ctx *c, const uint8_t **d_pyramid, int64_t *n_bytes)
{
    if (!c) return CNNC_E_INVAL;
    if (!(c->progress & DONE_PYR)) return fail(c, CNNC_E_STATE, "no pyramid yet");
    if (d_pyramid) *d_pyramid = c->d_pyr;
    if (n_bytes) *n_bytes = c->pyr_bytes;
    return CNNC_OK;
}

int cnnc_get_scoremap(cnnc_ctx *c, const float **d_scores, int64_t *n_windows)
{
    if (!c) return CNNC_E_INVAL;
    if (!(c->progress & DONE_S1)) return fail(c, CNNC_E_STATE, "no score map yet");
    if (d_scores) *d_scores = c->d_score1;
    if (n_windows) *n_windows = c->n_windows;
    return CNNC_OK;
}

int cnnc_get_survivors(cnnc_ctx *c, int stage, const uint32_t **d_index, const float **d_score)
{
    if (!c) return CNNC_E_INVAL;
    if (stage < 1 || stage > 3) return fail(c, CNNC_E_INVAL, "stage must be 1, 2 or 3");
    const int done[3] = {DONE_C1, DONE_C2, DONE_C3};
    if (!(c->progress & done[stage - 1])) return fail(c, CNNC_E_STATE, "that stage was not compacted");
    if (d_index) *d_index = c->d_idx[stage - 1];
    if (d_score) *d_score = c->d_sc[stage - 1];
    return CNNC_OK;
}

int cnnc_get_stage_scores(cnnc_ctx *c, int k, const float **d_score)
{
    if (!c) return CNNC_E_INVAL;
    if (k != 2 && k != 3) return fail(c, CNNC_E_INVAL, "stage must be 2 or 3");
    if (!(c->progress & (k == 2 ? DONE_E2 : DONE_E3))) return fail(c, CNNC_E_STATE, "that stage was not evaluated");
    if (d_score) *d_score = c->d_eval[k - 2];
    return CNNC_OK;
}

int cnnc_survivor_count(cnnc_ctx *c, int stage, int *n, void *stream)
{
    if (!c) return CNNC_E_INVAL;
    if (stage < 1 || stage > 3 || !n) return fail(c, CNNC_E_INVAL, "bad stage or null output");
    const int done[3] = {DONE_C1, DONE_C2, DONE_C3};
    if (!(c->progress & done[stage - 1])) return fail(c, CNNC_E_STATE, "that stage was not compacted");
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(c, hipMemcpyAsync(c->h_cnt, c->d_cnt, sizeof(Counters), hipMemcpyDeviceToHost, st));
    HIP_TRY(c, hipStreamSynchronize(st));
    if (c->last_stream == st) c->last_stream = nullptr;
    *n = c->h_cnt->n[stage - 1];
    return *n > c->max_surv ? fail(c, CNNC_E_OVERFLOW, "survivor list truncated") : CNNC_OK;
}

int cnnc_set_eval_impl(cnnc_ctx *c, int impl)
{
    if (!c) return CNNC_E_INVAL;
    if (impl < 0 || impl > 3) return fail(c, CNNC_E_INVAL, "implementation must be 0, 1, 2 or 3");
    c->eval_impl = impl;
    return CNNC_OK;
}

int cnnc_executed_mfma(const cnnc_ctx *c, int k, int64_t *per_crop)
{
    if (!c || !per_crop || (k != 2 && k != 3)) return CNNC_E_INVAL;
    *per_crop = c->eval_impl == 0 ? 0 : (k == 2 ? eval2_mfma_per_crop(c->eval_impl) : eval3_mfma_per_crop(c->eval_impl));
    return CNNC_OK;
}

int cnnc_set_timing(cnnc_ctx *c, int on)
{
    if (!c) return CNNC_E_INVAL;
    c->timing = on != 0;
    return CNNC_OK;
}

int cnnc_get_timings(cnnc_ctx *c, double *ms_sum, int32_t *calls)
{
    if (!c) return CNNC_E_INVAL;
    HIP_TRY(c, wait_last_stream(c));
    for (int s = 0; s < CNNC_T_COUNT; ++s) {
        StepTimer &t = c->timers[s];
        for (size_t i = 0; i < t.begin.size(); ++i) {
            float ms = 0;
            HIP_TRY(c, hipEventSynchronize(t.end[i]));
            HIP_TRY(c, hipEventElapsedTime(&ms, t.begin[i], t.end[i]));
            t.ms += ms; t.calls += 1;
            t.pool.push_back(t.begin[i]); t.pool.push_back(t.end[i]);
        }
        t.begin.clear(); t.end.clear();
        if (ms_sum) ms_sum[s] = t.ms;
        if (calls) calls[s] = t.calls;
        t.ms = 0; t.calls = 0;
    }
    return CNNC_OK;
}

}  // extern "C"
