// First stage in the paper's own geometry (paper, Section 3.1, 3.3: a 27 x 31 window at a 4 pixel step): host side and
// the kernel around the workgroup routine of scan_body.h.  As for stage 1 there are two builds of that routine: scan_kernel
// reads its weights from memory, and the code object of k_scan_lit.hip carries them as instruction literals that are
// filled in when cnnc_scan_set_weights is called (literal_weights.h); the second is used whenever its module loads.
#include "literal_weights.h"
#include "scan_body.h"

#include "scan_lit_image.inc"        // written by the build: kScanLitImage, kScanLitPatch

namespace cnnc {

using namespace scanbody;

constexpr int64_t kLargeTileMin = 128;       // 16 x 16 tiles from this many on: below, the smaller tiles reach more compute units

template <int ACT, class S>
__global__ __launch_bounds__(S::kThreads)
void scan_kernel(const uint8_t *__restrict__ pyr, const ScanLevel *__restrict__ levels, const uint32_t *__restrict__ tiles,
                 const float *__restrict__ wt, float *__restrict__ out)
{
    scan_tile<ACT, S>(pyr, levels, tiles, wt, out);
}

struct ScanLiteral {
    LiteralModule *mod = nullptr;
    hipFunction_t fn[3][2] = {};                             // [activation - 1][0: 8 x 8 tiles, 1: 16 x 16 tiles]
};

namespace {
void scan_literal_destroy(ScanLiteral *s)
{
    if (!s) return;
    literal_release(s->mod);
    delete s;
}

ScanLiteral *scan_literal_create(const float *weights)
{
    static const LiteralImage img = {kScanLitImage, sizeof(kScanLitImage), kScanLitPatch,
                                     sizeof(kScanLitPatch) / sizeof(kScanLitPatch[0]), kScanParams};
    LiteralModule *m = literal_acquire(img, weights);
    if (!m) return nullptr;
    ScanLiteral *s = new ScanLiteral();
    s->mod = m;
    static const char *const names[3][2] = {{"cnnc_scan_lit_act1_t8", "cnnc_scan_lit_act1_t16"},
                                            {"cnnc_scan_lit_act2_t8", "cnnc_scan_lit_act2_t16"},
                                            {"cnnc_scan_lit_act3_t8", "cnnc_scan_lit_act3_t16"}};
    for (int a = 0; a < 3; ++a)
        for (int t = 0; t < 2; ++t)
            if (!(s->fn[a][t] = literal_function(m, names[a][t]))) {
                scan_literal_destroy(s);
                return nullptr;
            }
    return s;
}
}  // namespace

namespace {
#define HIP_TRY(c, expr)                                         \
    do {                                                         \
        hipError_t e_ = (expr);                                  \
        if (e_ != hipSuccess) return hip_fail((c), e_, #expr);   \
    } while (0)

// Response-map geometry of the current pyramid: level l gives ((w - 27) / 4 + 1) x ((h - 31) / 4 + 1) responses,
// none when it is smaller than the window.
void scan_geometry(const std::vector<LevelDev> &lv, std::vector<ScanLevel> &sl, std::vector<uint32_t> *tiles, int64_t &total,
                   int tile_side = 8)
{
    sl.clear();
    total = 0;
    for (size_t l = 0; l < lv.size(); ++l) {
        ScanLevel S{};
        S.w = lv[l].w; S.h = lv[l].h; S.pyr_off = lv[l].pyr_off; S.out_off = (int32_t)total;
        if (S.w >= kWinW && S.h >= kWinH) { S.ow = (S.w - kWinW) / kStep + 1; S.oh = (S.h - kWinH) / kStep + 1; }
        total += (int64_t)S.ow * S.oh;
        if (tiles)
            for (int ty = 0; ty * tile_side < S.oh; ++ty)
                for (int tx = 0; tx * tile_side < S.ow; ++tx) tiles->push_back(pack_tile((int)l, ty, tx));
        sl.push_back(S);
    }
}
}  // namespace

void scan_release(cnnc_ctx *c)
{
    scan_literal_destroy(c->scan_literal);
    c->scan_literal = nullptr;
    (void)hipFree(c->d_scan_wt); (void)hipFree(c->d_scan_levels); (void)hipFree(c->d_scan_tiles); (void)hipFree(c->d_scan_map);
    c->d_scan_wt = nullptr; c->d_scan_levels = nullptr; c->d_scan_tiles = nullptr; c->d_scan_map = nullptr;
}

}  // namespace cnnc

using namespace cnnc;

extern "C" {

int cnnc_scan_set_weights(cnnc_ctx *c, const float *weights, int n_floats, int act)
{
    if (!c) return CNNC_E_INVAL;
    if (!weights || n_floats != kScanParams) return fail(c, CNNC_E_INVAL, "the scanning network has 806 parameters");
    if (act < CNNC_ACT_RATIONAL || act > CNNC_ACT_TANH) return fail(c, CNNC_E_INVAL, "activation kind must be 1, 2 or 3");
    HIP_TRY(c, wait_last_stream(c));            // a scan may still be reading the old weights
    if (!c->d_scan_wt) HIP_TRY(c, hipMalloc((void **)&c->d_scan_wt, sizeof(float) * kScanParams));
    HIP_TRY(c, hipMemcpy(c->d_scan_wt, weights, sizeof(float) * kScanParams, hipMemcpyHostToDevice));
    scan_literal_destroy(c->scan_literal);
    c->scan_literal = scan_literal_create(weights);              // optional: without it the scan reads its weights from memory
    c->scan_act = act;
    c->scan_done = false;
    c->sel_done = false;
    return CNNC_OK;
}

int cnnc_scan_set_tile(cnnc_ctx *c, int side)
{
    if (!c) return CNNC_E_INVAL;
    if (side != 0 && side != 8 && side != 16) return fail(c, CNNC_E_INVAL, "tile side must be 0 (chosen from the frame), 8 or 16");
    if (side != c->scan_tile_request) {
        c->scan_tile_request = side;
        c->scan_serial = -1;                                     // the tile table is rebuilt by the next scan
    }
    return CNNC_OK;
}

int cnnc_scan_tile(cnnc_ctx *c)
{
    return c ? c->scan_tile_side : CNNC_E_INVAL;
}

int cnnc_scan_layout(cnnc_ctx *c, int w, int h, int *n_levels, int32_t *out_w, int32_t *out_h, int64_t *out_off)
{
    if (!c || !n_levels) return CNNC_E_INVAL;
    if (w < kWin || h < kWin || w > c->max_w || h > c->max_h) return fail(c, CNNC_E_INVAL, "frame size outside [12, max]");
    std::vector<LevelDev> lv;
    int64_t pb = 0, nw = 0, total = 0;
    if (compute_levels(c, w, h, lv, pb, nw) != CNNC_OK) return fail(c, CNNC_E_INVAL, "frame has no pyramid level");
    std::vector<ScanLevel> sl;
    scan_geometry(lv, sl, nullptr, total);
    *n_levels = (int)sl.size();
    for (size_t l = 0; l < sl.size(); ++l) {
        if (out_w) out_w[l] = sl[l].ow;
        if (out_h) out_h[l] = sl[l].oh;
        if (out_off) out_off[l] = sl[l].out_off;
    }
    if (out_off) out_off[sl.size()] = total;
    return CNNC_OK;
}

int cnnc_scan_scoremap(cnnc_ctx *c, void *stream)
{
    if (!c) return CNNC_E_INVAL;
    if (!c->d_scan_wt) return fail(c, CNNC_E_STATE, "cnnc_scan_set_weights has not been called");
    if (!(c->progress & DONE_PYR)) return fail(c, CNNC_E_STATE, "the scan needs a pyramid");
    hipStream_t st = (hipStream_t)stream;
    if (c->scan_serial != c->layout_serial) {
        std::vector<ScanLevel> sl;
        std::vector<uint32_t> tiles;
        int64_t total = 0;
        // Tiles of 16 x 16 responses do a third less arithmetic per response; they are taken when there are enough of
        // them for two workgroups on every compute unit, otherwise 8 x 8 tiles spread the frame over more of the chip.
        int side = c->scan_tile_request;
        if (side == 0) {
            scan_geometry(c->levels, sl, &tiles, total, 16);
            side = (int64_t)tiles.size() >= kLargeTileMin ? 16 : 8;
            if (side != 16) tiles.clear();
        }
        if (tiles.empty()) scan_geometry(c->levels, sl, &tiles, total, side);
        c->scan_tile_side = side;
        HIP_TRY(c, wait_last_stream(c));        // the old tables may still be in use
        if (!c->d_scan_levels) HIP_TRY(c, hipMalloc((void **)&c->d_scan_levels, sizeof(ScanLevel) * CNNC_MAX_LEVELS));
        if ((int64_t)tiles.size() > c->cap_scan_tiles) {
            if (c->d_scan_tiles) { HIP_TRY(c, hipFree(c->d_scan_tiles)); c->d_scan_tiles = nullptr; c->cap_scan_tiles = 0; }
            HIP_TRY(c, hipMalloc((void **)&c->d_scan_tiles, sizeof(uint32_t) * tiles.size()));
            c->cap_scan_tiles = (int64_t)tiles.size();
        }
        if (total > c->cap_scan_map) {
            if (c->d_scan_map) { HIP_TRY(c, hipFree(c->d_scan_map)); c->d_scan_map = nullptr; c->cap_scan_map = 0; }
            HIP_TRY(c, hipMalloc((void **)&c->d_scan_map, sizeof(float) * (size_t)total));
            c->cap_scan_map = total;
        }
        HIP_TRY(c, hipMemcpy(c->d_scan_levels, sl.data(), sizeof(ScanLevel) * sl.size(), hipMemcpyHostToDevice));
        if (!tiles.empty())
            HIP_TRY(c, hipMemcpy(c->d_scan_tiles, tiles.data(), sizeof(uint32_t) * tiles.size(), hipMemcpyHostToDevice));
        c->n_scan_tiles = (int)tiles.size();
        c->n_scan = total;
        c->scan_serial = c->layout_serial;
    }
    c->last_stream = st;
    if (c->n_scan_tiles > 0) {
        ScopedTimer tm(c, CNNC_T_SCAN, st);
        const bool large = c->scan_tile_side == 16;
        const unsigned threads = large ? Shape16::kThreads : Shape8::kThreads;
        dim3 grid(c->n_scan_tiles), block(threads);
        if (c->scan_literal && c->use_literals) {
            const uint8_t *pyr = c->d_pyr;
            const ScanLevel *levels = c->d_scan_levels;
            const uint32_t *tiles = c->d_scan_tiles;
            float *out = c->d_scan_map;
            void *args[] = {&pyr, &levels, &tiles, &out};
            HIP_TRY(c, hipModuleLaunchKernel(c->scan_literal->fn[c->scan_act - 1][large ? 1 : 0], (unsigned)c->n_scan_tiles, 1, 1, threads, 1, 1, 0, st, args, nullptr));
        } else
#define CNNC_SCAN(ACT)                                                                                                        \
    do {                                                                                                                      \
        if (large) hipLaunchKernelGGL((scan_kernel<ACT, Shape16>), grid, block, 0, st, c->d_pyr, c->d_scan_levels, c->d_scan_tiles, c->d_scan_wt, c->d_scan_map); \
        else hipLaunchKernelGGL((scan_kernel<ACT, Shape8>), grid, block, 0, st, c->d_pyr, c->d_scan_levels, c->d_scan_tiles, c->d_scan_wt, c->d_scan_map);       \
    } while (0)
        switch (c->scan_act) {
        case CNNC_ACT_RATIONAL: CNNC_SCAN(CNNC_ACT_RATIONAL); break;
        case CNNC_ACT_SCALED_TANH: CNNC_SCAN(CNNC_ACT_SCALED_TANH); break;
        default: CNNC_SCAN(CNNC_ACT_TANH); break;
        }
#undef CNNC_SCAN
        HIP_TRY(c, hipGetLastError());
    }
    c->scan_done = true;
    c->sel_done = false;
    return CNNC_OK;
}

int cnnc_get_scan_scoremap(cnnc_ctx *c, const float **d_scores, int64_t *n)
{
    if (!c) return CNNC_E_INVAL;
    if (!c->scan_done) return fail(c, CNNC_E_STATE, "no response map: call cnnc_scan_scoremap first");
    if (d_scores) *d_scores = c->d_scan_map;
    if (n) *n = c->n_scan;
    return CNNC_OK;
}

}  // extern "C"
