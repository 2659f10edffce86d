// First stage in the paper's own geometry (paper, Section 3.1: a CNN without fully connected layer,
// convolution stride 1, pooling stride 2; Section 3.3: the responses of its output layer correspond to a
// 27 x 31 window moved over a pyramid image with a 4 pixel step; Section 3.4: one fused routine per
// network instead of a stack of layers).
//
// The layer shapes were printed only in the paper's Figure 1.  Built in here:
//   conv 4x4 1->4, f, pool 2 | conv 3x3 4->11, f, pool 2 | conv 5x6 (width x height) 11->1
// which takes a 27 x 31 window to one response (806 parameters; the paper states 797).
// Because both pools are anchored at the level's corner, the whole scan is one pass of these layers over
// the level; a workgroup produces an 8 x 8 tile of responses from a 55 x 59 pixel patch with every
// intermediate map in LDS:
//   patch 55 x 59 -> conv1 52 x 56 x 4 -> pooled 26 x 28 x 4 -> conv2 24 x 26 x 11 -> pooled 12 x 13 x 11 -> 8 x 8.
// f is monotone, so it is applied after each max.  Weights are uniform per wave and come through scalar loads.
#include "act.h"
#include "cnnc_internal.h"

namespace cnnc {

namespace {
constexpr int kWinW = kScanWinW, kWinH = kScanWinH, kStep = kScanStep;
constexpr int kC1 = 4, kC2 = 11;
constexpr int kScanParams = 806;
// offsets (floats) inside the weight blob: per layer w[cout][cin][kh][kw] then bias[cout]
constexpr int W1 = 0, B1 = W1 + kC1 * 16, W2 = B1 + kC1, B2 = W2 + kC2 * kC1 * 9, W3 = B2 + kC2, B3 = W3 + kC2 * 30;
static_assert(B3 + 1 == kScanParams, "blob layout");

typedef uint32_t __attribute__((aligned(1))) pixel_quad;        // four neighbouring pixels of a row, any address
constexpr int kThreads = 256;
constexpr int TO = 8;                                           // responses per tile side
constexpr int IN_W = kStep * (TO - 1) + kWinW, IN_H = kStep * (TO - 1) + kWinH, IN_P = 56;   // 55 x 59 patch, row pitch 56
constexpr int P1_W = (IN_W - 3) / 2, P1_H = (IN_H - 3) / 2, P1_P = 28;                      // 26 x 28, row pitch 28
constexpr int P2_W = (P1_W - 2) / 2, P2_H = (P1_H - 2) / 2;                                 // 12 x 13
static_assert(P2_W - 5 + 1 == TO && P2_H - 6 + 1 == TO, "tile geometry");
static_assert(IN_W <= IN_P && 2 * (P1_W - 1) + 5 < IN_P && P1_W <= P1_P, "row pitches cover every read");
}  // namespace

template <int ACT>
__global__ __launch_bounds__(kThreads)
void scan_kernel(const uint8_t *__restrict__ pyr, const ScanLevel *__restrict__ levels, const uint32_t *__restrict__ tiles,
                 const float *__restrict__ wt, float *__restrict__ out)
{
    __shared__ __attribute__((aligned(16))) float sIn[IN_H * IN_P];
    __shared__ __attribute__((aligned(16))) float sP1[kC1 * P1_H * P1_P];
    __shared__ __attribute__((aligned(16))) float sP2[kC2 * P2_H * P2_W];
    __shared__ float sPart[4 * 64];

    const uint32_t t = tiles[blockIdx.x];
    const int lvl = t >> 24, ty = (t >> 12) & 0xFFF, tx = t & 0xFFF;
    const ScanLevel L = levels[lvl];
    const uint8_t *img = pyr + L.pyr_off;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int x_in = kStep * TO * tx, y_in = kStep * TO * ty;

    // ---- patch, normalised; positions past the level edge repeat the edge (they feed only responses that are not
    // written).  All loads of a thread are issued before the first is used.
    if (x_in + IN_P <= L.w && y_in + IN_H <= L.h) {
        constexpr int kQuads = IN_H * (IN_P / 4), kIt = (kQuads + kThreads - 1) / kThreads;
        uint32_t px[kIt];
#pragma unroll
        for (int it = 0; it < kIt; ++it) {
            const int e = min(it * kThreads + tid, kQuads - 1), r = e / (IN_P / 4), c = 4 * (e % (IN_P / 4));
            px[it] = *reinterpret_cast<const pixel_quad *>(img + (size_t)(y_in + r) * L.w + x_in + c);
        }
#pragma unroll
        for (int it = 0; it < kIt; ++it) {
            const int e = it * kThreads + tid;
            if (e < kQuads)
                *reinterpret_cast<float4 *>(sIn + 4 * e) =
                    make_float4(normalise((float)(px[it] & 255u)), normalise((float)((px[it] >> 8) & 255u)),
                                normalise((float)((px[it] >> 16) & 255u)), normalise((float)(px[it] >> 24)));
        }
    } else {
        constexpr int kIt = (IN_H * IN_P + kThreads - 1) / kThreads;
        uint8_t pb[kIt];
#pragma unroll
        for (int it = 0; it < kIt; ++it) {
            const int e = min(it * kThreads + tid, IN_H * IN_P - 1), r = e / IN_P, c = e % IN_P;
            pb[it] = img[(size_t)min(y_in + r, L.h - 1) * L.w + min(x_in + c, L.w - 1)];
        }
#pragma unroll
        for (int it = 0; it < kIt; ++it) {
            const int e = it * kThreads + tid;
            if (e < IN_H * IN_P) sIn[e] = normalise((float)pb[it]);
        }
    }
    __syncthreads();

    // ---- conv1 4x4 1->4, max over each 2x2 block, f: one pooled position (all four maps) per thread and round
    for (int p = tid; p < P1_H * P1_W; p += kThreads) {
        const int py = p / P1_W, px = p % P1_W;
        float acc[kC1][2][2];
#pragma unroll
        for (int ch = 0; ch < kC1; ++ch)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[ch][q >> 1][q & 1] = 0.0f;
#pragma unroll
        for (int r = 0; r < 5; ++r) {                            // patch rows 2 py .. 2 py + 4, columns 2 px .. 2 px + 4
            const float *row = sIn + (2 * py + r) * IN_P + 2 * px;
            const float2 r0 = *reinterpret_cast<const float2 *>(row), r1 = *reinterpret_cast<const float2 *>(row + 2),
                         r2 = *reinterpret_cast<const float2 *>(row + 4);
            const float v[6] = {r0.x, r0.y, r1.x, r1.y, r2.x, r2.y};
#pragma unroll
            for (int dy = 0; dy < 2; ++dy) {
                const int a = r - dy;
                if (a < 0 || a > 3) continue;
#pragma unroll
                for (int ch = 0; ch < kC1; ++ch)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const float w = wt[W1 + (ch * 4 + a) * 4 + b];
                        acc[ch][dy][0] = fmaf(w, v[b], acc[ch][dy][0]);
                        acc[ch][dy][1] = fmaf(w, v[b + 1], acc[ch][dy][1]);
                    }
            }
        }
#pragma unroll
        for (int ch = 0; ch < kC1; ++ch) {
            const float m = fmaxf(fmaxf(acc[ch][0][0], acc[ch][0][1]), fmaxf(acc[ch][1][0], acc[ch][1][1]));
            sP1[(ch * P1_H + py) * P1_P + px] = act_f<ACT>(m + wt[B1 + ch]);
        }
    }
    __syncthreads();

    // ---- conv2 3x3 4->11, max, f: lanes take pooled positions, wave w the output maps w, w + 4, w + 8
    for (int p = lane; p < P2_H * P2_W; p += 64) {
        const int qy = p / P2_W, qx = p % P2_W;
        float v[kC1][4][4];                                      // rows 2 qy .. 2 qy + 3, columns 2 qx .. 2 qx + 3 of every map
#pragma unroll
        for (int c = 0; c < kC1; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float *row = sP1 + (c * P1_H + 2 * qy + r) * P1_P + 2 * qx;
                const float2 r0 = *reinterpret_cast<const float2 *>(row), r1 = *reinterpret_cast<const float2 *>(row + 2);
                v[c][r][0] = r0.x; v[c][r][1] = r0.y; v[c][r][2] = r1.x; v[c][r][3] = r1.y;
            }
#pragma unroll
        for (int kk = 0; kk < 3; ++kk) {
            const int k = wave + 4 * kk;
            if (k >= kC2) break;
            float acc[2][2] = {{0.0f, 0.0f}, {0.0f, 0.0f}};
#pragma unroll
            for (int c = 0; c < kC1; ++c)
#pragma unroll
                for (int a = 0; a < 3; ++a)
#pragma unroll
                    for (int b = 0; b < 3; ++b) {
                        const float w = wt[W2 + ((k * kC1 + c) * 3 + a) * 3 + b];
#pragma unroll
                        for (int q = 0; q < 4; ++q) acc[q >> 1][q & 1] = fmaf(w, v[c][(q >> 1) + a][(q & 1) + b], acc[q >> 1][q & 1]);
                    }
            const float m = fmaxf(fmaxf(acc[0][0], acc[0][1]), fmaxf(acc[1][0], acc[1][1]));
            sP2[(k * P2_H + qy) * P2_W + qx] = act_f<ACT>(m + wt[B2 + k]);
        }
    }
    __syncthreads();

    // ---- conv3 5x6 11->1: lane = response of the tile, wave w sums the maps w, w + 4, w + 8
    {
        const int oy = lane >> 3, ox = lane & 7;
        float acc = 0.0f;
#pragma unroll
        for (int kk = 0; kk < 3; ++kk) {
            const int k = wave + 4 * kk;
            if (k >= kC2) break;
#pragma unroll
            for (int i = 0; i < 6; ++i)
#pragma unroll
                for (int j = 0; j < 5; ++j)
                    acc = fmaf(wt[W3 + (k * 6 + i) * 5 + j], sP2[(k * P2_H + oy + i) * P2_W + ox + j], acc);
        }
        sPart[wave * 64 + lane] = acc;
    }
    __syncthreads();
    if (tid < 64) {
        const int oy = tid >> 3, ox = tid & 7, gy = TO * ty + oy, gx = TO * tx + ox;
        if (gy < L.oh && gx < L.ow)
            out[(size_t)L.out_off + (size_t)gy * L.ow + gx] = ((sPart[tid] + sPart[64 + tid]) + (sPart[128 + tid] + sPart[192 + tid])) + wt[B3];
    }
}

namespace {
#define HIP_TRY(c, expr)                                         \
    do {                                                         \
        hipError_t e_ = (expr);                                  \
        if (e_ != hipSuccess) return hip_fail((c), e_, #expr);   \
    } while (0)

// Response-map geometry of the current pyramid: level l gives ((w - 27) / 4 + 1) x ((h - 31) / 4 + 1) responses,
// none when it is smaller than the window.
void scan_geometry(const std::vector<LevelDev> &lv, std::vector<ScanLevel> &sl, std::vector<uint32_t> *tiles, int64_t &total)
{
    sl.clear();
    total = 0;
    for (size_t l = 0; l < lv.size(); ++l) {
        ScanLevel S{};
        S.w = lv[l].w; S.h = lv[l].h; S.pyr_off = lv[l].pyr_off; S.out_off = (int32_t)total;
        if (S.w >= kWinW && S.h >= kWinH) { S.ow = (S.w - kWinW) / kStep + 1; S.oh = (S.h - kWinH) / kStep + 1; }
        total += (int64_t)S.ow * S.oh;
        if (tiles)
            for (int ty = 0; ty * TO < S.oh; ++ty)
                for (int tx = 0; tx * TO < S.ow; ++tx) tiles->push_back(pack_tile((int)l, ty, tx));
        sl.push_back(S);
    }
}
}  // namespace

void scan_release(cnnc_ctx *c)
{
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
    HIP_TRY(c, hipStreamSynchronize(c->last_stream));            // a scan may still be reading the old weights
    if (!c->d_scan_wt) HIP_TRY(c, hipMalloc((void **)&c->d_scan_wt, sizeof(float) * kScanParams));
    HIP_TRY(c, hipMemcpy(c->d_scan_wt, weights, sizeof(float) * kScanParams, hipMemcpyHostToDevice));
    c->scan_act = act;
    c->scan_done = false;
    c->sel_done = false;
    return CNNC_OK;
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
        scan_geometry(c->levels, sl, &tiles, total);
        HIP_TRY(c, hipStreamSynchronize(c->last_stream));        // the old tables may still be in use
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
        dim3 grid(c->n_scan_tiles), block(kThreads);
#define CNNC_SCAN(ACT) \
    hipLaunchKernelGGL(scan_kernel<ACT>, grid, block, 0, st, c->d_pyr, c->d_scan_levels, c->d_scan_tiles, c->d_scan_wt, c->d_scan_map)
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
