// The selective unit in the paper's geometry (paper, Section 3.3): every window position of the first stage whose
// response exceeded T_1 is read from the original image together with a neighbourhood and scaled to 51 x 55 pixels,
// its histogram is equalised, and the region and its mirror image go through CNN_2 and CNN_3, each of which gives a
// 5 x 5 response map; the numbers K of responses above the threshold enter decision rule (2).
//
// Readings (the paper leaves them open; the shapes were in its Figure 1):
//   neighbourhood = 12 level pixels on every side of the 27 x 31 window (51 x 55 level pixels, resampled from the
//   frame in 16.16 fixed point with 8-bit weights and rounded to uint8 because a histogram follows);
//   equalisation v -> round((cdf(v) - c0) * 255 / (n - c0)), c0 = cdf of the smallest value present;
//   CNN_2 / CNN_3 = conv 4x4 1->c1, f, pool | conv 3x3 c1->c2, f, pool | conv 7x8 (w x h) c2->1 on a 35 x 39 window
//   at the 4 pixel step of the two pools, (c1, c2) = (4, 19) and (5, 28);
//   response (v, u) of the region and response (v, 4 - u) of the mirror image are averaged.
//
// One workgroup per surviving position, everything of a region in LDS; workgroups stride over the survivor list whose
// length is read from device memory.
#include "act.h"
#include "cnnc_internal.h"

namespace cnnc {

namespace {
constexpr int kThreads = 256;
constexpr int kRegW = 51, kRegH = 55, kRegP = 52, kMargin = 12;
constexpr int kWinW = 35, kWinH = 39;
constexpr int kP1W = (kRegW - 3) / 2, kP1H = (kRegH - 3) / 2;         // 24 x 26
constexpr int kP2W = (kP1W - 2) / 2, kP2H = (kP1H - 2) / 2, kP2P = 12; // 11 x 12
constexpr int kK3W = 7, kK3H = 8;
constexpr int kMapW = kP2W - kK3W + 1, kMapH = kP2H - kK3H + 1, kMap = kMapW * kMapH;
static_assert(kMapW == 5 && kMapH == 5 && (kRegW - kWinW) / 4 + 1 == 5 && (kRegH - kWinH) / 4 + 1 == 5, "5 x 5 response maps");
constexpr int kC1Max = 5, kC2Max = 28;

constexpr int net_params(int c1, int c2) { return c1 * 17 + c2 * (c1 * 9 + 1) + c2 * kK3W * kK3H + 1; }
constexpr int kNet2C1 = 4, kNet2C2 = 19, kNet3C1 = 5, kNet3C2 = 28;
constexpr int kNet2Params = net_params(kNet2C1, kNet2C2), kNet3Params = net_params(kNet3C1, kNet3C2);
static_assert(kNet2Params == 1836 && kNet3Params == 2942, "parameter counts of the chosen shapes");

// conv (KW x KH, stride 1) + 2x2 max-pool of the pre-activations + bias + f.  in: [CIN][.][IN_P], out: [COUT][PO_H][OUT_P].
// MIRROR reads the input columns right to left (the mirror image of a one-channel input).
template <int CIN, int COUT, int KW, int KH, int IN_W, int IN_H, int IN_P, int OUT_P, bool MIRROR, int ACT>
__device__ void conv_pool(const float *in, float *out, const float *__restrict__ w, const float *__restrict__ bias)
{
    constexpr int PO_W = (IN_W - KW + 1) / 2, PO_H = (IN_H - KH + 1) / 2;
    for (int e = threadIdx.x; e < COUT * PO_H * PO_W; e += kThreads) {
        const int oc = e / (PO_H * PO_W), py = (e / PO_W) % PO_H, px = e % PO_W;
        float a00 = 0.0f, a01 = 0.0f, a10 = 0.0f, a11 = 0.0f;
        const float *wp = w + oc * CIN * KW * KH;
        for (int ic = 0; ic < CIN; ++ic) {
            const float *ip = in + (ic * IN_H + 2 * py) * IN_P;
#pragma unroll
            for (int a = 0; a < KH + 1; ++a) {
                float v[KW + 1];
#pragma unroll
                for (int b = 0; b < KW + 1; ++b) v[b] = ip[a * IN_P + (MIRROR ? IN_W - 1 - (2 * px + b) : 2 * px + b)];
#pragma unroll
                for (int b = 0; b < KW; ++b) {
                    if (a < KH) {
                        const float wv = wp[(ic * KH + a) * KW + b];
                        a00 = fmaf(wv, v[b], a00);
                        a01 = fmaf(wv, v[b + 1], a01);
                    }
                    if (a > 0) {
                        const float wv = wp[(ic * KH + a - 1) * KW + b];
                        a10 = fmaf(wv, v[b], a10);
                        a11 = fmaf(wv, v[b + 1], a11);
                    }
                }
            }
        }
        out[(oc * PO_H + py) * OUT_P + px] = act_f<ACT>(fmaxf(fmaxf(a00, a01), fmaxf(a10, a11)) + bias[oc]);
    }
    __syncthreads();
}

// The output convolution (7 x 8 kernel over [C2][12][kP2P]) -> 25 responses in res[25].  Ten groups of threads split
// the input maps; their partial sums meet in LDS.
template <int C2>
__device__ void conv_out(const float *in, const float *__restrict__ w, const float *__restrict__ bias, float *part, float *res)
{
    const int tid = threadIdx.x;
    if (tid < 10 * kMap) {
        const int o = tid % kMap, grp = tid / kMap, v = o / kMapW, u = o % kMapW;
        float acc = 0.0f;
        for (int k = grp; k < C2; k += 10)
#pragma unroll
            for (int a = 0; a < kK3H; ++a)
#pragma unroll
                for (int b = 0; b < kK3W; ++b)
                    acc = fmaf(w[(k * kK3H + a) * kK3W + b], in[(k * kP2H + v + a) * kP2P + u + b], acc);
        part[grp * kMap + o] = acc;
    }
    __syncthreads();
    if (tid < kMap) {
        float s = bias[0];
        for (int g = 0; g < 10; ++g) s += part[g * kMap + tid];
        res[tid] = s;
    }
    __syncthreads();
}

// One network on the region (and on its mirror image): res[25].
template <int C1, int C2, bool MIRROR, int ACT>
__device__ void region_net(const float *sReg, float *sP1, float *sP2, float *sPart, const float *__restrict__ wt, float *res)
{
    constexpr int W1 = 0, B1 = W1 + C1 * 16, W2 = B1 + C1, B2 = W2 + C2 * C1 * 9, W3 = B2 + C2, B3 = W3 + C2 * kK3W * kK3H;
    conv_pool<1, C1, 4, 4, kRegW, kRegH, kRegP, kP1W, MIRROR, ACT>(sReg, sP1, wt + W1, wt + B1);
    conv_pool<C1, C2, 3, 3, kP1W, kP1H, kP1W, kP2P, false, ACT>(sP1, sP2, wt + W2, wt + B2);
    conv_out<C2>(sP2, wt + W3, wt + B3, sPart, res);
}

// region + mirror -> combined map in sComb[25], written to `map`, and the count of responses above thr.
template <int C1, int C2, int ACT>
__device__ int region_votes(const float *sReg, float *sP1, float *sP2, float *sPart, float *sRes, const float *__restrict__ wt,
                            float thr, float *__restrict__ map)
{
    region_net<C1, C2, false, ACT>(sReg, sP1, sP2, sPart, wt, sRes);
    region_net<C1, C2, true, ACT>(sReg, sP1, sP2, sPart, wt, sRes + kMap);
    int votes = 0;
    if (threadIdx.x < 64) {
        const int o = threadIdx.x, v = o / kMapW, u = o % kMapW;
        float r = 0.0f;
        if (o < kMap) {
            r = 0.5f * (sRes[o] + sRes[kMap + v * kMapW + (kMapW - 1 - u)]);
            map[o] = r;
        }
        votes = __popcll(__ballot(o < kMap && r > thr));
        if (o == 0) sPart[0] = __int_as_float(votes);
    }
    __syncthreads();
    votes = __float_as_int(sPart[0]);
    __syncthreads();
    return votes;
}
}  // namespace

template <int ACT>
__global__ __launch_bounds__(kThreads)
void select_kernel(const uint8_t *__restrict__ frame, int fw, int fh, int pitch, const LevelDev *__restrict__ levels,
                   const ScanLevel *__restrict__ slev, int n_levels, const uint32_t *__restrict__ idx,
                   const float *__restrict__ resp, const int32_t *__restrict__ d_n, int n_max,
                   const float *__restrict__ w2, const float *__restrict__ w3, float t2, float t3, int t_nn, int rule,
                   cnnc_region *__restrict__ rec, float *__restrict__ maps2, float *__restrict__ maps3)
{
    __shared__ float sReg[kRegH * kRegP];
    __shared__ float sP1[kC1Max * kP1H * kP1W];
    __shared__ float sP2[kC2Max * kP2H * kP2P];
    __shared__ float sPart[10 * kMap];
    __shared__ float sRes[2 * kMap];
    __shared__ uint32_t sTab[kRegW + kRegH];
    __shared__ int sHist[256];
    __shared__ int sC0;
    __shared__ uint8_t sPix[kRegW * kRegH];
    const int tid = threadIdx.x;
    const int n = min(*d_n, n_max);
    for (int s = blockIdx.x; s < n; s += gridDim.x) {
        // ---- which window: level, column i, row j of the response map
        const uint32_t g = idx[s];
        int l = 0;
        while (l + 1 < n_levels && g >= (uint32_t)slev[l + 1].out_off) ++l;
        const int rel = (int)(g - (uint32_t)slev[l].out_off), ow = slev[l].ow;
        const int wj = rel / ow, wi = rel % ow;
        const int64_t S = levels[l].scale_q16;

        // ---- region with its neighbourhood from the frame, rounded to uint8; histogram
        if (tid < kRegW + kRegH) {
            const bool is_y = tid >= kRegW;
            const int i = is_y ? tid - kRegW : tid, n_in = is_y ? fh : fw;
            const int origin = kScanStep * (is_y ? wj : wi) - kMargin;
            int64_t P = (int64_t)origin * S + ((int64_t)(2 * i + 1) * S) / 2 - 32768;
            const int64_t hi = (int64_t)(n_in - 1) << 16;
            P = P < 0 ? 0 : (P > hi ? hi : P);
            sTab[tid] = ((uint32_t)(P >> 16) << 9) | (uint32_t)(((P & 0xFFFF) + 128) >> 8);
        }
        sHist[tid] = 0;
        if (tid == 0) sC0 = 0x7fffffff;
        __syncthreads();
        for (int e = tid; e < kRegW * kRegH; e += kThreads) {
            const int r = e / kRegW, c = e % kRegW;
            const uint32_t ex = sTab[c], ey = sTab[kRegW + r];
            const int xa = ex >> 9, ya = ey >> 9, xb = min(xa + 1, fw - 1), yb = min(ya + 1, fh - 1);
            const uint32_t qx = ex & 511u, qy = ey & 511u;
            const uint8_t *r0 = frame + (size_t)ya * pitch, *r1 = frame + (size_t)yb * pitch;
            const uint32_t sum = r0[xa] * (256u - qx) * (256u - qy) + r0[xb] * qx * (256u - qy) + r1[xa] * (256u - qx) * qy + r1[xb] * qx * qy;
            const uint32_t p = (sum + 32768u) >> 16;
            sPix[e] = (uint8_t)p;
            atomicAdd(&sHist[p], 1);
        }
        __syncthreads();
        // ---- cumulative histogram (wave 0: four bins per lane), smallest non-zero value of it, look-up table
        if (tid < 64) {
            const int h0 = sHist[4 * tid], h1 = sHist[4 * tid + 1], h2 = sHist[4 * tid + 2], h3 = sHist[4 * tid + 3];
            int incl = h0 + h1 + h2 + h3;
            const int own = incl;
            for (int d = 1; d < 64; d <<= 1) {
                const int o = __shfl_up(incl, d, 64);
                if (tid >= d) incl += o;
            }
            const int base = incl - own;
            sHist[4 * tid] = base + h0;
            sHist[4 * tid + 1] = base + h0 + h1;
            sHist[4 * tid + 2] = base + h0 + h1 + h2;
            sHist[4 * tid + 3] = incl;
        }
        __syncthreads();
        if (sHist[tid] > 0) atomicMin(&sC0, sHist[tid]);
        __syncthreads();
        {
            const int nn = kRegW * kRegH, c0 = sC0, cdf = sHist[tid];
            int lut = tid;
            if (nn > c0) lut = cdf >= c0 ? (2 * (cdf - c0) * 255 + (nn - c0)) / (2 * (nn - c0)) : 0;
            __syncthreads();
            sHist[tid] = lut;
        }
        __syncthreads();
        for (int e = tid; e < kRegW * kRegH; e += kThreads)
            sReg[(e / kRegW) * kRegP + e % kRegW] = normalise((float)sHist[sPix[e]]);
        __syncthreads();

        // ---- CNN_2 on the region and its mirror image; CNN_3 only if CNN_2 left a vote; decision rule (2)
        float *m2 = maps2 + (size_t)s * kMap, *m3 = maps3 + (size_t)s * kMap;
        const int k2 = region_votes<kNet2C1, kNet2C2, ACT>(sReg, sP1, sP2, sPart, sRes, w2, t2, m2);
        int k3 = 0;
        if (k2 > 0) k3 = region_votes<kNet3C1, kNet3C2, ACT>(sReg, sP1, sP2, sPart, sRes, w3, t3, m3);
        else if (tid < kMap) m3[tid] = 0.0f;
        if (tid == 0) {
            cnnc_region R;
            R.index = (int32_t)g; R.level = l; R.i = wi; R.j = wj; R.k2 = k2; R.k3 = k3;
            if (rule == 3) R.face = (k2 >= t_nn || k3 >= t_nn) ? 1 : 0;                          // eq. (3), Section 4.3
            else R.face = ((k2 >= t_nn && k3 > 0) || (k2 > 0 && k3 >= t_nn)) ? 1 : 0;              // eq. (2)
            R.response = resp[s];
            rec[s] = R;
        }
        __syncthreads();
    }
}

void select_release(cnnc_ctx *c)
{
    (void)hipFree(c->d_sel_w2); (void)hipFree(c->d_sel_w3); (void)hipFree(c->d_sel_idx); (void)hipFree(c->d_sel_sc);
    (void)hipFree(c->d_sel_rec); (void)hipFree(c->d_sel_maps); (void)hipFree(c->d_sel_cnt);
    (void)hipFree(c->d_sel_fsc); (void)hipFree(c->d_sel_pick); (void)hipFree(c->d_sel_det);
    c->d_sel_fsc = nullptr; c->d_sel_pick = nullptr; c->d_sel_det = nullptr;
    if (c->h_sel_cnt) (void)hipHostFree(c->h_sel_cnt);
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
    HIP_TRY(c, hipStreamSynchronize(c->last_stream));
    if (!c->d_sel_w2) {
        const size_t cap = (size_t)c->max_surv;
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_w2, sizeof(float) * kNet2Params));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_w3, sizeof(float) * kNet3Params));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_idx, sizeof(uint32_t) * cap));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_sc, sizeof(float) * cap));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_rec, sizeof(cnnc_region) * cap));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_maps, sizeof(float) * 2 * kMap * cap));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_cnt, sizeof(int32_t) * 4));
        HIP_TRY(c, hipHostMalloc((void **)&c->h_sel_cnt, sizeof(int32_t) * 4, hipHostMallocDefault));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_fsc, sizeof(float) * (size_t)c->merge_cap));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_pick, sizeof(uint32_t) * (size_t)c->merge_cap));
        HIP_TRY(c, hipMalloc((void **)&c->d_sel_det, sizeof(cnnc_rdet) * (size_t)c->merge_cap));
    }
    HIP_TRY(c, hipMemcpy(c->d_sel_w2, w2, sizeof(float) * kNet2Params, hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemcpy(c->d_sel_w3, w3, sizeof(float) * kNet3Params, hipMemcpyHostToDevice));
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
    HIP_TRY(c, launch_compact(c, c->d_scan_map, nullptr, nullptr, c->n_scan, t1, c->d_sel_idx, c->d_sel_sc, c->d_sel_cnt, st));
    dim3 grid(256 * 3), block(kThreads);
    float *m2 = c->d_sel_maps, *m3 = c->d_sel_maps + (size_t)kMap * c->max_surv;
#define CNNC_SEL(ACT)                                                                                             \
    hipLaunchKernelGGL(select_kernel<ACT>, grid, block, 0, st, c->d_frame, c->fw, c->fh, c->fpitch, c->d_levels,  \
                       c->d_scan_levels, c->n_levels, c->d_sel_idx, c->d_sel_sc, c->d_sel_cnt, c->max_surv,       \
                       c->d_sel_w2, c->d_sel_w3, t2, t3, t_nn, c->sel_rule, c->d_sel_rec, m2, m3)
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
    HIP_TRY(c, hipStreamSynchronize(c->last_stream));
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
    HIP_TRY(c, hipStreamSynchronize(st));
    *n_out = 0;
    if (c->h_sel_cnt[0] > c->max_surv) return fail(c, CNNC_E_OVERFLOW, "more positions passed T_1 than the context's survivor capacity");
    if (c->h_sel_cnt[1] > c->merge_cap) return fail(c, CNNC_E_OVERFLOW, "more regions accepted than the merge can take");
    const int total = c->h_sel_cnt[2], m = std::min(total, cap);
    *n_out = total;
    if (m > 0) HIP_TRY(c, hipMemcpy(out, c->d_sel_det, sizeof(cnnc_rdet) * (size_t)m, hipMemcpyDeviceToHost));
    if (total > cap) return fail(c, CNNC_E_OVERFLOW, "output array too small");
    return CNNC_OK;
}

}  // extern "C"
