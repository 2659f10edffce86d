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
// One workgroup per surviving position, everything of a region in 40 KiB of LDS (four workgroups per compute unit);
// workgroups stride over the survivor list whose length is read from device memory.  Per network pass: first
// convolution on the vector ALU with a thread per pooled position, second convolution on the matrix cores, output
// convolution split over ten groups of threads.
//
// The workgroup routine is written once for two kinds of operand of the first layers' weights (wave-uniform): a pointer
// (scalar loads) or literal constants that the host fills in (literal_weights.h).
#pragma once
#include "act.h"
#include "cnnc_internal.h"

namespace cnnc {

namespace selbody {
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

typedef float floatx4 __attribute__((ext_vector_type(4)));

// conv 4x4 1 -> C1 + 2x2 max-pool of the pre-activations + bias + f.  A thread takes a pooled position and all C1
// maps, so each of its 25 inputs is read once and the weights are wave-uniform (scalar loads).
// in: the region [kRegH][kRegP]; out: [C1][kP1H][kP1W].  MIRROR reads the columns right to left (the mirror image).
// W1T: what `w[i]` reads weight i of the layer (16 per map, then the biases) from: a pointer or literal constants.
template <int C1, bool MIRROR, int ACT, class W1T>
__device__ void conv1_pool(const float *in, float *out, const W1T w)
{
    for (int p = threadIdx.x; p < kP1H * kP1W; p += kThreads) {
        const int py = p / kP1W, px = p % kP1W;
        float acc[C1][4];                                         // the four positions of the pooling block: 2 dy + dx
#pragma unroll
        for (int ch = 0; ch < C1; ++ch)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[ch][q] = 0.0f;
#pragma unroll
        for (int r = 0; r < 5; ++r) {                            // region rows 2 py .. 2 py + 4, columns 2 px .. 2 px + 4
            float v[5];
#pragma unroll
            for (int c = 0; c < 5; ++c) v[c] = in[(2 * py + r) * kRegP + (MIRROR ? kRegW - 1 - (2 * px + c) : 2 * px + c)];
#pragma unroll
            for (int dy = 0; dy < 2; ++dy) {
                const int a = r - dy;
                if (a < 0 || a > 3) continue;
#pragma unroll
                for (int ch = 0; ch < C1; ++ch)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const float wv = w[(ch * 4 + a) * 4 + b];
                        acc[ch][2 * dy] = fmaf(wv, v[b], acc[ch][2 * dy]);
                        acc[ch][2 * dy + 1] = fmaf(wv, v[b + 1], acc[ch][2 * dy + 1]);
                    }
            }
        }
#pragma unroll
        for (int ch = 0; ch < C1; ++ch)
            out[(ch * kP1H + py) * kP1W + px] =
                act_f<ACT>(fmaxf(fmaxf(acc[ch][0], acc[ch][1]), fmaxf(acc[ch][2], acc[ch][3])) + w[C1 * 16 + ch]);
    }
    __syncthreads();
}

// conv 3x3 C1 -> C2 + 2x2 max-pool + bias + f on the matrix cores (it is 70 % of a network's arithmetic).
// GEMM rows = positions of the 22 x 24 map, sixteen a tile = four pooling blocks with their four positions each, so
// that a lane's four result registers are one block and the pooling stays in registers; K = C1 x 9 taps in steps of
// four (padded with zero weights), N = the C2 maps in two tiles of sixteen.  132 pooling blocks = 33 tiles: a wave takes
// eight of them, two at a time, and the last tile's two halves (of output maps) go to two waves.  frag: the B operand in lane order, [n tile][k step][64] (the output layer's weights follow it).
constexpr int kConv2Tiles = kP2W * kP2H / 4;
static_assert(kConv2Tiles * 4 == kP2W * kP2H && kConv2Tiles == 33, "pooling blocks come in fours");
constexpr int conv2_steps(int c1) { return (c1 * 9 + 3) / 4; }

template <int C1, int C2, int ACT>
__device__ void conv2_pool_mfma(const float *in, float *out, const float *__restrict__ frag, const float *__restrict__ bias)
{
    constexpr int K = C1 * 9, KS = conv2_steps(C1);
    static_assert(C2 > 16 && C2 <= 32, "two tiles of output maps");
    int lane = threadIdx.x & 63;
    // opaque per call: otherwise the weight fragments and tap offsets of all four network passes are hoisted out of
    // the loop over regions and kept alive across it, which spills 40 registers per lane
    asm volatile("" : "+v"(lane));
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), g = lane >> 4, i = lane & 15;
    float bf[2][KS];
    int koff[KS];
#pragma unroll
    for (int st = 0; st < KS; ++st) {
        bf[0][st] = frag[st * 64 + lane];
        bf[1][st] = frag[(KS + st) * 64 + lane];
        const int k = min(4 * st + g, K - 1), c = k / 9, a = (k % 9) / 3, b = k % 3;     // padded taps have zero weights
        koff[st] = (c * kP1H + a) * kP1W + b;
    }
    const int sub_off = ((i >> 1) & 1) * kP1W + (i & 1);          // position (i % 4) inside its pooling block
    const float bias0 = bias[i], bias1 = 16 + i < C2 ? bias[16 + i] : 0.0f;
    static_assert(kConv2Tiles == 33 && kThreads == 256, "four waves: eight tiles each in pairs, and the last tile's two halves");
#pragma unroll 1
    for (int t0 = wave; t0 < kConv2Tiles - 1; t0 += 8) {
        floatx4 acc[2][2];
        int base[2];
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            const int pb = 4 * (t0 + 4 * v) + (i >> 2), by = pb / kP2W, bx = pb % kP2W;
            base[v] = 2 * by * kP1W + 2 * bx + sub_off;
            acc[v][0] = acc[v][1] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
        }
#pragma unroll
        for (int st = 0; st < KS; ++st)
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                const float av = in[base[v] + koff[st]];
                acc[v][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bf[0][st], acc[v][0], 0, 0, 0);
                acc[v][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bf[1][st], acc[v][1], 0, 0, 0);
            }
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            const int pb = 4 * (t0 + 4 * v) + g, by = pb / kP2W, bx = pb % kP2W;    // lane (g, i): block g of the tile, map i
            const floatx4 lo = acc[v][0], hi = acc[v][1];
            out[(i * kP2H + by) * kP2P + bx] = act_f<ACT>(fmaxf(fmaxf(lo[0], lo[1]), fmaxf(lo[2], lo[3])) + bias0);
            if (16 + i < C2)
                out[((16 + i) * kP2H + by) * kP2P + bx] = act_f<ACT>(fmaxf(fmaxf(hi[0], hi[1]), fmaxf(hi[2], hi[3])) + bias1);
        }
    }
    if (wave < 2) {                                              // the thirty-third tile: wave 0 its first sixteen maps, wave 1 the rest
        constexpr int t = kConv2Tiles - 1;
        const int pa = 4 * t + (i >> 2), base = 2 * (pa / kP2W) * kP1W + 2 * (pa % kP2W) + sub_off;
        const int pb = 4 * t + g, by = pb / kP2W, bx = pb % kP2W;
        floatx4 acc = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
        if (wave == 0) {
#pragma unroll
            for (int st = 0; st < KS; ++st) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(in[base + koff[st]], bf[0][st], acc, 0, 0, 0);
            out[(i * kP2H + by) * kP2P + bx] = act_f<ACT>(fmaxf(fmaxf(acc[0], acc[1]), fmaxf(acc[2], acc[3])) + bias0);
        } else {
#pragma unroll
            for (int st = 0; st < KS; ++st) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(in[base + koff[st]], bf[1][st], acc, 0, 0, 0);
            if (16 + i < C2)
                out[((16 + i) * kP2H + by) * kP2P + bx] = act_f<ACT>(fmaxf(fmaxf(acc[0], acc[1]), fmaxf(acc[2], acc[3])) + bias1);
        }
    }
    __syncthreads();
}

// The output convolution (7 x 8 kernel over [C2][12][kP2P]) -> 25 responses in res[25].  A lane takes one row of five
// responses of one input map: per kernel row it reads the twelve values of a map row once (three 16-byte reads) for
// 35 multiply-adds, where a lane per response would read one value per multiply-add and be bound by LDS.  Lane =
// 8 x (map of the wave) + response row; a wave has up to eight maps, which are summed with three exchanges between
// lanes, and the four waves' sums meet in LDS.  wq: the layer's weights as [C2][8][8] (kernel rows padded to eight).
constexpr int kOutRowPad = 8;
template <int C2>
__device__ void conv_out(const float *in, const float *__restrict__ wq, const float *__restrict__ bias, float *part, float *res)
{
    static_assert(kK3W < kOutRowPad && kMapW - 1 + kK3W <= kP2P && kP2P == 12 && C2 <= 32 && kThreads == 256, "row of a map in three reads");
    constexpr int kPer = (C2 + 3) / 4;                           // maps per wave
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int v = lane & 7, kk = lane >> 3, k = wave * kPer + kk;
    float acc[kMapW];
#pragma unroll
    for (int u = 0; u < kMapW; ++u) acc[u] = 0.0f;
    if (v < kMapH && kk < kPer && k < C2) {
#pragma unroll
        for (int a = 0; a < kK3H; ++a) {
            const floatx4 *row = reinterpret_cast<const floatx4 *>(in + (k * kP2H + v + a) * kP2P);
            const floatx4 *wr = reinterpret_cast<const floatx4 *>(wq + (k * kK3H + a) * kOutRowPad);
            const floatx4 x0 = row[0], x1 = row[1], x2 = row[2], w0 = wr[0], w1 = wr[1];
            const float x[12] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3], x2[0], x2[1], x2[2], x2[3]};
            const float w[kOutRowPad] = {w0[0], w0[1], w0[2], w0[3], w1[0], w1[1], w1[2], w1[3]};
#pragma unroll
            for (int b = 0; b < kK3W; ++b)
#pragma unroll
                for (int u = 0; u < kMapW; ++u) acc[u] = fmaf(w[b], x[u + b], acc[u]);
        }
    }
#pragma unroll
    for (int u = 0; u < kMapW; ++u) {
        acc[u] += __shfl_xor(acc[u], 8, 64);
        acc[u] += __shfl_xor(acc[u], 16, 64);
        acc[u] += __shfl_xor(acc[u], 32, 64);
    }
    if (lane < kMapH)
#pragma unroll
        for (int u = 0; u < kMapW; ++u) part[wave * kMap + lane * kMapW + u] = acc[u];
    __syncthreads();
    if (tid < kMap) res[tid] = ((part[tid] + part[kMap + tid]) + (part[2 * kMap + tid] + part[3 * kMap + tid])) + bias[0];
    __syncthreads();
}

// One network on the region (and on its mirror image): res[25].
template <int C1, int C2, bool MIRROR, int ACT, class W1T>
__device__ void region_net(const float *sReg, float *sP1, float *sP2, float *sPart, const float *__restrict__ wt, const W1T w1,
                           const float *__restrict__ frag, float *res)
{
    constexpr int W1 = 0, B1 = W1 + C1 * 16, W2 = B1 + C1, B2 = W2 + C2 * C1 * 9, W3 = B2 + C2, B3 = W3 + C2 * kK3W * kK3H;
    (void)W2; (void)W3;
    static_assert(W1 == 0 && B1 == C1 * 16, "the first layer's weights and biases open the blob");
    conv1_pool<C1, MIRROR, ACT>(sReg, sP1, w1);
    conv2_pool_mfma<C1, C2, ACT>(sP1, sP2, frag, wt + B2);
    conv_out<C2>(sP2, frag + 2 * conv2_steps(C1) * 64, wt + B3, sPart, res);
}

// region + mirror -> combined map in sComb[25], written to `map`, and the count of responses above thr.
template <int C1, int C2, int ACT, class W1T>
__device__ int region_votes(const float *sReg, float *sP1, float *sP2, float *sPart, float *sRes, const float *__restrict__ wt,
                            const W1T w1, const float *__restrict__ frag, float thr, float *__restrict__ map)
{
    region_net<C1, C2, false, ACT>(sReg, sP1, sP2, sPart, wt, w1, frag, sRes);
    region_net<C1, C2, true, ACT>(sReg, sP1, sP2, sPart, wt, w1, frag, sRes + kMap);
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
// W2T / W3T: the operand type of the first layers' weights of CNN_2 and CNN_3 (pointer or literal constants).
template <int ACT, class W2T, class W3T>
__device__ __forceinline__ void select_regions(const uint8_t *__restrict__ frame, int fw, int fh, int pitch, const LevelDev *__restrict__ levels,
                   const ScanLevel *__restrict__ slev, int n_levels, const uint32_t *__restrict__ idx,
                   const float *__restrict__ resp, const int32_t *__restrict__ d_n, int n_max,
                   const float *__restrict__ w2, const float *__restrict__ w3, const W2T w2_first, const W3T w3_first,
                   const float *__restrict__ f2,
                   const float *__restrict__ f3, float t2, float t3, int t_nn, int rule,
                   cnnc_region *__restrict__ rec, float *__restrict__ maps2, float *__restrict__ maps3)
{
    // 40 KiB in all, so that four workgroups share a compute unit.  The sample tables, the histogram and the uint8
    // region are only needed until the equalised region is written and live in the (then idle) second map buffer;
    // the partial sums of the output convolution live in the first map buffer, which is idle by then.
    __shared__ float sReg[kRegH * kRegP];
    __shared__ float sP1[kC1Max * kP1H * kP1W];
    __shared__ __attribute__((aligned(16))) float sP2[kC2Max * kP2H * kP2P];
    __shared__ float sRes[2 * kMap];
    __shared__ int sC0;
    float *sPart = sP1;
    uint32_t *sTab = reinterpret_cast<uint32_t *>(sP2);
    int *sHist = reinterpret_cast<int *>(sP2) + 128;
    uint8_t *sPix = reinterpret_cast<uint8_t *>(sP2 + 128 + 256);
    static_assert(kRegW + kRegH <= 128 && (128 + 256) * 4 + kRegW * kRegH <= (int)sizeof(float) * kC2Max * kP2H * kP2P &&
                  4 * kMap <= kC1Max * kP1H * kP1W, "scratch arrays fit in the map buffers");
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

        // ---- CNN_2 on the region and its mirror image; under rule (2) CNN_3 only if CNN_2 left a vote (K2 = 0 already
        // decides); under rule (3) CNN_3's count alone can accept a region, so it always runs
        float *m2 = maps2 + (size_t)s * kMap, *m3 = maps3 + (size_t)s * kMap;
        const int k2 = region_votes<kNet2C1, kNet2C2, ACT>(sReg, sP1, sP2, sPart, sRes, w2, w2_first, f2, t2, m2);
        int k3 = 0;
        if (k2 > 0 || rule == 3) k3 = region_votes<kNet3C1, kNet3C2, ACT>(sReg, sP1, sP2, sPart, sRes, w3, w3_first, f3, t3, m3);
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

// literal weights of the first layers: CNN_2's 64 + 4, then CNN_3's 80 + 5
constexpr int kFirst2 = kNet2C1 * 17, kFirst3 = kNet3C1 * 17, kFirstLayers = kFirst2 + kFirst3;
}  // namespace selbody

}  // namespace cnnc
