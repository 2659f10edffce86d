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
// f is monotone, so it is applied after each max.
//
// The work of one workgroup, written once for two kinds of weight operand: WT is what `wt[i]` reads weight i of the
// blob from, a pointer (wave-uniform scalar loads) or LiteralWeights (instruction literals that the host fills in,
// literal_weights.h).
#pragma once
#include <type_traits>

#include "act.h"
#include "cnnc_internal.h"

namespace cnnc {

namespace scanbody {
constexpr int kWinW = kScanWinW, kWinH = kScanWinH, kStep = kScanStep;
constexpr int kC1 = 4, kC2 = 11;
constexpr int kScanParams = 806;
// offsets (floats) inside the weight blob: per layer w[cout][cin][kh][kw] then bias[cout]
constexpr int W1 = 0, B1 = W1 + kC1 * 16, W2 = B1 + kC1, B2 = W2 + kC2 * kC1 * 9, W3 = B2 + kC2, B3 = W3 + kC2 * 30;
static_assert(B3 + 1 == kScanParams, "blob layout");

typedef uint32_t __attribute__((aligned(1))) pixel_quad;        // four neighbouring pixels of a row, any address

// Geometry of a workgroup that produces TOX x TOY responses with THREADS threads.  A larger tile computes less of the
// border that neighbouring tiles compute again (the first convolution is evaluated on 2.8x the positions it needs at
// 8 x 8, on 1.8x at 16 x 16) but there are fewer of them to fill the chip with.
template <int TOX_, int TOY_, int THREADS_, int P1_PITCH_, int P2_PITCH_, int STRIP_>
struct Shape {
    static constexpr int TOX = TOX_, TOY = TOY_, kThreads = THREADS_, kWaves = THREADS_ / 64;
    static constexpr int IN_W = kStep * (TOX - 1) + kWinW, IN_H = kStep * (TOY - 1) + kWinH, IN_P = (IN_W + 4) / 4 * 4;   // patch
    static constexpr int P1_W = (IN_W - 3) / 2, P1_H = (IN_H - 3) / 2, P1_P = P1_PITCH_;                                 // after conv1, pool
    static constexpr int P2_W = (P1_W - 2) / 2, P2_H = (P1_H - 2) / 2, P2_P = P2_PITCH_;                                 // after conv2, pool
    static constexpr int R = TOX * TOY;                        // responses of a tile
    static constexpr int kStrip = STRIP_;                      // conv3: neighbouring responses of a row that a lane computes
    static constexpr int kPosGroups = kWaves / 4;              // conv2: four groups of maps x this many groups of positions
    static constexpr int kRespGroups = R / kStrip / 64;        // conv3: this many groups of responses x four groups of maps
    static constexpr int kInFloats = IN_H * IN_P, kP2Floats = kC2 * P2_H * P2_P;
    static_assert(P2_W - 5 + 1 == TOX && P2_H - 6 + 1 == TOY, "tile geometry");
    static_assert(IN_W < IN_P && IN_P % 4 == 0 && 2 * (P1_W - 1) + 5 < IN_P && P1_W <= P1_P && P1_P % 2 == 0 && P2_W <= P2_P,
                  "row pitches cover every read");
    static_assert(kWaves % 4 == 0 && R % (64 * kStrip) == 0 && kWaves == 4 * kRespGroups, "work split over the waves");
    static_assert(kStrip == 1 || (kStrip == 2 && TOX == 16 && TOY % 8 == 0 && P2_P % 2 == 0), "lane order of the strips");
};
// 55 x 59 patch -> 26 x 28 x 4 -> 12 x 13 x 11 -> 8 x 8 responses, 27 KB of LDS
typedef Shape<8, 8, 256, 28, 12, 1> Shape8;
// 87 x 91 patch -> 42 x 44 x 4 -> 20 x 21 x 11 -> 16 x 16 responses, 71 KB of LDS.  The row pitches 52 and 24 make the
// eight-byte reads of the second and third convolution free of bank conflicts (64 banks, 32 lanes a pass): 20 lanes
// of one row and 12 of the next cover 2 * 20 + 2 * 12 = 64 banks when two rows are 104 = 64 + 40 floats apart, and
// 4 strips x 8 rows of 8 floats each do when rows are 24 floats apart.
typedef Shape<16, 16, 512, 52, 24, 2> Shape16;

// The branch on `i` (0..3) is uniform over a wave and selects a copy of `f` in which the number is a constant, so that
// every weight index in it is one too.
template <class F>
__device__ __forceinline__ void for_constant4(int i, F &&f)
{
    switch (i) {
    case 0: f(std::integral_constant<int, 0>{}); break;
    case 1: f(std::integral_constant<int, 1>{}); break;
    case 2: f(std::integral_constant<int, 2>{}); break;
    default: f(std::integral_constant<int, 3>{}); break;
    }
}

template <int ACT, class S, class WT>
__device__ __forceinline__ void scan_tile(const uint8_t *__restrict__ pyr, const ScanLevel *__restrict__ levels,
                                          const uint32_t *__restrict__ tiles, const WT wt, float *__restrict__ out)
{
    constexpr int TOX = S::TOX, TOY = S::TOY, kThreads = S::kThreads, IN_W = S::IN_W, IN_H = S::IN_H, IN_P = S::IN_P,
                  P1_W = S::P1_W, P1_H = S::P1_H, P1_P = S::P1_P, P2_W = S::P2_W, P2_H = S::P2_H, P2_P = S::P2_P, R = S::R;
    // the patch is dead once the first convolution is done; the second one's result takes its place
    __shared__ __attribute__((aligned(16))) float sInP2[S::kInFloats > S::kP2Floats ? S::kInFloats : S::kP2Floats];
    __shared__ __attribute__((aligned(16))) float sP1[kC1 * P1_H * P1_P];
    __shared__ __attribute__((aligned(16))) float sPart[4 * R];
    float *const sIn = sInP2, *const sP2 = sInP2;
    (void)IN_W;

    const uint32_t t = tiles[blockIdx.x];
    const int lvl = t >> 24, ty = (t >> 12) & 0xFFF, tx = t & 0xFFF;
    const ScanLevel L = levels[lvl];
    const uint8_t *img = pyr + L.pyr_off;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int x_in = kStep * TOX * tx, y_in = kStep * TOY * ty;

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

    // ---- conv2 3x3 4->11, max, f: lanes take pooled positions; wave w the output maps w % 4, w % 4 + 4, w % 4 + 8 on
    // the positions of group w / 4
    for_constant4(wave & 3, [&](auto group) {
        constexpr int k0 = decltype(group)::value;
        for (int p = (wave >> 2) * 64 + lane; p < P2_H * P2_W; p += 64 * S::kPosGroups) {
            const int qy = p / P2_W, qx = p % P2_W;
            float v[kC1][4][4];                                  // rows 2 qy .. 2 qy + 3, columns 2 qx .. 2 qx + 3 of every map
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
                const int k = k0 + 4 * kk;
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
                sP2[(k * P2_H + qy) * P2_P + qx] = act_f<ACT>(m + wt[B2 + k]);
            }
        }
    });
    __syncthreads();

    // ---- conv3 5x6 11->1: wave w sums the maps w % 4, w % 4 + 4, w % 4 + 8 for the responses of group w / 4; a lane has
    // one response or a strip of two neighbours (then a half wave is 4 strips x 8 rows of the tile).  Every response is
    // summed in the same order whatever the tile.
    for_constant4(wave & 3, [&](auto group) {
        constexpr int k0 = decltype(group)::value;
        if constexpr (S::kStrip == 1) {
            const int r = (wave >> 2) * 64 + lane, oy = r / TOX, ox = r % TOX;
            float acc = 0.0f;
#pragma unroll
            for (int k = k0; k < kC2; k += 4)
#pragma unroll
                for (int i = 0; i < 6; ++i)
#pragma unroll
                    for (int j = 0; j < 5; ++j)
                        acc = fmaf(wt[W3 + (k * 6 + i) * 5 + j], sP2[(k * P2_H + oy + i) * P2_P + ox + j], acc);
            sPart[k0 * R + r] = acc;
        } else {
            const int oy = 8 * (wave >> 2) + ((lane >> 2) & 7), ox = 2 * (4 * (lane >> 5) + (lane & 3));
            float acc0 = 0.0f, acc1 = 0.0f;
#pragma unroll
            for (int k = k0; k < kC2; k += 4)
#pragma unroll
                for (int i = 0; i < 6; ++i) {
                    const float *row = sP2 + (k * P2_H + oy + i) * P2_P + ox;
                    const float2 r0 = *reinterpret_cast<const float2 *>(row), r1 = *reinterpret_cast<const float2 *>(row + 2),
                                 r2 = *reinterpret_cast<const float2 *>(row + 4);
                    const float v[6] = {r0.x, r0.y, r1.x, r1.y, r2.x, r2.y};
#pragma unroll
                    for (int j = 0; j < 5; ++j) {
                        const float w = wt[W3 + (k * 6 + i) * 5 + j];
                        acc0 = fmaf(w, v[j], acc0);
                        acc1 = fmaf(w, v[j + 1], acc1);
                    }
                }
            *reinterpret_cast<float2 *>(sPart + k0 * R + oy * TOX + ox) = make_float2(acc0, acc1);
        }
    });
    __syncthreads();
    if (tid < R) {
        const int oy = tid / TOX, ox = tid % TOX, gy = TOY * ty + oy, gx = TOX * tx + ox;
        if (gy < L.oh && gx < L.ow)
            out[(size_t)L.out_off + (size_t)gy * L.ow + gx] =
                ((sPart[tid] + sPart[R + tid]) + (sPart[2 * R + tid] + sPart[3 * R + tid])) + wt[B3];
    }
}
}  // namespace scanbody

}  // namespace cnnc
