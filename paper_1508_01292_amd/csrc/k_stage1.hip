// Stage 1 (paper, Section 3.3: the first CNN densely scans every pyramid image; Section 3.4: the
// network is coded as one fused routine instead of a stack of layers).
//
// One launch covers every level through a (level, tile) table.  A workgroup produces a
// kS1TileW x kS1TileH tile of the score map from the (tile + 11)^2 input patch, all intermediates
// in LDS.  The stride-2 pool of the 12x12 network becomes a stride-1 max map M and a tap spacing
// of 2 in everything after it, which gives exactly the per-window result at every position:
//   A_c = f(b1_c + sum w1_c[a][b] X(y+a, x+b))                      conv 3x3, 1 -> 4
//   M_c = max of A_c over (y..y+1, x..x+1)
//   C_k = f(b2_k + sum w2_k[c][a][b] M_c(y+2a, x+2b))              conv 3x3, 4 -> 8, spacing 2
//   score = b3 + sum w3[k][i][j] C_k(y+2i, x+2j)                    fc over 8x3x3, spacing 2
#include "act.h"
#include "cnnc_internal.h"

namespace cnnc {

namespace {
constexpr int TW = kS1TileW, TH = kS1TileH;
constexpr int IN_W = TW + 11, IN_H = TH + 11;
constexpr int A_W = TW + 9, A_H = TH + 9;
constexpr int M_W = TW + 8, M_H = TH + 8;
constexpr int C_W = TW + 4, C_H = TH + 4;
constexpr int kThreads = 256;
constexpr int kRegionX = 8 * C_W * C_H;                 // C maps; earlier holds A maps + input
constexpr int kRegionM = 4 * M_W * M_H;
static_assert(4 * A_W * A_H + IN_W * IN_H <= kRegionX, "A maps and input must fit in the C region");
}  // namespace

template <int ACT>
__global__ __launch_bounds__(kThreads)
void stage1_kernel(const uint8_t *__restrict__ pyr, const LevelDev *__restrict__ levels,
                   const uint32_t *__restrict__ tiles, const float *__restrict__ wt,
                   float *__restrict__ score)
{
    __shared__ float sX[kRegionX];
    __shared__ float sM[kRegionM];
    float *sA = sX;                         // [4][A_H][A_W]
    float *sIn = sX + 4 * A_W * A_H;        // [IN_H][IN_W]
    float *sC = sX;                         // [8][C_H][C_W], written after A and the input are dead

    const uint32_t t = tiles[blockIdx.x];
    const int lvl = t >> 24, oy = ((t >> 12) & 0xFFF) * TH, ox = (t & 0xFFF) * TW;
    const LevelDev L = levels[lvl];
    const uint8_t *img = pyr + L.pyr_off;
    const int tid = threadIdx.x;

    // input patch, normalised; positions past the level edge repeat the edge (they only feed
    // outputs that are not written)
    for (int e = tid; e < IN_W * IN_H; e += kThreads) {
        const int r = e / IN_W, c = e % IN_W;
        const int y = min(oy + r, L.h - 1), x = min(ox + c, L.w - 1);
        sIn[e] = normalise((float)img[(size_t)y * L.w + x]);
    }
    __syncthreads();

    // conv1 + f
    for (int e = tid; e < A_W * A_H; e += kThreads) {
        const int r = e / A_W, c = e % A_W;
        float v[9];
#pragma unroll
        for (int a = 0; a < 3; ++a)
#pragma unroll
            for (int b = 0; b < 3; ++b) v[a * 3 + b] = sIn[(r + a) * IN_W + c + b];
#pragma unroll
        for (int ch = 0; ch < 4; ++ch) {
            float acc = wt[s1::B1 + ch];
#pragma unroll
            for (int q = 0; q < 9; ++q) acc = fmaf(wt[s1::W1 + ch * 9 + q], v[q], acc);
            sA[(ch * A_H + r) * A_W + c] = act_f<ACT>(acc);
        }
    }
    __syncthreads();

    // stride-1 2x2 max
    for (int e = tid; e < 4 * M_W * M_H; e += kThreads) {
        const int ch = e / (M_W * M_H), r = (e / M_W) % M_H, c = e % M_W;
        const float *p = sA + (ch * A_H + r) * A_W + c;
        sM[e] = fmaxf(fmaxf(p[0], p[1]), fmaxf(p[A_W], p[A_W + 1]));
    }
    __syncthreads();

    // conv2 (tap spacing 2) + f, all 8 output channels of a position in one thread
    for (int e = tid; e < C_W * C_H; e += kThreads) {
        const int r = e / C_W, c = e % C_W;
        float acc[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = wt[s1::B2 + k];
#pragma unroll
        for (int ch = 0; ch < 4; ++ch)
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int b = 0; b < 3; ++b) {
                    const float m = sM[(ch * M_H + r + 2 * a) * M_W + c + 2 * b];
#pragma unroll
                    for (int k = 0; k < 8; ++k)
                        acc[k] = fmaf(wt[s1::W2 + ((k * 4 + ch) * 3 + a) * 3 + b], m, acc[k]);
                }
#pragma unroll
        for (int k = 0; k < 8; ++k) sC[(k * C_H + r) * C_W + c] = act_f<ACT>(acc[k]);
    }
    __syncthreads();

    // fc over the 8x3x3 block at tap spacing 2
    for (int e = tid; e < TW * TH; e += kThreads) {
        const int r = e / TW, c = e % TW;
        const int y = oy + r, x = ox + c;
        if (y >= L.oh || x >= L.ow) continue;
        float acc = wt[s1::B3];
#pragma unroll
        for (int k = 0; k < 8; ++k)
#pragma unroll
            for (int i = 0; i < 3; ++i)
#pragma unroll
                for (int j = 0; j < 3; ++j)
                    acc = fmaf(wt[s1::W3 + (k * 3 + i) * 3 + j], sC[(k * C_H + r + 2 * i) * C_W + c + 2 * j], acc);
        score[(size_t)L.score_off + (size_t)y * L.ow + x] = acc;
    }
}

hipError_t launch_stage1(const cnnc_ctx *c, hipStream_t st)
{
    dim3 grid(c->n_tiles_s1), block(kThreads);
#define CNNC_S1(ACT)                                                                              \
    hipLaunchKernelGGL(stage1_kernel<ACT>, grid, block, 0, st, c->d_pyr, c->d_levels, c->d_tiles_s1, \
                       c->d_wt[0], c->d_score1)
    switch (c->act) {
    case CNNC_ACT_RATIONAL: CNNC_S1(CNNC_ACT_RATIONAL); break;
    case CNNC_ACT_SCALED_TANH: CNNC_S1(CNNC_ACT_SCALED_TANH); break;
    default: CNNC_S1(CNNC_ACT_TANH); break;
    }
#undef CNNC_S1
    return hipGetLastError();
}

}  // namespace cnnc
