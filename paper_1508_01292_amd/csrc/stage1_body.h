// Stage 1 (paper, Section 3.3: the first CNN densely scans every pyramid image; Section 3.4: the
// network is coded as one fused routine instead of a stack of layers): the work of one workgroup, written once
// for two kinds of weight operand.
//
// A workgroup produces a kS1TileW x kS1TileH tile of the score map from the (tile + 11)^2 input patch, all
// intermediates in LDS.  The stride-2 pool of the 12x12 network becomes a stride-1 max map M and a tap spacing
// of 2 in everything after it, which gives exactly the per-window result at every position:
//   A_c = f(b1_c + sum w1_c[a][b] X(y+a, x+b))                      conv 3x3, 1 -> 4
//   M_c = max of A_c over (y..y+1, x..x+1)
//   C_k = f(b2_k + sum w2_k[c][a][b] M_c(y+2a, x+2b))              conv 3x3, 4 -> 8, spacing 2 (Winograd F(3,3) along rows)
//   score = b3 + sum w3[k][i][j] C_k(y+2i, x+2j)                    fc over 8x3x3, spacing 2
//
// Register blocking: a thread computes four (conv2: three) neighbouring positions at a time, so every
// LDS value is read once per unit.  For the spacing-2 layers the maps M and C are stored with even and
// odd columns apart ([channel][row][column parity][column / 2]); the positions of a thread are then
// consecutive entries of one parity, and their taps are consecutive too.  The unit sizes are chosen so
// that every phase fills the 256 threads (250, 240, 240 units, and 128 units by two halves of the channels).
//
// WT is what `wt[i]` reads weight i of the prepared array (layout s1p: conv2 in the Winograd domain) from: a pointer (wave-uniform scalar loads; a multiply-add
// with a scalar-register operand issues at half the rate of one with vector or literal operands on this chip), or
// LiteralWeights (every weight a distinct constant that the compiler encodes as an instruction literal; the host
// overwrites those literals with a weight set before it loads the code).
#pragma once
#include <type_traits>

#include "act.h"
#include "cnnc_internal.h"

namespace cnnc {

namespace s1body {
constexpr int TW = kS1TileW, TH = kS1TileH;
static_assert(TW == 32 && TH == 16, "the unit decomposition below is written for 32 x 16 tiles");
constexpr int kThreads = 256;
constexpr int IN_H = TH + 11, IN_P = 44;          // input patch rows, row pitch (43 columns used)
constexpr int A_H = TH + 9, A_P = 44;             // conv1 map: 41 columns used
constexpr int M_H = TH + 8, M_P = 40;             // max map: 2 parities x 20 columns
constexpr int C_H = TH + 4, C_P = 40;             // conv2 map: 2 parities x 20 columns (18 used)
constexpr int kIn = IN_H * IN_P + 4, kA = 4 * A_H * A_P, kM = 4 * M_H * M_P, kC = 8 * C_H * C_P;
constexpr int kRegionX = kC > kA + kIn ? kC : kA + kIn;   // A maps + input, later the C maps

typedef uint32_t __attribute__((aligned(1))) pixel_quad;        // four neighbouring pixels of a row, any address

struct f6 { float v[6]; };
// six consecutive floats starting at a 16-byte aligned LDS address
__device__ __forceinline__ f6 load6(const float *p)
{
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float2 b = *reinterpret_cast<const float2 *>(p + 4);
    return {{a.x, a.y, a.z, a.w, b.x, b.y}};
}

// EMIT = false: every score goes to the score map.  EMIT = true: only windows with score > thr leave the kernel,
// as one bit per window (a word per 32-window row of the tile, collected in LDS and stored by one thread, so the
// words in memory have one writer each and need no clearing) plus the score at the window's place in the map.
template <int ACT, bool EMIT, class WT>
__device__ __forceinline__ void stage1_tile(const uint8_t *__restrict__ pyr, const LevelDev *__restrict__ levels,
                                            const uint32_t *__restrict__ tiles, const WT wt,
                                            float *__restrict__ score, float thr, uint32_t *__restrict__ mask)
{
    // 40 KiB: four workgroups share a compute unit's LDS.  sM sits first so that the two floats some lanes
    // read past its end (feeding only discarded columns) fall inside the same array.
    __shared__ __attribute__((aligned(16))) float sAll[kM + kRegionX];
    float *sM = sAll, *sX = sAll + kM;
    float *sA = sX;                 // [4][A_H][A_P]
    float *sIn = sX + kA;           // [IN_H][IN_P]
    float *sC = sX;                 // [8][C_H][2][20], written after A and the input are dead

    const uint32_t t = tiles[blockIdx.x];
    const int lvl = t >> 24, oy = ((t >> 12) & 0xFFF) * TH, ox = (t & 0xFFF) * TW;
    const LevelDev L = levels[lvl];
    const uint8_t *img = pyr + L.pyr_off;
    const int tid = threadIdx.x;

    // ---- input patch, normalised; positions past the level edge repeat the edge (they only feed
    // outputs that are not written)
    if (ox + IN_P <= L.w && oy + IN_H <= L.h) {
        // the whole patch lies inside the level: four pixels a load
        for (int e = tid; e < IN_H * (IN_P / 4); e += kThreads) {
            const int r = e / (IN_P / 4), c = 4 * (e % (IN_P / 4));
            const uint32_t p = *reinterpret_cast<const pixel_quad *>(img + (size_t)(oy + r) * L.w + ox + c);
            *reinterpret_cast<float4 *>(sIn + r * IN_P + c) =
                make_float4(normalise((float)(p & 255u)), normalise((float)((p >> 8) & 255u)),
                            normalise((float)((p >> 16) & 255u)), normalise((float)(p >> 24)));
        }
        if (tid < 4) sIn[IN_H * IN_P + tid] = 0.0f;
    } else {
        for (int e = tid; e < kIn; e += kThreads) {
            const int r = min(e / IN_P, IN_H - 1), c = e % IN_P;
            const int y = min(oy + r, L.h - 1), x = min(ox + c, L.w - 1);
            sIn[e] = normalise((float)img[(size_t)y * L.w + x]);
        }
    }
    __syncthreads();

    // ---- conv1 + f: 25 rows x 10 groups of four columns, then the single column 40 by 25 threads of the last wave
    if (tid < A_H * 10) {
        const int r = tid / 10, x0 = 4 * (tid % 10);
        float acc[4][4];
#pragma unroll
        for (int ch = 0; ch < 4; ++ch)
#pragma unroll
            for (int p = 0; p < 4; ++p) acc[ch][p] = wt[s1p::B1 + ch];
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            const f6 in = load6(sIn + (r + a) * IN_P + x0);
#pragma unroll
            for (int b = 0; b < 3; ++b)
#pragma unroll
                for (int ch = 0; ch < 4; ++ch)
#pragma unroll
                    for (int p = 0; p < 4; ++p) acc[ch][p] = fmaf(wt[s1p::W1 + ch * 9 + a * 3 + b], in.v[p + b], acc[ch][p]);
        }
#pragma unroll
        for (int ch = 0; ch < 4; ++ch)
            *reinterpret_cast<float4 *>(sA + (ch * A_H + r) * A_P + x0) =
                make_float4(act_f<ACT>(acc[ch][0]), act_f<ACT>(acc[ch][1]), act_f<ACT>(acc[ch][2]), act_f<ACT>(acc[ch][3]));
    }
    if (tid >= 192 && tid < 192 + A_H) {
        // column 40: a row each, all four channels
        const int r = tid - 192;
        float acc[4];
#pragma unroll
        for (int ch = 0; ch < 4; ++ch) acc[ch] = wt[s1p::B1 + ch];
#pragma unroll
        for (int a = 0; a < 3; ++a)
#pragma unroll
            for (int b = 0; b < 3; ++b) {
                const float v = sIn[(r + a) * IN_P + 40 + b];
#pragma unroll
                for (int ch = 0; ch < 4; ++ch) acc[ch] = fmaf(wt[s1p::W1 + ch * 9 + a * 3 + b], v, acc[ch]);
            }
#pragma unroll
        for (int ch = 0; ch < 4; ++ch) sA[(ch * A_H + r) * A_P + 40] = act_f<ACT>(acc[ch]);
    }
    __syncthreads();

    // ---- stride-1 2x2 max, stored with even and odd columns apart: 24 rows x 10 groups of four columns
    if (tid < M_H * 10) {
        const int r = tid / 10, g = tid % 10, x0 = 4 * g;
#pragma unroll
        for (int ch = 0; ch < 4; ++ch) {
            const float *p0 = sA + (ch * A_H + r) * A_P + x0, *p1 = p0 + A_P;
            const float4 u = *reinterpret_cast<const float4 *>(p0), v = *reinterpret_cast<const float4 *>(p1);
            const float u4 = p0[4], v4 = p1[4];
            const float c0 = fmaxf(u.x, v.x), c1 = fmaxf(u.y, v.y), c2 = fmaxf(u.z, v.z), c3 = fmaxf(u.w, v.w),
                        c4 = fmaxf(u4, v4);
            float *m = sM + (ch * M_H + r) * M_P + 2 * g;
            *reinterpret_cast<float2 *>(m) = make_float2(fmaxf(c0, c1), fmaxf(c2, c3));        // even columns x0, x0+2
            *reinterpret_cast<float2 *>(m + 20) = make_float2(fmaxf(c1, c2), fmaxf(c3, c4));   // odd columns x0+1, x0+3
        }
    }
    __syncthreads();

    // ---- conv2 (tap spacing 2) + f: 20 rows x 2 parities x 6 groups of three same-parity columns (18 per parity
    // are needed), all 8 channels: 240 units for the 256 threads.  Three neighbouring outputs of a 3-tap row filter
    // by the Winograd form F(3,3): five multiplications instead of nine,
    //   m = (G w) * (BT d),  out = AT m summed over input channels and kernel rows before AT is applied,
    //   BT = [2 -1 -2 1 0; 0 -2 -1 1 0; 0 2 -3 1 0; 0 -1 0 1 0; 0 2 -1 -2 1],  AT = [1 1 1 1 0; 0 1 -1 2 0; 0 1 1 4 1];
    // the input transform (nine operations per five-vector) is shared by the eight output channels.
    if (tid < C_H * 12) {
        const int r = tid / 12, px = (tid % 12) / 6, j0 = 3 * (tid % 6);
        float m[8][5];
#pragma unroll
        for (int ch = 0; ch < 4; ++ch)
#pragma unroll
            for (int a = 0; a < 3; ++a) {
                const float *mp = sM + (ch * M_H + r + 2 * a) * M_P + px * 20 + j0;
                float d[5];
#pragma unroll
                for (int b = 0; b < 5; ++b) d[b] = mp[b];
                const float v3 = d[3] - d[1];
                const float v[5] = {fmaf(2.0f, d[0] - d[2], v3), v3 - (d[1] + d[2]), fmaf(3.0f, d[1] - d[2], v3), v3,
                                    fmaf(-2.0f, v3, d[4] - d[2])};
#pragma unroll
                for (int k = 0; k < 8; ++k)
#pragma unroll
                    for (int p = 0; p < 5; ++p) {
                        const float u = wt[s1p::U2 + (((k * 4 + ch) * 3 + a) * 5) + p];
                        // the bias rides on m0 and m4, which enter the first and the last output once each
                        if (ch == 0 && a == 0) m[k][p] = (p == 0 || p == 4) ? fmaf(u, v[p], wt[s1p::B2 + k]) : u * v[p];
                        else m[k][p] = fmaf(u, v[p], m[k][p]);
                    }
            }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float s = m[k][1] + m[k][2], t = m[k][1] - m[k][2];
            float *cp = sC + (k * C_H + r) * C_P + px * 20 + j0;
            cp[0] = act_f<ACT>(m[k][0] + s + m[k][3]);
            cp[1] = act_f<ACT>(fmaf(2.0f, m[k][3], t) + wt[s1p::B2 + k]);
            cp[2] = act_f<ACT>(fmaf(4.0f, m[k][3], s) + m[k][4]);
        }
    }
    __syncthreads();

    // ---- fc over the 8x3x3 block at tap spacing 2: 16 rows x 2 parities x 4 groups of four same-parity columns = 128
    // units.  Waves 0, 1 sum channels 0..3 of a unit, waves 2, 3 channels 4..7 (a wave-uniform choice, so every weight
    // index is a constant); the halves meet in LDS, in the max-map buffer, which is idle by now.
    // Lane order inside a wave: (group, parity, row) bits spread so that the sixteen lanes the LDS serves together
    // read sixteen different 16-byte columns of the banks.
    {
        const int lane = tid & 63, wave = tid >> 6;
        const int half = __builtin_amdgcn_readfirstlane(wave >> 1);
        const int r = 8 * (wave & 1) + (((lane >> 5) & 1) | (((lane >> 3) & 1) << 1) | (((lane >> 4) & 1) << 2));
        const int px = (lane >> 2) & 1, j0 = 4 * (lane & 3);
        const int unit = (r * 2 + px) * 4 + (lane & 3);
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        auto four_channels = [&](auto first) {
            constexpr int K0 = decltype(first)::value;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const f6 c = load6(sC + ((K0 + kk) * C_H + r + 2 * i) * C_P + px * 20 + j0);
#pragma unroll
                    for (int j = 0; j < 3; ++j) {
                        const float w = wt[s1p::W3 + ((K0 + kk) * 3 + i) * 3 + j];
#pragma unroll
                        for (int p = 0; p < 4; ++p) acc[p] = fmaf(w, c.v[p + j], acc[p]);
                    }
                }
        };
        if (half) {
            four_channels(std::integral_constant<int, 4>{});
            *reinterpret_cast<float4 *>(sM + 4 * unit) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        } else {
            four_channels(std::integral_constant<int, 0>{});
        }
        uint32_t *sBits = reinterpret_cast<uint32_t *>(sM + 4 * 128);      // EMIT: one word per row of the tile
        if (EMIT && tid < TH) sBits[tid] = 0u;
        __syncthreads();
        const int y = oy + r;
        if (!half) {
            const float4 other = *reinterpret_cast<const float4 *>(sM + 4 * unit);
            const float b3 = wt[s1p::B3];
            const float sc[4] = {acc[0] + other.x + b3, acc[1] + other.y + b3, acc[2] + other.z + b3, acc[3] + other.w + b3};
            float *row = score + (size_t)L.score_off + (size_t)y * L.ow;
            uint32_t bits = 0;                   // EMIT: this thread's four windows of the row's 32-bit word
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int x = ox + 2 * (j0 + p) + px;
                if (y < L.oh && x < L.ow) {
                    if (!EMIT) {
                        row[x] = sc[p];
                    } else if (sc[p] > thr) {
                        row[x] = sc[p];
                        bits |= 1u << (x - ox);
                    }
                }
            }
            if (EMIT && bits) atomicOr(&sBits[r], bits);
        }
        if (EMIT) {
            __syncthreads();
            if (tid < TH && oy + tid < L.oh) mask[L.word_off + (oy + tid) * L.words_per_row + ox / TW] = sBits[tid];
        }
    }
}
}  // namespace s1body

}  // namespace cnnc
