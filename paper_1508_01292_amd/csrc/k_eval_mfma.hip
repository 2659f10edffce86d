// Stages 2 and 3 on the matrix cores (paper, Section 3.3, selective unit; Section 3.4: code written
// for each network shape).
//
// The convolutions of the later stages are dense contractions once a crop sits in LDS: stage-3 conv2
// is M = 324 positions x N = 32 channels x K = 400 per crop.  They run as implicit GEMMs on
// v_mfma_f32_16x16x4_f32 (fp32 in, fp32 accumulate):
//   * A operand (16 positions x 4 k) is read straight from the LDS map: lane (i = lane % 16,
//     g = lane / 16) reads the input value of position i for k-index g of the step.
//   * B operand (4 k x 16 channels) comes from weights that the host re-orders once into the lane
//     order of the instruction ("fragments"), so a wave loads them with one coalesced access.
//   * The 16 positions of a tile are four 2x2 pooling blocks, so the four accumulator registers of a
//     lane are exactly one pooling block of one channel: max-pool, bias and activation happen in
//     registers and only the pooled map goes back to LDS.
// The order of the k-indices is free as long as A and B agree; it is chosen so that the LDS address
// of the A operand is (per-lane base) + (compile-time or wave-uniform offset).
//
// The fully connected layers are batched over crops in a second kernel (M = crops), so their
// weights are read once per 16 crops instead of once per crop.
#include <type_traits>

#include "eval_common.h"

namespace cnnc {

typedef float floatx4 __attribute__((ext_vector_type(4)));
#define CNNC_MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x4f32((a), (b), (c), 0, 0, 0)

namespace {
using namespace evalc;

__device__ __forceinline__ float max4(const floatx4 v) { return fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])); }

// ---- stage 3 geometry ---------------------------------------------------------------------------
constexpr int kCropW = 48;                 // crop row pitch in LDS
constexpr int kP1Row = 24, kP1Ch = 22 * kP1Row;   // pooled conv1 map [16][22][24] (row padded: bank spread)
constexpr int kP2Ch = 81;                  // pooled conv2 map [32][9][9] of the direct-sum variant
constexpr int kP2RowW = 10, kP2ChW = 9 * kP2RowW;   // Winograd variant: rows padded to 10 so that row reads are 8-byte aligned
constexpr int kRegionA = 32 * kP2ChW;      // crop (2304) then pooled conv2 map (2592 or 2880)
// position of pooling block `blk` (0..80) of channel `oc` in the pooled conv2 map
template <int WINO>
__device__ __forceinline__ int p2_index(int oc, int blk)
{
    return WINO ? oc * kP2ChW + (blk / 9) * kP2RowW + blk % 9 : oc * kP2Ch + blk;
}
constexpr int kRegionB = 16 * kP1Ch;       // pooled conv1 map (8448) then conv3 partial sums [4][32][66]
constexpr int kP3Pitch = 66;
static_assert(4 * 32 * kP3Pitch <= kRegionB, "conv3 partial sums must fit the conv1 region");

// conv2 of stage 3 for the NT position tiles wslot, wslot + 4, ... of one crop.
template <int NT, int ACT>
__device__ __forceinline__ void s3_conv2(const float *sP1, float *sP2, const float *__restrict__ B2F, int wslot,
                                         int lane, float bias_lo, float bias_hi)
{
    const int i = lane & 15, g = lane >> 4;
    floatx4 acc[NT][2];
    int abase[NT];
#pragma unroll
    for (int u = 0; u < NT; ++u) {
        acc[u][0] = floatx4{0, 0, 0, 0};
        acc[u][1] = floatx4{0, 0, 0, 0};
        const int pb = min(4 * (wslot + 4 * u) + (i >> 2), 80);       // pooling block of this lane's position
        const int y = 2 * (pb / 9) + ((i >> 1) & 1), x = 2 * (pb % 9) + (i & 1);
        abase[u] = g * kP1Ch + y * kP1Row + x;
    }
    const float4 *bp = reinterpret_cast<const float4 *>(B2F) + lane;   // [tap][n-tile][lane] float4 (4 channel quads)
    float4 bc0 = bp[0], bc1 = bp[64];
#pragma unroll 1
    for (int tap = 0; tap < 25; ++tap) {
        const int tn = min(tap + 1, 24);
        const float4 bn0 = bp[tn * 128], bn1 = bp[tn * 128 + 64];      // next tap's weights, in flight during the math
        asm volatile("" ::: "memory");                                 // keeps the loads here: they must not sink to their use
        const int toff = (tap / 5) * kP1Row + tap % 5;
        const float b0[4] = {bc0.x, bc0.y, bc0.z, bc0.w}, b1[4] = {bc1.x, bc1.y, bc1.z, bc1.w};
#pragma unroll
        for (int cq = 0; cq < 4; ++cq)
#pragma unroll
            for (int u = 0; u < NT; ++u) {
                const float a = sP1[abase[u] + toff + cq * 4 * kP1Ch];
                acc[u][0] = CNNC_MFMA(a, b0[cq], acc[u][0]);
                acc[u][1] = CNNC_MFMA(a, b1[cq], acc[u][1]);
            }
        bc0 = bn0; bc1 = bn1;
    }
    const int j = lane & 15;
#pragma unroll
    for (int u = 0; u < NT; ++u) {
        const int pb = 4 * (wslot + 4 * u) + g;
        if (pb < 81) {
            sP2[p2_index<0>(j, pb)] = act_f<ACT>(max4(acc[u][0]) + bias_lo);
            sP2[p2_index<0>(16 + j, pb)] = act_f<ACT>(max4(acc[u][1]) + bias_hi);
        }
    }
}

// ---- conv2 of stage 3 by the Winograd minimal-filtering algorithm F(2, 5) along the rows ---------------
// Two horizontally adjacent outputs of a 5-tap row filter cost 6 multiplications instead of 10:
//   out(x0 + q) = sum_b AT[q][b] * (sum_l G[b][l] w[l]) * (sum_p BT[b][p] d[x0 + p]),   q = 0, 1, x0 even.
// For the 5x5, 16 -> 32 convolution this gives six GEMMs (one per b) with M = 162 positions (18 rows x 9
// column pairs), K = 16 channels x 5 kernel rows = 80 and N = 32, i.e. 60 % of the matrix work of the direct
// sum.  The lane that feeds the A operand reads six consecutive floats of one input row and transforms them
// in registers; the filter side U = G w is prepared on the host in fp64.  Interpolation points 0, 1, -1, 2, -2 and
// infinity: BT then pairs up into even and odd parts (twelve operations per six-vector),
//   BT = [4 0 -5 0 1 0; 0 -4 -4 1 1 0; 0 4 -4 -1 1 0; 0 -2 -1 2 1 0; 0 2 -1 -2 1 0; 0 4 0 -5 0 1],
//   AT = [1 1 1 1 1 0; 0 1 -1 2 -2 1],
// and the fp32 result stays within about 2e-6 of the direct fp32 sum here.
// Positions are ordered so that the four accumulator registers of a lane hold two pooling blocks
// (block, line) = (2 g + r / 2, r % 2) of the M-tile, and the output transform leaves both columns of a
// line in the same lane: max-pooling stays in registers.
constexpr int kWinoTiles = 11;          // 81 pooling blocks, eight per M-tile

// One M-tile per pass over the filter.  (Two tiles per pass would halve the filter's L2 -> register traffic,
// but the 96 accumulator registers spill: measured slower.)  The loop is software-pipelined by hand: the filter
// fragments are fetched two k-steps ahead and the input row one step ahead, and the compiler is kept from
// sinking those loads to their uses.
template <int NT, int ACT>
__device__ __forceinline__ void s3_conv2_wino_tiles(const float *sP1, float *sP2, const float *__restrict__ UF, int mt0,
                                                    int lane, float bias_lo, float bias_hi)
{
    static_assert(NT == 1, "one M-tile per pass");
    const int i = lane & 15, g = lane >> 4, j = lane & 15;
    const float *dptr[NT];
    floatx4 acc[NT][6][2];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int pb = min(8 * (mt0 + 4 * t) + (i >> 1), 80);    // this lane's A rows: pooling block and line i % 2
        dptr[t] = sP1 + g * kP1Ch + (2 * (pb / 9) + (i & 1)) * kP1Row + 2 * (pb % 9);
#pragma unroll
        for (int b = 0; b < 6; ++b) { acc[t][b][0] = floatx4{0, 0, 0, 0}; acc[t][b][1] = floatx4{0, 0, 0, 0}; }
    }
    // filter fragments [k-step][lane] three float4: uniform base + 32-bit lane offset, so the address math is scalar
    const char *ubase = reinterpret_cast<const char *>(UF);
    const uint32_t lane_off = lane * 48;
    auto ldu = [&](int step, int k) {
        return *reinterpret_cast<const float4 *>(ubase + (size_t)(step * 3072 + k * 16) + lane_off);
    };
    float4 u0 = ldu(0, 0), u1 = ldu(0, 1), u2 = ldu(0, 2);                     // step s
    float4 v0 = ldu(1, 0), v1 = ldu(1, 1), v2 = ldu(1, 2);                     // step s + 1
    float2 c0 = *reinterpret_cast<const float2 *>(dptr[0]), c1 = *reinterpret_cast<const float2 *>(dptr[0] + 2),
           c2 = *reinterpret_cast<const float2 *>(dptr[0] + 4);
#pragma unroll 1
    for (int a = 0; a < 5; ++a) {                                // kernel row
#pragma unroll
        for (int cq = 0; cq < 4; ++cq) {                         // input channels 4 cq + g
            const int nstep = min(a * 4 + cq + 2, 19);
            const float4 n0 = ldu(nstep, 0), n1 = ldu(nstep, 1), n2 = ldu(nstep, 2);
            // input row of the next step (the last step reads its own row again)
            const float *nrow = dptr[0] + (cq == 3 ? min(a + 1, 4) * kP1Row + (a == 4 ? 3 : 0) * 4 * kP1Ch
                                                   : a * kP1Row + (cq + 1) * 4 * kP1Ch);
            const float2 m0 = *reinterpret_cast<const float2 *>(nrow), m1 = *reinterpret_cast<const float2 *>(nrow + 2),
                         m2 = *reinterpret_cast<const float2 *>(nrow + 4);
            asm volatile("" ::: "memory");                        // the loads above stay in flight during the math below
            const float ub[12] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w, u2.x, u2.y, u2.z, u2.w};
            // transformed input BT d
            const float e1 = fmaf(-4.0f, c1.x, c2.x), o1 = fmaf(-4.0f, c0.y, c1.y);
            const float e2 = c2.x - c1.x, o2 = c1.y - c0.y;
            const float v[6] = {fmaf(4.0f, c0.x, fmaf(-5.0f, c1.x, c2.x)), e1 + o1, e1 - o1, fmaf(2.0f, o2, e2), fmaf(-2.0f, o2, e2),
                                fmaf(4.0f, c0.y, fmaf(-5.0f, c1.y, c2.y))};
#pragma unroll
            for (int b = 0; b < 6; ++b) {
                acc[0][b][0] = CNNC_MFMA(v[b], ub[2 * b], acc[0][b][0]);
                acc[0][b][1] = CNNC_MFMA(v[b], ub[2 * b + 1], acc[0][b][1]);
            }
            u0 = v0; u1 = v1; u2 = v2;
            v0 = n0; v1 = n1; v2 = n2;
            c0 = m0; c1 = m1; c2 = m2;
        }
    }
    // output transform AT m, pooling, bias, activation
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const floatx4 R0 = acc[t][0][nt] + (acc[t][1][nt] + acc[t][2][nt]) + (acc[t][3][nt] + acc[t][4][nt]);
            const floatx4 R1 = (acc[t][1][nt] - acc[t][2][nt]) + 2.0f * (acc[t][3][nt] - acc[t][4][nt]) + acc[t][5][nt];
            const float bias = nt ? bias_hi : bias_lo;
            const int oc = 16 * nt + j;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const int blk = 8 * (mt0 + 4 * t) + 2 * g + sub;
                const float m = fmaxf(fmaxf(R0[2 * sub], R1[2 * sub]), fmaxf(R0[2 * sub + 1], R1[2 * sub + 1]));
                if (blk < 81) sP2[p2_index<1>(oc, blk)] = act_f<ACT>(m + bias);
            }
        }
}

// ---- conv2 of stage 3 by Winograd F(4, 5) along the rows: four adjacent outputs of a 5-tap row filter cost 8
// multiplications instead of 20 (F(2, 5) above: 12), points 0, 1, -1, 2, -2, 1/2, -1/2 and infinity:
//   BT = [-1 0 21/4 0 -21/4 0 1 0; 0 1 1 -17/4 -17/4 1 1 0; 0 -1 1 17/4 -17/4 -1 1 0; 0 1/2 1/4 -5/2 -5/4 2 1 0;
//         0 -1/2 1/4 5/2 -5/4 -2 1 0; 0 2 4 -5/2 -5 1/2 1 0; 0 -2 4 5/2 -5 -1/2 1 0; 0 -1 0 21/4 0 -21/4 0 1],
//   AT = [1 1 1 1 1 1 1 0; 0 1 -1 2 -2 1/2 -1/2 0; 0 1 1 4 4 1/4 1/4 0; 0 1 -1 8 -8 1/8 -1/8 1],
// both in even / odd pairs (26 operations per eight-vector); the fp32 result stays within about 2e-6 of the direct
// fp32 sum here, as for F(2, 5).  Eight GEMMs with M = 90 rows (18 output rows x 5 groups of four columns, the last
// group half empty), K = 80, N = 32: 1920 matrix instructions against 2640.
// A unit is one pooling-block row pair Y and one column group xg: 45 units, eight per M-tile, two A rows each (the two
// output rows of the pair).  A lane's four accumulator registers hold two units x two rows, and the output transform
// leaves four columns = two pooling blocks per row in the lane, so max-pooling stays in registers.
// Reads columns 22, 23 of the pooled conv1 map for its half-empty group: the kernel clears them once.

// NTN = 2: the tile for all 32 output channels.  NTN = 1: for the sixteen channels of n-tile nt0 only (half the
// matrix work with the same input transform).  The six tiles are dealt as one whole tile per wave (tiles 0..3) plus
// one half of tile 4 or 5 per wave, so the four waves carry equal loads.
template <int ACT, int NTN>
__device__ __forceinline__ void s3_conv2_wino4_tile(const float *sP1, float *sP2, const float *__restrict__ UF, int mt, int nt0,
                                                    int lane, const float *__restrict__ bias2)
{
    const int i = lane & 15, g = lane >> 4, j = lane & 15;
    const int unit = min(8 * mt + (i >> 1), 44);
    const float *dptr = sP1 + g * kP1Ch + (2 * (unit / 5) + (i & 1)) * kP1Row + 4 * (unit % 5);
    floatx4 acc[8][NTN];
#pragma unroll
    for (int b = 0; b < 8; ++b)
#pragma unroll
        for (int t = 0; t < NTN; ++t) acc[b][t] = floatx4{0, 0, 0, 0};
    // filter fragments [k-step][lane][n-tile][8 points]: a wave-uniform pointer per k-step (kept in scalar registers:
    // the empty asm stops the compiler from folding it into a per-lane 64-bit address) + 32-bit lane offset
    const char *ubase = reinterpret_cast<const char *>(UF);
    const uint32_t lane_off = lane * 64 + (NTN == 1 ? nt0 * 32 : 0);
    auto step_ptr = [&](int step) {
        const char *sp = ubase + step * 4096;
        asm volatile("" : "+s"(sp));
        return sp;
    };
    // (the pointer comes out of the asm without its address space: say again that it is global memory)
    typedef const __attribute__((address_space(1))) floatx4 *global_x4_ptr;
    auto ldu = [&](const char *sp, int k) {
        const floatx4 v = *(global_x4_ptr)(sp + lane_off + k * 16);
        return make_float4(v[0], v[1], v[2], v[3]);
    };
    float4 u[2 * NTN], n[2 * NTN];
    {
        const char *sp = step_ptr(0);
#pragma unroll
        for (int k = 0; k < 2 * NTN; ++k) u[k] = ldu(sp, k);
    }
    float4 c0 = *reinterpret_cast<const float4 *>(dptr), c1 = *reinterpret_cast<const float4 *>(dptr + 4);
#pragma unroll 1
    for (int a = 0; a < 5; ++a) {                                // kernel row
#pragma unroll
        for (int cq = 0; cq < 4; ++cq) {                         // input channels 4 cq + g
            const char *np = step_ptr(min(a * 4 + cq + 1, 19));
#pragma unroll
            for (int k = 0; k < 2 * NTN; ++k) n[k] = ldu(np, k);
            const float *nrow = dptr + (cq == 3 ? min(a + 1, 4) * kP1Row + (a == 4 ? 3 : 0) * 4 * kP1Ch
                                                : a * kP1Row + (cq + 1) * 4 * kP1Ch);
            const float4 m0 = *reinterpret_cast<const float4 *>(nrow), m1 = *reinterpret_cast<const float4 *>(nrow + 4);
            asm volatile("" ::: "memory");                        // the loads above stay in flight during the math below
            // transformed input BT d, d = (c0.x .. c1.w)
            const float e1 = fmaf(-4.25f, c1.x, c0.z) + c1.z, o1 = fmaf(-4.25f, c0.w, c0.y) + c1.y;
            const float e2 = fmaf(-1.25f, c1.x, fmaf(0.25f, c0.z, c1.z)), o2 = fmaf(2.0f, c1.y, fmaf(-2.5f, c0.w, 0.5f * c0.y));
            const float e3 = fmaf(-5.0f, c1.x, fmaf(4.0f, c0.z, c1.z)), o3 = fmaf(0.5f, c1.y, fmaf(-2.5f, c0.w, 2.0f * c0.y));
            const float v[8] = {fmaf(5.25f, c0.z - c1.x, c1.z - c0.x), e1 + o1, e1 - o1, e2 + o2, e2 - o2, e3 + o3, e3 - o3,
                                fmaf(5.25f, c0.w - c1.y, c1.w - c0.y)};
#pragma unroll
            for (int t = 0; t < NTN; ++t) {
                const float ub[8] = {u[2 * t].x, u[2 * t].y, u[2 * t].z, u[2 * t].w, u[2 * t + 1].x, u[2 * t + 1].y, u[2 * t + 1].z, u[2 * t + 1].w};
#pragma unroll
                for (int b = 0; b < 8; ++b) acc[b][t] = CNNC_MFMA(v[b], ub[b], acc[b][t]);
            }
#pragma unroll
            for (int k = 0; k < 2 * NTN; ++k) u[k] = n[k];
            c0 = m0; c1 = m1;
        }
    }
    // output transform AT m (four columns per row), pooling over the two rows and the two column pairs, bias, activation
#pragma unroll
    for (int t = 0; t < NTN; ++t) {
        const floatx4 s1 = acc[1][t] + acc[2][t], d1 = acc[1][t] - acc[2][t];
        const floatx4 s2 = acc[3][t] + acc[4][t], d2 = acc[3][t] - acc[4][t];
        const floatx4 s3 = acc[5][t] + acc[6][t], d3 = acc[5][t] - acc[6][t];
        const floatx4 Y0 = acc[0][t] + s1 + (s2 + s3);
        const floatx4 Y1 = d1 + 2.0f * d2 + 0.5f * d3;
        const floatx4 Y2 = s1 + 4.0f * s2 + 0.25f * s3;
        const floatx4 Y3 = d1 + 8.0f * d2 + 0.125f * d3 + acc[7][t];
        const int oc = 16 * (NTN == 1 ? nt0 : t) + j;
        const float bias = bias2[oc];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {                      // registers 2 sub, 2 sub + 1 = the two rows of unit 2 g + sub
            const int q = 8 * mt + 2 * g + sub;
            if (q < 45) {
                const int Y = q / 5, xg = q % 5;
                const float left = fmaxf(fmaxf(Y0[2 * sub], Y1[2 * sub]), fmaxf(Y0[2 * sub + 1], Y1[2 * sub + 1]));
                sP2[p2_index<1>(oc, Y * 9 + 2 * xg)] = act_f<ACT>(left + bias);
                if (xg < 4) {
                    const float right = fmaxf(fmaxf(Y2[2 * sub], Y3[2 * sub]), fmaxf(Y2[2 * sub + 1], Y3[2 * sub + 1]));
                    sP2[p2_index<1>(oc, Y * 9 + 2 * xg + 1)] = act_f<ACT>(right + bias);
                }
            }
        }
    }
}

// ---- conv3 of stage 3, direct sums: 49 positions = 4 tiles.  The waves split K (wave w takes input channels
// 8w .. 8w+7 of every tap), so each needs only a quarter of the weights, all loaded up front; the partial tiles
// go to LDS as [wave][channel 32][kP3Pitch] and are summed by s3_conv3_direct_finish after a barrier.
__device__ __forceinline__ void s3_conv3_direct(const float *sP2, float *sPart, const float *__restrict__ B3F, int wave, int lane)
{
    const int g = lane >> 4, j = lane & 15;
    float2 b3[9][2];
    const float2 *bp = reinterpret_cast<const float2 *>(B3F) + lane * 4 + wave;   // [tap][n-tile][lane][8]
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
        b3[tap][0] = bp[(tap * 2) * 256];
        b3[tap][1] = bp[(tap * 2 + 1) * 256];
    }
    floatx4 acc[4][2];
    int abase[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        acc[u][0] = floatx4{0, 0, 0, 0};
        acc[u][1] = floatx4{0, 0, 0, 0};
        const int pos = min(16 * u + j, 48);
        abase[u] = (8 * wave + g) * kP2Ch + (pos / 7) * 9 + pos % 7;
    }
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float w0 = h ? b3[tap][0].y : b3[tap][0].x, w1 = h ? b3[tap][1].y : b3[tap][1].x;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float a = sP2[abase[u] + (tap / 3) * 9 + tap % 3 + h * 4 * kP2Ch];
                acc[u][0] = CNNC_MFMA(a, w0, acc[u][0]);
                acc[u][1] = CNNC_MFMA(a, w1, acc[u][1]);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int p = 16 * u + 4 * g + r;
            sPart[(wave * 32 + j) * kP3Pitch + p] = acc[u][0][r];
            sPart[(wave * 32 + 16 + j) * kP3Pitch + p] = acc[u][1][r];
        }
}

template <int ACT>
__device__ __forceinline__ void s3_conv3_direct_finish(const float *sPart, const float *__restrict__ wt, float *__restrict__ dst)
{
    for (int e = threadIdx.x; e < 1568; e += kThreads) {
        const int oc = e / 49, p = e % 49;
        const float v = sPart[oc * kP3Pitch + p] + sPart[(32 + oc) * kP3Pitch + p] + sPart[(64 + oc) * kP3Pitch + p] +
                        sPart[(96 + oc) * kP3Pitch + p];
        dst[e] = act_f<ACT>(v + wt[s3::B3 + oc]);
    }
}

// ---- conv3 of stage 3 by Winograd F(2, 3) along the rows: two adjacent outputs of a 3-tap row filter cost four
// multiplications instead of six (points 0, 1, -1, infinity):
//   m0 = (d0 - d2) g0, m1 = (d1 + d2)(g0 + g1 + g2)/2, m2 = (d2 - d1)(g0 - g1 + g2)/2, m3 = (d1 - d3) g2,
//   out(x0) = m0 + m1 + m2, out(x0 + 1) = m1 - m2 - m3.
// Four GEMMs with M = 28 positions (7 rows x 4 column pairs; the 8th column is discarded), K = 32 channels x 3
// kernel rows, N = 32: wave w takes M-tile w / 2 and output channels 16 (w % 2) .. +15, so nothing has to be
// summed across waves and the activations go straight to global memory (order [channel][row][col]).
template <int ACT>
__device__ __forceinline__ void s3_conv3_wino(const float *sP2, const float *__restrict__ U3F, const float *__restrict__ wt,
                                              float *__restrict__ dst, int wave, int lane)
{
    const int mtile = wave >> 1, nt = wave & 1;
    const int i = lane & 15, g = lane >> 4, j = lane & 15;
    const int p = min(16 * mtile + i, 27);
    const float *dptr = sP2 + g * kP2ChW + (p >> 2) * kP2RowW + 2 * (p & 3);
    floatx4 acc[4] = {floatx4{0, 0, 0, 0}, floatx4{0, 0, 0, 0}, floatx4{0, 0, 0, 0}, floatx4{0, 0, 0, 0}};
    const float4 *up = reinterpret_cast<const float4 *>(U3F) + nt * 24 * 64 + lane;   // [n-tile][k-step][lane] four points
    // filter fragments run eight k-steps ahead: a step is only four matrix instructions long, and the loads come from L2
    float4 ring[8] = {up[0], up[64], up[128], up[192], up[256], up[320], up[384], up[448]};
    up += 512;
    float2 r0 = *reinterpret_cast<const float2 *>(dptr), r1 = *reinterpret_cast<const float2 *>(dptr + 2);
#pragma unroll
    for (int ks = 0; ks < 24; ++ks) {                            // k-step = kernel row a (3) x channel quad cq (8)
        const float4 u = ring[ks & 7];
        if (ks + 8 < 24) {
            ring[ks & 7] = *up;
            up += 64;
            asm volatile("" : "+v"(up));                          // one running address instead of twenty precomputed ones
        }
        const int kn = ks + 1 < 24 ? ks + 1 : ks;                 // input row of the next step, fetched one step ahead
        const float *nrow = dptr + (kn & 7) * 4 * kP2ChW + (kn >> 3) * kP2RowW;
        const float2 n0 = *reinterpret_cast<const float2 *>(nrow), n1 = *reinterpret_cast<const float2 *>(nrow + 2);
        asm volatile("" ::: "memory");                            // keeps the prefetch distance: loads stay where written
        acc[0] = CNNC_MFMA(r0.x - r1.x, u.x, acc[0]);
        acc[1] = CNNC_MFMA(r0.y + r1.x, u.y, acc[1]);
        acc[2] = CNNC_MFMA(r1.x - r0.y, u.z, acc[2]);
        acc[3] = CNNC_MFMA(r0.y - r1.y, u.w, acc[3]);
        r0 = n0; r1 = n1;
    }
    const int oc = 16 * nt + j;
    const float bias = wt[s3::B3 + oc];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int pp = 16 * mtile + 4 * g + r;                    // row pp / 4, column pair r
        if (pp < 28) {
            float *o = dst + oc * 49 + (pp >> 2) * 7 + 2 * r;
            o[0] = act_f<ACT>(acc[0][r] + acc[1][r] + acc[2][r] + bias);
            if (r < 3) o[1] = act_f<ACT>(acc[1][r] - acc[2][r] - acc[3][r] + bias);
        }
    }
}
}  // namespace

// Fragment buffer of stage 3 (floats): conv1 [7][64], conv2 [25][2][64][4], conv3 [9][2][64][8], fc [98][4][64][4].
// plus the Winograd-domain conv2 weights [5 kernel rows][4 channel quads][64][6 points x 2 n-tiles]
// and conv3 weights [2 n-tiles][3 kernel rows x 8 channel quads][64][4 points], and the F(4,5) conv2 weights
// [5 kernel rows][4 channel quads][64][2 n-tiles][8 points].
constexpr int kS3F1 = 0, kS3F2 = kS3F1 + 7 * 64, kS3F3 = kS3F2 + 25 * 2 * 64 * 4, kS3F4 = kS3F3 + 9 * 2 * 64 * 8,
              kS3F5 = kS3F4 + 98 * 4 * 64 * 4, kS3F6 = kS3F5 + 20 * 64 * 12, kS3F7 = kS3F6 + 2 * 24 * 64 * 4, kS3FragFloats = kS3F7 + 20 * 64 * 16;
static_assert(kS3F5 % 4 == 0 && kS3F6 % 4 == 0 && kS3F7 % 4 == 0, "16-byte loads from the Winograd filter blocks");
constexpr int kS3Feat = 1568;
// The conv3 activations go from the convolution kernel to the fully connected kernel through a buffer of this many
// windows; a longer survivor list is worked off in segments of that length, one pair of launches each.
constexpr int kS3Segment = 65536;

// Crop -> conv1 -> pool -> conv2 -> pool -> conv3 for each surviving window; writes the 1568 conv3
// activations of the window (order [channel][row][col]) to `feat`.
template <int ACT, int WINO>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3, 3)))
void eval3_conv_kernel(const uint8_t *__restrict__ frame, int fw, int fh, int pitch, const LevelDev *__restrict__ levels,
                       int n_levels, const uint32_t *__restrict__ idx, const int32_t *__restrict__ d_begin,
                       const int32_t *__restrict__ d_n, int seg_lo, int n_max, const float *__restrict__ wt,
                       const float *__restrict__ frag, float *__restrict__ feat)
{
    __shared__ __attribute__((aligned(16))) float sA[kRegionA];
    __shared__ __attribute__((aligned(16))) float sB[kRegionB];
    __shared__ uint32_t sTab[2 * kS3In];
    __shared__ uint32_t sLut[484];          // per pooling block of conv1: crop offset of its corner | pooled-map offset << 16
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, g = lane >> 4, j = lane & 15;
    for (int pb = tid; pb < 484; pb += kThreads)
        sLut[pb] = (uint32_t)(2 * (pb / 22) * kCropW + 2 * (pb % 22)) | (uint32_t)((pb / 22) * kP1Row + pb % 22) << 16;
    if (WINO == 2)                                                   // columns 22, 23 of the pooled conv1 map: read, never written
        for (int e = tid; e < 16 * 22 * 2; e += kThreads) sB[(e >> 1) * kP1Row + 22 + (e & 1)] = 0.0f;
    const int in_lane = ((j >> 1) & 1) * kCropW + (j & 1) + g;     // A rows: line and column of the block, plus the tap column g
    // (the first barrier of the gather below orders the table before its readers)

    // conv1 k-order: steps 0..4 = taps (a = step, b = g); step 5 = taps (a = g, b = 4);
    // step 6 = tap (4, 4) in group 0, zero weights elsewhere (those lanes re-read their own pixel)
    const int off5 = g * kCropW + 4 - g, off6 = g == 0 ? 4 * kCropW + 4 : -g;     // relative to a base that includes + g

    const int n = min(*d_n, n_max);
    int rot = 0;
    // Static striding over the list.  (Handing windows out through an atomic ticket counter was measured:
    // it does not shorten the kernel, the device-scope atomics cost more than the balance gains.)
    // The gather of a window is software-pipelined: its tables are computed during conv1 of the previous
    // window, its pixel loads are in flight during conv3, and it lands in LDS once conv3 has released the buffer.
    int crop = max(min(*d_begin, n_max), seg_lo) + blockIdx.x;      // the launch covers list entries seg_lo .. n_max - 1 of the range
    if (crop < n) {
        const Survivor sv = decode(idx[crop], levels, n_levels);
        gather_crop<kS3In>(frame, fw, fh, pitch, sv.x, sv.y, levels[sv.level].scale_q16, sTab, sA);
    }
    for (; crop < n; crop += gridDim.x, ++rot) {
        const int next = crop + gridDim.x;

        // ---- conv1 5x5 1->16 + pool: 121 tiles of four pooling blocks, four tiles in flight per wave
        // (small per-layer constants are re-read per window instead of living in registers through the other layers)
        float b1f[7];
#pragma unroll
        for (int s = 0; s < 7; ++s) b1f[s] = frag[kS3F1 + s * 64 + lane];
        const float bias1 = wt[s3::B1 + j];
#pragma unroll 1
        for (int q0 = 0; q0 < 32; q0 += 4) {
            floatx4 acc[4];
            int base[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                acc[u] = floatx4{0, 0, 0, 0};
                const int t = min(wave + 4 * (q0 + u), 120);
                base[u] = (int)(sLut[4 * t + (j >> 2)] & 0xFFFFu) + in_lane;
            }
#pragma unroll
            for (int s = 0; s < 5; ++s)
#pragma unroll
                for (int u = 0; u < 4; ++u) acc[u] = CNNC_MFMA(sA[base[u] + s * kCropW], b1f[s], acc[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] = CNNC_MFMA(sA[base[u] + off5], b1f[5], acc[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] = CNNC_MFMA(sA[base[u] + off6], b1f[6], acc[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int t = wave + 4 * (q0 + u);
                if (t < 121) sB[j * kP1Ch + (sLut[4 * t + g] >> 16)] = act_f<ACT>(max4(acc[u]) + bias1);
            }
        }
        if (next < n) {          // sample tables of the next window; the table buffer is idle until conv3
            const Survivor sv = decode(idx[next], levels, n_levels);
            crop_tables<kS3In>(sv.x, sv.y, levels[sv.level].scale_q16, fw, fh, sTab);
        }
        __syncthreads();

        // ---- conv2 5x5 16->32 + pool (overwrites the crop with the pooled map)
        const int wslot = (wave + rot + blockIdx.x + (blockIdx.x >> 8)) & 3;
        const float bias2_lo = wt[s3::B2 + j], bias2_hi = wt[s3::B2 + 16 + j];
        if (WINO == 2) {
            // six M-tiles of eight units: a whole tile per wave, then half (one n-tile) of tile 4 or 5 per wave
            s3_conv2_wino4_tile<ACT, 2>(sB, sA, frag + kS3F7, wslot, 0, lane, wt + s3::B2);
            s3_conv2_wino4_tile<ACT, 1>(sB, sA, frag + kS3F7, 4 + (wslot >> 1), wslot & 1, lane, wt + s3::B2);
        } else if (WINO == 1) {
            // eleven M-tiles of eight pooling blocks, dealt round-robin from a slot that rotates per window.
            // (Two tiles per pass over the filter halve its L2 traffic but spill registers: measured slower.)
#pragma unroll 1
            for (int mt = wslot; mt < kWinoTiles; mt += 4)
                s3_conv2_wino_tiles<1, ACT>(sB, sA, frag + kS3F5, mt, lane, bias2_lo, bias2_hi);
        } else if (wslot == 0) {
            // 21 tiles of four pooling blocks; the wave that takes six of them rotates per window
            s3_conv2<6, ACT>(sB, sA, frag + kS3F2, wslot, lane, bias2_lo, bias2_hi);
        } else {
            s3_conv2<5, ACT>(sB, sA, frag + kS3F2, wslot, lane, bias2_lo, bias2_hi);
        }
        __syncthreads();

        // ---- pixel loads of the next window go out now and stay in flight during conv3
        CropPixels<kS3In> px;
        if (next < n) crop_issue<kS3In>(frame, pitch, sTab, px);

        // ---- conv3 3x3 32->32 and out to global memory
        float *dst = feat + (size_t)(crop - seg_lo) * kS3Feat;
        if (WINO) s3_conv3_wino<ACT>(sA, frag + kS3F6, wt, dst, wave, fresh(lane));
        else s3_conv3_direct(sA, sB, frag + kS3F3, wave, lane);
        __syncthreads();                                   // conv3 has released the pooled map (and, direct form, written its partial sums)
        if (!WINO) s3_conv3_direct_finish<ACT>(sB, wt, dst);
        if (next < n) crop_finish<kS3In>(px, sTab, sA);
        __syncthreads();                                   // next crop in place; partial sums consumed before conv1 rewrites sB
    }
}

// fc 1568->64 + f, fc 64->1 for 16 windows per workgroup: eight waves split K (the loop is bound by the latency of its
// loads, so more waves with their own loads in flight shorten it), partial tiles meet in LDS.
constexpr int kFcThreads = 512, kFcWaves = kFcThreads / 64;
template <int ACT>
__global__ __launch_bounds__(kFcThreads)
void eval3_fc_kernel(const float *__restrict__ feat, const int32_t *__restrict__ d_begin, const int32_t *__restrict__ d_n, int seg_lo, int n_max,
                     const float *__restrict__ wt, const float *__restrict__ frag, float *__restrict__ out)
{
    __shared__ float sPart[kFcWaves][16][65];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 4, j = lane & 15;
    const int n = min(*d_n, n_max);
    const float4 *wf = reinterpret_cast<const float4 *>(frag + kS3F4) + lane;     // [chunk][n-tile][lane] float4
    const int first = max(min(*d_begin, n_max), seg_lo);   // tiles of sixteen windows are counted from the range's first one
    for (int tile = blockIdx.x; first + tile * 16 < n; tile += gridDim.x) {
        const int row = min(first + tile * 16 + j, n - 1);
        const float4 *ap = reinterpret_cast<const float4 *>(feat + (size_t)(row - seg_lo) * kS3Feat) + g;
        floatx4 acc[4] = {floatx4{0, 0, 0, 0}, floatx4{0, 0, 0, 0}, floatx4{0, 0, 0, 0}, floatx4{0, 0, 0, 0}};
        for (int ch = wave; ch < 98; ch += kFcWaves) {
            const float4 a4 = ap[ch * 4];
            const float a[4] = {a4.x, a4.y, a4.z, a4.w};
            float4 b4[4];
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) b4[nt] = wf[(ch * 4 + nt) * 64];
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    const float b = s == 0 ? b4[nt].x : s == 1 ? b4[nt].y : s == 2 ? b4[nt].z : b4[nt].w;
                    acc[nt] = CNNC_MFMA(a[s], b, acc[nt]);
                }
        }
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) sPart[wave][4 * g + r][nt * 16 + j] = acc[nt][r];
        __syncthreads();
        if (tid < 256) {
            const int r = tid >> 4, c0 = tid & 15;
            float part = 0.0f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = c0 + 16 * q;
                float h = wt[s3::B4 + c];
#pragma unroll
                for (int w = 0; w < kFcWaves; ++w) h += sPart[w][r][c];
                part = fmaf(wt[s3::W5 + c], act_f<ACT>(h), part);
            }
#pragma unroll
            for (int d = 8; d >= 1; d >>= 1) part += __shfl_xor(part, d, 64);
            if (c0 == 0 && first + tile * 16 + r < n) out[first + tile * 16 + r] = part + wt[s3::B5];
        }
        __syncthreads();
    }
}

// ---- host: weight fragments ---------------------------------------------------------------------
size_t eval3_frag_floats() { return kS3FragFloats; }
size_t eval3_feat_floats() { return kS3Feat; }
int eval3_feat_rows(int max_surv) { return max_surv < kS3Segment ? max_surv : kS3Segment; }

// Re-order the stage-3 weights (blob layout: [cout][cin][k][k] per layer) into MFMA B fragments.
void eval3_make_fragments(const float *w, float *f)
{
    for (int s = 0; s < 7; ++s)
        for (int lane = 0; lane < 64; ++lane) {
            const int g = lane >> 4, j = lane & 15;
            int a = -1, b = -1;
            if (s < 5) { a = s; b = g; }
            else if (s == 5) { a = g; b = 4; }
            else if (g == 0) { a = 4; b = 4; }
            f[kS3F1 + s * 64 + lane] = a < 0 ? 0.0f : w[s3::W1 + (j * 5 + a) * 5 + b];
        }
    for (int tap = 0; tap < 25; ++tap)
        for (int nt = 0; nt < 2; ++nt)
            for (int lane = 0; lane < 64; ++lane)
                for (int cq = 0; cq < 4; ++cq) {
                    const int g = lane >> 4, j = lane & 15, oc = nt * 16 + j, c = 4 * cq + g;
                    f[kS3F2 + ((tap * 2 + nt) * 64 + lane) * 4 + cq] = w[s3::W2 + (oc * 16 + c) * 25 + tap];
                }
    for (int tap = 0; tap < 9; ++tap)
        for (int nt = 0; nt < 2; ++nt)
            for (int lane = 0; lane < 64; ++lane)
                for (int cq = 0; cq < 8; ++cq) {
                    const int g = lane >> 4, j = lane & 15, oc = nt * 16 + j, c = 4 * cq + g;
                    f[kS3F3 + ((tap * 2 + nt) * 64 + lane) * 8 + cq] = w[s3::W3 + (oc * 32 + c) * 9 + tap];
                }
    for (int ch = 0; ch < 98; ++ch)
        for (int nt = 0; nt < 4; ++nt)
            for (int lane = 0; lane < 64; ++lane)
                for (int s = 0; s < 4; ++s) {
                    const int g = lane >> 4, j = lane & 15;
                    f[kS3F4 + ((ch * 4 + nt) * 64 + lane) * 4 + s] = w[s3::W4 + (nt * 16 + j) * 1568 + 16 * ch + 4 * g + s];
                }
    // Winograd-domain conv2 weights U_b = sum_l G[b][l] w[.][.][a][l] (fp64, then rounded); G for the points
    // 0, 1, -1, 2, -2, infinity: row j = (a_j^l / prod_{i != j} (a_j - a_i)), last row picks the leading tap
    static const double G[6][5] = {{1.0 / 4, 0, 0, 0, 0},
                                   {-1.0 / 6, -1.0 / 6, -1.0 / 6, -1.0 / 6, -1.0 / 6},
                                   {-1.0 / 6, 1.0 / 6, -1.0 / 6, 1.0 / 6, -1.0 / 6},
                                   {1.0 / 24, 1.0 / 12, 1.0 / 6, 1.0 / 3, 2.0 / 3},
                                   {1.0 / 24, -1.0 / 12, 1.0 / 6, -1.0 / 3, 2.0 / 3},
                                   {0, 0, 0, 0, 1}};
    for (int oc = 0; oc < 32; ++oc)
        for (int c = 0; c < 16; ++c)
            for (int a = 0; a < 5; ++a) {
                const float *k = w + s3::W2 + ((oc * 16 + c) * 5 + a) * 5;
                const int cq = c >> 2, g = c & 3, nt = oc >> 4, j = oc & 15, lane = g * 16 + j;
                for (int b = 0; b < 6; ++b) {
                    double acc = 0;
                    for (int l = 0; l < 5; ++l) acc += G[b][l] * (double)k[l];
                    f[kS3F5 + ((a * 4 + cq) * 64 + lane) * 12 + b * 2 + nt] = (float)acc;
                }
            }
    // Winograd-domain conv3 weights along the kernel columns: g0, (g0 + g1 + g2) / 2, (g0 - g1 + g2) / 2, g2
    for (int oc = 0; oc < 32; ++oc)
        for (int c = 0; c < 32; ++c)
            for (int a = 0; a < 3; ++a) {
                const float *k = w + s3::W3 + ((oc * 32 + c) * 3 + a) * 3;
                const double g0 = k[0], g1 = k[1], g2 = k[2];
                const double u[4] = {g0, (g0 + g1 + g2) / 2, (g0 - g1 + g2) / 2, g2};
                const int cq = c >> 2, g = c & 3, nt = oc >> 4, j = oc & 15, lane = g * 16 + j, ks = a * 8 + cq;
                for (int b = 0; b < 4; ++b) f[kS3F6 + ((nt * 24 + ks) * 64 + lane) * 4 + b] = (float)u[b];
            }
    // F(4,5) conv2 weights: G[j][l] = a_j^l / prod_{i != j} (a_j - a_i) for the finite points, last row picks the leading tap
    {
        const double pts[7] = {0, 1, -1, 2, -2, 0.5, -0.5};
        double G4[8][5];
        for (int jj = 0; jj < 7; ++jj) {
            double den = 1;
            for (int ii = 0; ii < 7; ++ii)
                if (ii != jj) den *= pts[jj] - pts[ii];
            double pw = 1;
            for (int l = 0; l < 5; ++l) { G4[jj][l] = pw / den; pw *= pts[jj]; }
        }
        for (int l = 0; l < 5; ++l) G4[7][l] = l == 4 ? 1.0 : 0.0;
        for (int oc = 0; oc < 32; ++oc)
            for (int c = 0; c < 16; ++c)
                for (int a = 0; a < 5; ++a) {
                    const float *k = w + s3::W2 + ((oc * 16 + c) * 5 + a) * 5;
                    const int cq = c >> 2, g = c & 3, nt = oc >> 4, j = oc & 15, lane = g * 16 + j;
                    for (int b = 0; b < 8; ++b) {
                        double acc = 0;
                        for (int l = 0; l < 5; ++l) acc += G4[b][l] * (double)k[l];
                        f[kS3F7 + ((a * 4 + cq) * 64 + lane) * 16 + nt * 8 + b] = (float)acc;
                    }
                }
    }
}

// =================================================================================================
// Stage 2.  The network is small (162 k MAC per crop), so one WAVE owns a crop: no workgroup barriers,
// four independent crops per workgroup, everything of a crop in that wave's slice of LDS.
// =================================================================================================
namespace {
constexpr int kC2W = 24;                                   // crop row pitch
constexpr int kQ1Row = 16, kQ1Ch = 10 * kQ1Row + 8;        // pooled conv1 map [8][10][16], channel pitch 168 (bank spread)
constexpr int kS2Crop = 24 * 24, kS2Tab = 48, kS2P1 = 8 * kQ1Ch;
constexpr int kS2WaveFloats = kS2Crop + kS2Tab + kS2P1;    // 1968 floats per wave
static_assert(kS2WaveFloats % 4 == 0, "per-wave LDS slices must keep 16-byte alignment");

// Orders this wave's LDS writes before its later LDS reads by other lanes.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    __builtin_amdgcn_wave_barrier();
}
}  // namespace

// Fragment buffer of stage 2 (floats): conv1 [8][64], conv2 [9 taps][2 quads][64], fc [16][2][64][4], and the
// Winograd F(4,3) form of conv2 [3 kernel rows][2 quads][6 points][64].
constexpr int kS2F1 = 0, kS2F2 = kS2F1 + 8 * 64, kS2F3 = kS2F2 + 18 * 64, kS2F4 = kS2F3 + 16 * 2 * 64 * 4,
              kS2FragFloats = kS2F4 + 36 * 64;
constexpr int kS2Feat = 256;

template <int ACT, bool WINO>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3, 3)))
void eval2_conv_kernel(const uint8_t *__restrict__ frame, int fw, int fh, int pitch, const LevelDev *__restrict__ levels,
                       int n_levels, const uint32_t *__restrict__ idx, const int32_t *__restrict__ d_begin,
                       const int32_t *__restrict__ d_n, int n_max, const float *__restrict__ wt,
                       const float *__restrict__ frag, float *__restrict__ feat)
{
    __shared__ __attribute__((aligned(16))) float sMem[4][kS2WaveFloats];
    // per pooling block of conv1 (clamped to the last one): crop offset of its corner | pooled-map offset << 16
    __shared__ uint32_t sLut[112];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 4, j = lane & 15;
    if (tid < 112) {
        const int pb = min(tid, 99);
        sLut[tid] = (uint32_t)(2 * (pb / 10) * kC2W + 2 * (pb % 10)) | (uint32_t)((pb / 10) * kQ1Row + pb % 10) << 16;
    }
    __syncthreads();
    float *sCrop = sMem[wave];
    uint32_t *sTab = reinterpret_cast<uint32_t *>(sCrop + kS2Crop);
    float *sP1 = sCrop + kS2Crop + kS2Tab;
    float *sP2 = sCrop;                          // pooled conv2 output [16][16] re-uses the crop's space

    float b1f[8], b2f[WINO ? 36 : 18];
#pragma unroll
    for (int s = 0; s < 8; ++s) b1f[s] = frag[kS2F1 + s * 64 + lane];
#pragma unroll
    for (int s = 0; s < (WINO ? 36 : 18); ++s) b2f[s] = frag[(WINO ? kS2F4 : kS2F2) + s * 64 + lane];
    const float bias1 = wt[s2::B1 + (j >> 1)], bias2 = wt[s2::B2 + j];
    // conv1 runs with N = 8 channels x 2 adjacent output columns (the two columns of a pooling block), so no
    // half of the matrix tile is idle: K = 5 rows x 6 input columns = 30 -> 8 steps of 4.
    // k-order: steps 0..4 = (row = step, column = g); step 5 = (row = g, column 4); step 6 = (row = g, column 5);
    // step 7 = (4, 4) in group 0, (4, 5) in group 1, zero weights in groups 2 and 3.
    // (offsets relative to a lane base that already includes the tap column g)
    const int off5 = g * kC2W + 4 - g, off6 = g * kC2W + 5 - g, off7 = g == 0 ? 4 * kC2W + 4 : (g == 1 ? 4 * kC2W + 5 - g : -g);
    const int in_lane = (j & 1) * kC2W + g, in_blk = 2 * (j >> 2) + ((j >> 1) & 1), out_blk = 2 * g + (j & 1);

    const int n = min(*d_n, n_max);
    for (int crop = __builtin_amdgcn_readfirstlane(min(*d_begin, n_max) + blockIdx.x * 4 + wave); crop < n; crop += gridDim.x * 4) {
        const Survivor sv = decode(idx[crop], levels, n_levels);
        const int64_t S = levels[sv.level].scale_q16;
        if (lane < 24) crop_axis<kS2In>(sv.x, S, fw, sTab, lane);
        else if (lane < 48) crop_axis<kS2In>(sv.y, S, fh, sTab + 24, lane - 24);
        wave_sync();
        {   // all 18 pixel-pair loads of a lane are issued before the first blend
            uint32_t top[9], bot[9];
#pragma unroll
            for (int it = 0; it < 9; ++it) {
                const int e = it * 64 + lane, r = e / 24, q = e % 24;
                const uint8_t *r0 = frame + (uint32_t)((sTab[24 + r] >> 9) * pitch) + (sTab[q] >> 9);
                top[it] = *reinterpret_cast<const pixel_pair *>(r0);
                bot[it] = *reinterpret_cast<const pixel_pair *>(r0 + pitch);
            }
#pragma unroll
            for (int it = 0; it < 9; ++it) {
                const int e = it * 64 + lane, r = e / 24, q = e % 24;
                const uint32_t wx = sTab[q] & 511u, wy = sTab[24 + r] & 511u;
                const uint32_t tb = (top[it] & 255u) * (256u - wx) + (top[it] >> 8) * wx;
                const uint32_t bb = (bot[it] & 255u) * (256u - wx) + (bot[it] >> 8) * wx;
                const uint32_t acc = tb * (256u - wy) + bb * wy;
                sCrop[e] = normalise((float)acc * (1.0f / 65536.0f));
            }
        }
        wave_sync();

        // ---- conv1 5x5 1->8 + pool.  A tile is 16 base positions (even columns) = 8 pooling blocks:
        // row i of the tile = pooling block 8 t + 2 (i / 4) + (i / 2) % 2, line i % 2 of the block.
        // 100 blocks = 12.5 tiles, done as a round of seven and a round of six (half of the 13th tile is a clamped
        // duplicate that is not stored).
        auto conv1_round = [&](auto n_tiles, int t0) {
            constexpr int NT = decltype(n_tiles)::value;
            floatx4 acc[NT];
            int base[NT];
#pragma unroll
            for (int u = 0; u < NT; ++u) {
                acc[u] = floatx4{0, 0, 0, 0};
                base[u] = (int)(sLut[8 * (t0 + u) + in_blk] & 0xFFFFu) + in_lane;
            }
#pragma unroll
            for (int s = 0; s < 5; ++s)
#pragma unroll
                for (int u = 0; u < NT; ++u) acc[u] = CNNC_MFMA(sCrop[base[u] + s * kC2W], b1f[s], acc[u]);
#pragma unroll
            for (int u = 0; u < NT; ++u) acc[u] = CNNC_MFMA(sCrop[base[u] + off5], b1f[5], acc[u]);
#pragma unroll
            for (int u = 0; u < NT; ++u) acc[u] = CNNC_MFMA(sCrop[base[u] + off6], b1f[6], acc[u]);
#pragma unroll
            for (int u = 0; u < NT; ++u) acc[u] = CNNC_MFMA(sCrop[base[u] + off7], b1f[7], acc[u]);
            // lane (g, j = 2 channel + column): registers 0,1 = the two lines of block 8t + 2g, registers 2,3 of
            // block 8t + 2g + 1; the other column of each block sits in lane j ^ 1
#pragma unroll
            for (int u = 0; u < NT; ++u) {
                float lo = fmaxf(acc[u][0], acc[u][1]), hi = fmaxf(acc[u][2], acc[u][3]);
                lo = fmaxf(lo, lane_xor1(lo));
                hi = fmaxf(hi, lane_xor1(hi));
                const int pb = 8 * (t0 + u) + out_blk;                // even lanes finish the first block, odd the second
                if (pb < 100) sP1[(j >> 1) * kQ1Ch + (sLut[pb] >> 16)] = act_f<ACT>(((j & 1) ? hi : lo) + bias1);
            }
        };
        conv1_round(std::integral_constant<int, 7>{}, 0);
        conv1_round(std::integral_constant<int, 6>{}, 7);
        wave_sync();

        // ---- conv2 3x3 8->16 + pool
        if (WINO) {
            // Winograd F(4, 3) along the rows (points 0, 1, -1, 2, -2, infinity; BT and the pairing of rows as in the
            // F(2, 5) form of stage 3, AT = [1 1 1 1 1 0; 0 1 -1 2 -2 0; 0 1 1 4 4 0; 0 1 -1 8 -8 1]): the 8 x 8 output
            // map is 16 rows of the GEMM (8 output rows x 2 groups of four columns) = one tile, K = 8 channels x 3 kernel
            // rows = 6 steps, six GEMMs: 36 matrix instructions instead of 72.  Row i of the tile = output row
            // 2 (i / 4) + i % 2, column group (i / 2) % 2, so a lane's registers hold both rows of two pooling-block
            // pairs and the four columns of each: pooling stays in registers.
            const int i = lane & 15, unit = i >> 1, Y = unit >> 1, xg = unit & 1;
            const float *dptr = sP1 + g * kQ1Ch + (2 * Y + (i & 1)) * kQ1Row + 4 * xg;
            floatx4 acc[6];
#pragma unroll
            for (int b = 0; b < 6; ++b) acc[b] = floatx4{0, 0, 0, 0};
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int cq = 0; cq < 2; ++cq) {
                    const float *row = dptr + cq * 4 * kQ1Ch + a * kQ1Row;
                    const float4 c0 = *reinterpret_cast<const float4 *>(row);
                    const float2 c1 = *reinterpret_cast<const float2 *>(row + 4);
                    const float e1 = fmaf(-4.0f, c0.z, c1.x), o1 = fmaf(-4.0f, c0.y, c0.w);
                    const float e2 = c1.x - c0.z, o2 = c0.w - c0.y;
                    const float v[6] = {fmaf(4.0f, c0.x, fmaf(-5.0f, c0.z, c1.x)), e1 + o1, e1 - o1, fmaf(2.0f, o2, e2),
                                        fmaf(-2.0f, o2, e2), fmaf(4.0f, c0.y, fmaf(-5.0f, c0.w, c1.y))};
#pragma unroll
                    for (int b = 0; b < 6; ++b) acc[b] = CNNC_MFMA(v[b], b2f[(a * 2 + cq) * 6 + b], acc[b]);
                }
            const floatx4 s1 = acc[1] + acc[2], d1 = acc[1] - acc[2], s2 = acc[3] + acc[4], d2 = acc[3] - acc[4];
            const floatx4 Y0 = acc[0] + s1 + s2, Y1 = d1 + 2.0f * d2, Y2 = s1 + 4.0f * s2, Y3 = d1 + 8.0f * d2 + acc[5];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {                  // registers 2 sub, 2 sub + 1: the two rows of unit 2 g + sub
                const int u = 2 * g + sub, py = u >> 1, px = 2 * (u & 1);
                const float left = fmaxf(fmaxf(Y0[2 * sub], Y1[2 * sub]), fmaxf(Y0[2 * sub + 1], Y1[2 * sub + 1]));
                const float right = fmaxf(fmaxf(Y2[2 * sub], Y3[2 * sub]), fmaxf(Y2[2 * sub + 1], Y3[2 * sub + 1]));
                sP2[j * 16 + 4 * py + px] = act_f<ACT>(left + bias2);
                sP2[j * 16 + 4 * py + px + 1] = act_f<ACT>(right + bias2);
            }
        } else {
            // direct sums: 16 pooling blocks = 4 tiles
            floatx4 acc[4];
            int abase[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                acc[u] = floatx4{0, 0, 0, 0};
                const int pb = 4 * u + (j >> 2);
                abase[u] = g * kQ1Ch + (2 * (pb / 4) + ((j >> 1) & 1)) * kQ1Row + 2 * (pb % 4) + (j & 1);
            }
#pragma unroll
            for (int tap = 0; tap < 9; ++tap)
#pragma unroll
                for (int cq = 0; cq < 2; ++cq)
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        acc[u] = CNNC_MFMA(sP1[abase[u] + (tap / 3) * kQ1Row + tap % 3 + cq * 4 * kQ1Ch], b2f[tap * 2 + cq], acc[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) sP2[j * 16 + 4 * u + g] = act_f<ACT>(max4(acc[u]) + bias2);
        }
        wave_sync();
        reinterpret_cast<float4 *>(feat + (size_t)crop * kS2Feat)[lane] = reinterpret_cast<const float4 *>(sP2)[lane];
        wave_sync();
    }
}

// fc 256->32 + f, fc 32->1 for 16 windows per workgroup; the four waves split K.
template <int ACT>
__global__ __launch_bounds__(kThreads)
void eval2_fc_kernel(const float *__restrict__ feat, const int32_t *__restrict__ d_begin, const int32_t *__restrict__ d_n, int n_max,
                     const float *__restrict__ wt, const float *__restrict__ frag, float *__restrict__ out)
{
    __shared__ float sPart[4][16][33];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 4, j = lane & 15;
    const int n = min(*d_n, n_max);
    const float4 *wf = reinterpret_cast<const float4 *>(frag + kS2F3) + lane;     // [chunk][n-tile][lane] float4
    const int first = min(*d_begin, n_max);            // tiles of sixteen windows are counted from the range's first one
    for (int tile = blockIdx.x; first + tile * 16 < n; tile += gridDim.x) {
        const int row = min(first + tile * 16 + j, n - 1);
        const float4 *ap = reinterpret_cast<const float4 *>(feat + (size_t)row * kS2Feat) + g;
        floatx4 acc[2] = {floatx4{0, 0, 0, 0}, floatx4{0, 0, 0, 0}};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int ch = wave + 4 * q;
            const float4 a4 = ap[ch * 4];
            const float4 p = wf[(ch * 2) * 64], r = wf[(ch * 2 + 1) * 64];
            acc[0] = CNNC_MFMA(a4.x, p.x, acc[0]); acc[1] = CNNC_MFMA(a4.x, r.x, acc[1]);
            acc[0] = CNNC_MFMA(a4.y, p.y, acc[0]); acc[1] = CNNC_MFMA(a4.y, r.y, acc[1]);
            acc[0] = CNNC_MFMA(a4.z, p.z, acc[0]); acc[1] = CNNC_MFMA(a4.z, r.z, acc[1]);
            acc[0] = CNNC_MFMA(a4.w, p.w, acc[0]); acc[1] = CNNC_MFMA(a4.w, r.w, acc[1]);
        }
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) sPart[wave][4 * g + r][nt * 16 + j] = acc[nt][r];
        __syncthreads();
        {
            const int r = tid >> 4, c0 = tid & 15;
            float part = 0.0f;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int c = c0 + 16 * q;
                const float h = sPart[0][r][c] + sPart[1][r][c] + sPart[2][r][c] + sPart[3][r][c] + wt[s2::B3 + c];
                part = fmaf(wt[s2::W4 + c], act_f<ACT>(h), part);
            }
#pragma unroll
            for (int d = 8; d >= 1; d >>= 1) part += __shfl_xor(part, d, 64);
            if (c0 == 0 && first + tile * 16 + r < n) out[first + tile * 16 + r] = part + wt[s2::B4];
        }
        __syncthreads();
    }
}

size_t eval2_frag_floats() { return kS2FragFloats; }
size_t eval2_feat_floats() { return kS2Feat; }

void eval2_make_fragments(const float *w, float *f)
{
    // conv1: column n of the tile = (channel n / 2, output column n % 2); k = (row a, input column b) with the
    // input column counted from the even output column, so the weight is w[channel][a][b - n % 2]
    for (int s = 0; s < 8; ++s)
        for (int lane = 0; lane < 64; ++lane) {
            const int g = lane >> 4, j = lane & 15, ch = j >> 1, dx = j & 1;
            int a = -1, b = -1;
            if (s < 5) { a = s; b = g; }
            else if (s == 5) { a = g; b = 4; }
            else if (s == 6) { a = g; b = 5; }
            else if (g == 0) { a = 4; b = 4; }
            else if (g == 1) { a = 4; b = 5; }
            const int tap = b - dx;
            f[kS2F1 + s * 64 + lane] = (a < 0 || a > 4 || tap < 0 || tap > 4) ? 0.0f : w[s2::W1 + (ch * 5 + a) * 5 + tap];
        }
    for (int tap = 0; tap < 9; ++tap)
        for (int cq = 0; cq < 2; ++cq)
            for (int lane = 0; lane < 64; ++lane) {
                const int g = lane >> 4, j = lane & 15, c = 4 * cq + g;
                f[kS2F2 + (tap * 2 + cq) * 64 + lane] = w[s2::W2 + (j * 8 + c) * 9 + tap];
            }
    for (int ch = 0; ch < 16; ++ch)
        for (int nt = 0; nt < 2; ++nt)
            for (int lane = 0; lane < 64; ++lane)
                for (int s = 0; s < 4; ++s) {
                    const int g = lane >> 4, j = lane & 15;
                    f[kS2F3 + ((ch * 2 + nt) * 64 + lane) * 4 + s] = w[s2::W3 + (nt * 16 + j) * 256 + 16 * ch + 4 * g + s];
                }
    // conv2 in the Winograd F(4,3) domain along the kernel columns, points 0, 1, -1, 2, -2, infinity (fp64, then rounded)
    static const double G[6][3] = {{1.0 / 4, 0, 0}, {-1.0 / 6, -1.0 / 6, -1.0 / 6}, {-1.0 / 6, 1.0 / 6, -1.0 / 6},
                                   {1.0 / 24, 1.0 / 12, 1.0 / 6}, {1.0 / 24, -1.0 / 12, 1.0 / 6}, {0, 0, 1}};
    for (int a = 0; a < 3; ++a)
        for (int cq = 0; cq < 2; ++cq)
            for (int b = 0; b < 6; ++b)
                for (int lane = 0; lane < 64; ++lane) {
                    const int g = lane >> 4, j = lane & 15, c = 4 * cq + g;
                    const float *k = w + s2::W2 + ((j * 8 + c) * 3 + a) * 3;
                    f[kS2F4 + ((a * 2 + cq) * 6 + b) * 64 + lane] = (float)(G[b][0] * k[0] + G[b][1] * k[1] + G[b][2] * k[2]);
                }
}

// Matrix instructions (16x16x4, 1024 multiply-adds each) the convolution kernels issue per crop, padding tiles and
// Winograd forms included: what "executed" work means next to the algorithmic count of the layer definitions.
int64_t eval3_mfma_per_crop(int impl)
{
    const int64_t conv1 = 8 * 4 * 4 * 7;                                      // 8 rounds x 4 tiles x 4 waves, 7 k-steps
    const int64_t conv2 = impl == 3 ? 4 * (20 * 16 + 20 * 8)                   // F(4,5): a whole and a half tile per wave
                        : impl == 2 ? (int64_t)kWinoTiles * 20 * 12            // F(2,5)
                                    : 21 * 25 * 4 * 2;                         // direct: 21 tiles, 25 taps x 4 channel quads, 2 n-tiles
    const int64_t conv3 = impl >= 2 ? 4 * 24 * 4 : 4 * 9 * 2 * 4 * 2;
    return conv1 + conv2 + conv3;
}
int64_t eval2_mfma_per_crop(int impl) { return 13 * 8 + (impl == 3 ? 36 : 72); }

namespace {
int conv_grid(const cnnc_ctx *c)
{
    int g = 256 * 3;   // three workgroups fit a compute unit's LDS; each strides over the list
    return c->max_surv < g ? c->max_surv : g;
}
int fc_grid(const cnnc_ctx *c)
{
    const int tiles = (c->max_surv + 15) / 16;
    return tiles < 1024 ? tiles : 1024;
}
}  // namespace


hipError_t launch_eval3_mfma(cnnc_ctx *c, ListRange r, hipStream_t st)
{
#define CNNC_E3(ACT)                                                                                              \
    for (int seg_lo = 0; seg_lo < c->max_surv; seg_lo += kS3Segment) {                                            \
        const int seg_hi = std::min(seg_lo + kS3Segment, c->max_surv);                                            \
        {                                                                                                         \
            ScopedTimer timer_(c, CNNC_T_STAGE3_CONV, st);                                                        \
            hipLaunchKernelGGL((eval3_conv_kernel<ACT, WINO>), dim3(std::min(conv_grid(c), seg_hi - seg_lo)), dim3(kThreads), 0, st, \
                           c->d_frame, c->fw, c->fh, c->fpitch, c->d_levels, c->n_levels, c->d_idx[1], r.d_begin, r.d_end, \
                           seg_lo, seg_hi, c->d_wt[2], c->d_frag[1], c->d_feat[1]);                               \
        }                                                                                                         \
        hipLaunchKernelGGL(eval3_fc_kernel<ACT>, dim3(std::min(fc_grid(c), (seg_hi - seg_lo + 15) / 16)), dim3(kFcThreads), 0, st, \
                           c->d_feat[1], r.d_begin, r.d_end, seg_lo, seg_hi, c->d_wt[2], c->d_frag[1], c->d_eval[1]); \
    }
#define CNNC_E3W(ACT)                     \
    if (c->eval_impl == 3) {              \
        constexpr int WINO = 2;           \
        CNNC_E3(ACT);                     \
    } else if (c->eval_impl == 2) {       \
        constexpr int WINO = 1;           \
        CNNC_E3(ACT);                     \
    } else {                              \
        constexpr int WINO = 0;           \
        CNNC_E3(ACT);                     \
    }
    switch (c->act) {
    case CNNC_ACT_RATIONAL: CNNC_E3W(CNNC_ACT_RATIONAL); break;
    case CNNC_ACT_SCALED_TANH: CNNC_E3W(CNNC_ACT_SCALED_TANH); break;
    default: CNNC_E3W(CNNC_ACT_TANH); break;
    }
#undef CNNC_E3W
#undef CNNC_E3
    return hipGetLastError();
}

hipError_t launch_eval2_mfma(cnnc_ctx *c, ListRange r, hipStream_t st)
{
    const int waves = c->max_surv < 256 * 3 * 4 ? c->max_surv : 256 * 3 * 4;   // three workgroups of four crops per compute unit (register limit)
    const int grid = (waves + 3) / 4;
#define CNNC_E2(ACT)                                                                                              \
    {                                                                                                             \
        ScopedTimer timer_(c, CNNC_T_STAGE2_CONV, st);                                                            \
        hipLaunchKernelGGL((eval2_conv_kernel<ACT, WINO>), dim3(grid), dim3(kThreads), 0, st, c->d_frame, c->fw, c->fh, \
                       c->fpitch, c->d_levels, c->n_levels, c->d_idx[0], r.d_begin, r.d_end, c->max_surv, c->d_wt[1], \
                       c->d_frag[0], c->d_feat[0]);                                                                \
    }                                                                                                             \
    hipLaunchKernelGGL(eval2_fc_kernel<ACT>, dim3(fc_grid(c)), dim3(kThreads), 0, st, c->d_feat[0], r.d_begin, r.d_end, \
                       c->max_surv, c->d_wt[1], c->d_frag[0], c->d_eval[0])
#define CNNC_E2W(ACT)                     \
    if (c->eval_impl == 3) {              \
        constexpr bool WINO = true;       \
        CNNC_E2(ACT);                     \
    } else {                              \
        constexpr bool WINO = false;      \
        CNNC_E2(ACT);                     \
    }
    switch (c->act) {
    case CNNC_ACT_RATIONAL: CNNC_E2W(CNNC_ACT_RATIONAL); break;
    case CNNC_ACT_SCALED_TANH: CNNC_E2W(CNNC_ACT_SCALED_TANH); break;
    default: CNNC_E2W(CNNC_ACT_TANH); break;
    }
#undef CNNC_E2W
#undef CNNC_E2
    return hipGetLastError();
}

}  // namespace cnnc
