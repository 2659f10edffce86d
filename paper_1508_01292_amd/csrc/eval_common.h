// Device helpers shared by the stage-2 / stage-3 kernels: crop gathering and survivor decoding.
#pragma once
#include "act.h"
#include "cnnc_internal.h"

namespace cnnc {
namespace evalc {
constexpr int kThreads = 256;

// The value itself, in a form the compiler must treat as new at every call: index arithmetic that depends on it is
// then recomputed where it is used instead of being hoisted out of the per-window loop, kept in registers across all
// layers and spilled to scratch memory.
__device__ __forceinline__ int fresh(int x)
{
    asm volatile("" : "+v"(x));
    return x;
}

// Sample positions of one crop axis: tab[i] = (index of left pixel << 9) | weight of the right one (0..256).
// The left index never is the last pixel of the axis: a position clamped onto it is stored as the pixel
// before with weight 256, which blends to the same integer and lets every reader fetch index and index + 1.
template <int N>
__device__ __forceinline__ void crop_axis(int origin, int64_t S, int n_in, uint32_t *tab, int i)
{
    int64_t P = (int64_t)origin * S + ((int64_t)(2 * i + 1) * kWin * S) / (2 * N) - 32768;
    const int64_t hi = (int64_t)(n_in - 1) << 16;
    P = P < 0 ? 0 : (P > hi ? hi : P);
    uint32_t idx = (uint32_t)(P >> 16), w = (uint32_t)(((P & 0xFFFF) + 128) >> 8);
    if (idx == (uint32_t)(n_in - 1)) { idx -= 1; w = 256; }      // P == hi here, so w was 0
    tab[i] = (idx << 9) | w;
}

// The gather of a crop in three parts, so that a kernel can put other work between the issue of the pixel
// loads and their use: (1) tables of sample positions into LDS, (2) all pixel loads of a thread into
// registers, (3) blend, normalise and store into the crop buffer.  The caller synchronises between the parts
// and leaves the tables alone until part 3 is done.
typedef uint16_t __attribute__((aligned(1))) pixel_pair;           // two neighbouring pixels of a row, any address

template <int N>
struct CropPixels {
    static constexpr int kIt = (N * N + kThreads - 1) / kThreads;
    uint32_t top[kIt], bot[kIt];                                   // pixel pairs of the upper and the lower row
};

template <int N>
__device__ __forceinline__ void crop_tables(int x, int y, int64_t S, int fw, int fh, uint32_t *sTab)
{
    const int tid = threadIdx.x;
    if (tid < N) crop_axis<N>(x, S, fw, sTab, tid);
    else if (tid < 2 * N) crop_axis<N>(y, S, fh, sTab + N, tid - N);
}

template <int N>
__device__ __forceinline__ void crop_issue(const uint8_t *__restrict__ frame, int pitch, const uint32_t *sTab, CropPixels<N> &px)
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int it = 0; it < CropPixels<N>::kIt; ++it) {
        const int e = min(it * kThreads + tid, N * N - 1);
        const int i = e / N, j = e % N;
        const uint32_t x0 = sTab[j] >> 9, y0 = sTab[N + i] >> 9;
        const uint8_t *r0 = frame + (size_t)y0 * pitch + x0;
        px.top[it] = *reinterpret_cast<const pixel_pair *>(r0);
        px.bot[it] = *reinterpret_cast<const pixel_pair *>(r0 + pitch);
    }
}

template <int N>
__device__ __forceinline__ void crop_finish(const CropPixels<N> &px, const uint32_t *sTab, float *sCrop)
{
    const int tid = fresh(threadIdx.x);
#pragma unroll
    for (int it = 0; it < CropPixels<N>::kIt; ++it) {
        const int e = it * kThreads + tid, ec = min(e, N * N - 1);
        const uint32_t wx = sTab[ec % N] & 511u, wy = sTab[N + ec / N] & 511u;
        const uint32_t top = (px.top[it] & 255u) * (256u - wx) + (px.top[it] >> 8) * wx;     // the same integer as the
        const uint32_t bot = (px.bot[it] & 255u) * (256u - wx) + (px.bot[it] >> 8) * wx;     // four-term sum, below 2^24
        const uint32_t acc = top * (256u - wy) + bot * wy;
        if (e < N * N) sCrop[e] = normalise((float)acc * (1.0f / 65536.0f));
    }
}

template <int N>
__device__ void gather_crop(const uint8_t *__restrict__ frame, int fw, int fh, int pitch, int x, int y,
                            int64_t S, uint32_t *sTab, float *sCrop)
{
    crop_tables<N>(x, y, S, fw, fh, sTab);
    __syncthreads();
    CropPixels<N> px;
    crop_issue<N>(frame, pitch, sTab, px);
    crop_finish<N>(px, sTab, sCrop);
    __syncthreads();
}

struct Survivor { int level, x, y; };

__device__ __forceinline__ Survivor decode(uint32_t g, const LevelDev *__restrict__ levels, int n_levels)
{
    int l = 0;
    while (l + 1 < n_levels && g >= (uint32_t)levels[l + 1].score_off) ++l;
    const uint32_t rem = g - (uint32_t)levels[l].score_off;
    const int ow = levels[l].ow;
    return {l, (int)(rem % ow), (int)(rem / ow)};
}
}  // namespace evalc
}  // namespace cnnc
