// Device helpers shared by the stage-2 / stage-3 kernels: crop gathering and survivor decoding.
#pragma once
#include "act.h"
#include "cnnc_internal.h"

namespace cnnc {
namespace evalc {
constexpr int kThreads = 256;

// Sample positions of one crop axis: tab[i] = (index of left pixel << 9) | weight of the right one.
template <int N>
__device__ __forceinline__ void crop_axis(int origin, int64_t S, int n_in, uint32_t *tab, int i)
{
    int64_t P = (int64_t)origin * S + ((int64_t)(2 * i + 1) * kWin * S) / (2 * N) - 32768;
    const int64_t hi = (int64_t)(n_in - 1) << 16;
    P = P < 0 ? 0 : (P > hi ? hi : P);
    tab[i] = ((uint32_t)(P >> 16) << 9) | (uint32_t)(((P & 0xFFFF) + 128) >> 8);
}

template <int N>
__device__ void gather_crop(const uint8_t *__restrict__ frame, int fw, int fh, int pitch, int x, int y,
                            int64_t S, uint32_t *sTab, float *sCrop)
{
    const int tid = threadIdx.x;
    if (tid < N) crop_axis<N>(x, S, fw, sTab, tid);
    else if (tid < 2 * N) crop_axis<N>(y, S, fh, sTab + N, tid - N);
    __syncthreads();
    // all pixel loads of a thread are issued before the first blend, so their latency is paid once
    constexpr int kIt = (N * N + kThreads - 1) / kThreads;
    uint32_t p00[kIt], p01[kIt], p10[kIt], p11[kIt], wxy[kIt];
#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const int e = min(it * kThreads + tid, N * N - 1);
        const int i = e / N, j = e % N;
        const uint32_t ex = sTab[j], ey = sTab[N + i];
        const int x0 = ex >> 9, y0 = ey >> 9;
        const int x1 = min(x0 + 1, fw - 1), y1 = min(y0 + 1, fh - 1);
        const uint8_t *r0 = frame + (size_t)y0 * pitch, *r1 = frame + (size_t)y1 * pitch;
        p00[it] = r0[x0]; p01[it] = r0[x1]; p10[it] = r1[x0]; p11[it] = r1[x1];
        wxy[it] = ((ex & 511u) << 16) | (ey & 511u);
    }
#pragma unroll
    for (int it = 0; it < kIt; ++it) {
        const int e = it * kThreads + tid;
        const uint32_t wx = wxy[it] >> 16, wy = wxy[it] & 0xFFFFu;
        const uint32_t acc = p00[it] * (256u - wx) * (256u - wy) + p01[it] * wx * (256u - wy)
                           + p10[it] * (256u - wx) * wy + p11[it] * wx * wy;
        if (e < N * N) sCrop[e] = normalise((float)acc * (1.0f / 65536.0f));
    }
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
