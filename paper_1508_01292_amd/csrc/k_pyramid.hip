// Image pyramid (paper, Sections 2 and 3.3: the only pre-processing the detector needs).
// All levels are resampled from the frame in ONE launch over a (level, tile) table; each level
// pixel blends four frame pixels with 8-bit weights in integer arithmetic, so the result is
// bit-identical to any other implementation of the same rule.
#include "cnnc_internal.h"

namespace cnnc {

// Tap table entry: index of the left / upper source pixel in the high bits, weight of the
// right / lower neighbour (0..256) in the low 9 bits.
__global__ __launch_bounds__(kPyrTileW * kPyrTileH)
void pyramid_kernel(const uint8_t *__restrict__ frame, int fw, int fh, int pitch,
                    const LevelDev *__restrict__ levels, const uint32_t *__restrict__ taps,
                    const uint32_t *__restrict__ tiles, uint8_t *__restrict__ pyr)
{
    const uint32_t t = tiles[blockIdx.x];
    const int lvl = t >> 24, ty = (t >> 12) & 0xFFF, tx = t & 0xFFF;
    const LevelDev L = levels[lvl];
    const int x = tx * kPyrTileW + (threadIdx.x % kPyrTileW);
    const int y = ty * kPyrTileH + (threadIdx.x / kPyrTileW);
    if (x >= L.w || y >= L.h) return;
    const uint32_t ex = taps[L.xmap_off + x], ey = taps[L.ymap_off + y];
    const int x0 = ex >> 9, y0 = ey >> 9;
    const uint32_t wx = ex & 511u, wy = ey & 511u;
    const int x1 = min(x0 + 1, fw - 1), y1 = min(y0 + 1, fh - 1);
    const uint8_t *r0 = frame + (size_t)y0 * pitch, *r1 = frame + (size_t)y1 * pitch;
    const uint32_t p00 = r0[x0], p01 = r0[x1], p10 = r1[x0], p11 = r1[x1];
    const uint32_t acc = p00 * (256u - wx) * (256u - wy) + p01 * wx * (256u - wy)
                       + p10 * (256u - wx) * wy + p11 * wx * wy;
    pyr[(size_t)L.pyr_off + (size_t)y * L.w + x] = (uint8_t)((acc + 32768u) >> 16);
}

hipError_t launch_pyramid(const cnnc_ctx *c, hipStream_t st)
{
    hipLaunchKernelGGL(pyramid_kernel, dim3(c->n_tiles_pyr), dim3(kPyrTileW * kPyrTileH), 0, st,
                       c->d_frame, c->fw, c->fh, c->fpitch, c->d_levels, c->d_taps, c->d_tiles_pyr, c->d_pyr);
    return hipGetLastError();
}

}  // namespace cnnc
