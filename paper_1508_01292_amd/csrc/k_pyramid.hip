// Image pyramid (paper, Sections 2 and 3.3: the only pre-processing the detector needs).
// All levels are resampled from the frame in ONE launch that reads the frame ONCE: a workgroup stages a
// kPyrTileW x kPyrTileH tile of the frame (plus one column and one row of halo) in LDS with 16-byte row loads
// and then produces, for every level, the level pixels whose upper-left source pixel lies in that tile (a
// level pixel blends the 2 x 2 frame pixels at and after its source position, so the halo is all it needs
// from outside).  Each level pixel blends four frame pixels with 8-bit weights in integer arithmetic, so the
// result is bit-identical to any other implementation of the same rule.
#include "cnnc_internal.h"

namespace cnnc {

namespace {
constexpr int FW = kPyrTileW, FH = kPyrTileH, kPitch = FW + 16;     // LDS row: the tile's pixels, the halo pixel, padding
constexpr int kThreads = 256;
}  // namespace

// taps: per level a column and a row table; entry = index of the left / upper source pixel in the high bits, weight
// of the right / lower neighbour (0..256) in the low 9 bits.  first: per level ntx + 1 column entries and nty + 1 row
// entries; entry t = number of level columns (rows) whose source index lies before frame tile t, so tile t owns the
// columns [first[t], first[t + 1]).
__global__ __launch_bounds__(kThreads)
void pyramid_kernel(const uint8_t *__restrict__ frame, int fw, int fh, int pitch, const LevelDev *__restrict__ levels,
                    int n_levels, const uint32_t *__restrict__ taps, const uint32_t *__restrict__ first, int ntx, int nty,
                    uint8_t *__restrict__ pyr)
{
    __shared__ __attribute__((aligned(16))) uint8_t sT[(FH + 1) * kPitch];
    const int tid = threadIdx.x;
    // Workgroups go to the eight XCDs (each with its own L2) in turn.  Neighbouring tiles share their halo lines, so
    // every XCD gets a run of consecutive tiles: the line one tile reads as halo is in that L2 for the tile that owns it.
    const int n_tiles = ntx * nty, per_xcd = (n_tiles + 7) / 8;
    const int tile = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (tile >= n_tiles) return;
    const int tx = tile % ntx, ty = tile / ntx, x0 = tx * FW, y0 = ty * FH;

    // ---- per level: which of its columns and rows this tile produces, and where the level lives (one lane a level,
    // so that these dependent loads are in flight together with the tile's pixels)
    __shared__ int sXa[CNNC_MAX_LEVELS], sNx[CNNC_MAX_LEVELS], sYa[CNNC_MAX_LEVELS], sCum[CNNC_MAX_LEVELS + 1];
    __shared__ int sXmap[CNNC_MAX_LEVELS], sYmap[CNNC_MAX_LEVELS], sLw[CNNC_MAX_LEVELS], sOff[CNNC_MAX_LEVELS];
    if (tid < 64) {
        int n = 0;
        if (tid < n_levels) {
            const uint32_t *f = first + tid * (ntx + nty + 2);
            const int xa = (int)f[tx], nx = (int)f[tx + 1] - xa, ya = (int)f[ntx + 1 + ty], ny = (int)f[ntx + 2 + ty] - ya;
            sXa[tid] = xa; sNx[tid] = max(nx, 1); sYa[tid] = ya;
            sXmap[tid] = levels[tid].xmap_off; sYmap[tid] = levels[tid].ymap_off; sLw[tid] = levels[tid].w;
            sOff[tid] = levels[tid].pyr_off;
            n = nx > 0 && ny > 0 ? nx * ny : 0;
        }
        int incl = n;                                   // running number of pixels over the levels
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(incl, d, 64);
            if (tid >= d) incl += o;
        }
        sCum[tid + 1] = incl;
        if (tid == 0) sCum[0] = 0;
    }

    // ---- the tile: rows y0 .. y0 + FH, columns x0 .. x0 + FW, both clamped to the frame; sixteen pixels a load where
    // the frame's alignment allows it
    const bool wide = (pitch & 15) == 0 && (reinterpret_cast<uintptr_t>(frame) & 15) == 0;
    for (int e = tid; e < (FH + 1) * (FW / 16 + 1); e += kThreads) {
        const int r = e / (FW / 16 + 1), q = e % (FW / 16 + 1);
        const uint8_t *row = frame + (size_t)min(y0 + r, fh - 1) * pitch;
        uint8_t *dst = sT + r * kPitch + 16 * q;
        if (q == FW / 16) {
            dst[0] = row[min(x0 + FW, fw - 1)];                       // the halo pixel
        } else if (wide && x0 + 16 * q + 16 <= fw) {
            *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(row + x0 + 16 * q);
        } else {
            for (int k = 0; k < 16; ++k) dst[k] = row[min(x0 + 16 * q + k, fw - 1)];
        }
    }
    __syncthreads();

    // ---- the pixels of all levels that belong to this tile, as one list shared out over the threads
    const int total = sCum[n_levels];
    for (int e = tid; e < total; e += kThreads) {
        int lvl = 0;
        while (sCum[lvl + 1] <= e) ++lvl;               // most pixels belong to the first few levels
        const int k = e - sCum[lvl], nx = sNx[lvl];
        const int oy = sYa[lvl] + k / nx, ox = sXa[lvl] + k % nx;
        const uint32_t ex = taps[sXmap[lvl] + ox], ey = taps[sYmap[lvl] + oy];
        const int gx = (int)(ex >> 9), gy = (int)(ey >> 9);
        const uint32_t wx = ex & 511u, wy = ey & 511u;
        const uint8_t *r0 = sT + (gy - y0) * kPitch + (gx - x0);
        const int dx = gx + 1 < fw ? 1 : 0, dy = gy + 1 < fh ? kPitch : 0;     // the neighbour, or the pixel itself at the frame edge
        const uint32_t p00 = r0[0], p01 = r0[dx], p10 = r0[dy], p11 = r0[dy + dx];
        const uint32_t acc = p00 * (256u - wx) * (256u - wy) + p01 * wx * (256u - wy)
                           + p10 * (256u - wx) * wy + p11 * wx * wy;
        pyr[(size_t)sOff[lvl] + (size_t)oy * sLw[lvl] + ox] = (uint8_t)((acc + 32768u) >> 16);
    }
}

hipError_t launch_pyramid(const cnnc_ctx *c, hipStream_t st)
{
    hipLaunchKernelGGL(pyramid_kernel, dim3(8 * ((c->pyr_ntx * c->pyr_nty + 7) / 8)), dim3(kThreads), 0, st, c->d_frame, c->fw, c->fh,
                       c->fpitch, c->d_levels, c->n_levels, c->d_taps, c->d_tiles_pyr, c->pyr_ntx, c->pyr_nty, c->d_pyr);
    return hipGetLastError();
}

}  // namespace cnnc
