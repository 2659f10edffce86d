// Merging of the windows accepted by the last stage (paper, Section 3.3, last paragraph:
// non-maximum suppression aggregates the found regions; Section 4.2: minNeighbors).
// Greedy rule: in order of descending score (ties: ascending flat window index) a box not yet
// absorbed is kept and absorbs every later box whose intersection exceeds merge_iou * union.
//
// Two launches: a rank sort that also turns windows into frame-pixel boxes, and the greedy pass in
// one workgroup with the absorbed flags in LDS.
#include "cnnc_internal.h"

namespace cnnc {

namespace {
constexpr int kMergeThreads = 1024;
constexpr int kMergeCapMax = 32768;

struct SortedBox {
    int32_t x, y, size;
    float score;
    int32_t level, index;
};

__device__ __forceinline__ int32_t round_half_up(double v) { return (int32_t)floor(__dadd_rn(v, 0.5)); }
}  // namespace

size_t merge_workspace_bytes(int merge_cap) { return sizeof(SortedBox) * (size_t)merge_cap; }

__global__ __launch_bounds__(256)
void merge_rank_kernel(const uint32_t *__restrict__ idx, const float *__restrict__ sc,
                       const int32_t *__restrict__ d_n, int n_max, const LevelDev *__restrict__ levels,
                       int n_levels, SortedBox *__restrict__ sorted)
{
    const int n = min(*d_n, n_max);
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float s = sc[i];
    int rank = 0;
    for (int j = 0; j < n; ++j) {
        const float t = sc[j];
        rank += (t > s || (t == s && j < i)) ? 1 : 0;
    }
    const uint32_t g = idx[i];
    int l = 0;
    while (l + 1 < n_levels && g >= (uint32_t)levels[l + 1].score_off) ++l;
    const uint32_t rem = g - (uint32_t)levels[l].score_off;
    const int ow = levels[l].ow;
    const int x = rem % ow, y = rem / ow;
    const double scale = levels[l].scale;
    SortedBox b;
    b.x = round_half_up(__dmul_rn((double)x, scale));
    b.y = round_half_up(__dmul_rn((double)y, scale));
    b.size = round_half_up(__dmul_rn((double)kWin, scale));
    b.score = s;
    b.level = l;
    b.index = (int32_t)g;
    sorted[rank] = b;
}

__global__ __launch_bounds__(kMergeThreads)
void merge_greedy_kernel(const SortedBox *__restrict__ sorted, const int32_t *__restrict__ d_n, int n_max,
                         float iou, int min_neighbors, cnnc_det *__restrict__ det, int det_cap,
                         int32_t *__restrict__ d_ndet)
{
    __shared__ uint8_t dead[kMergeCapMax];
    __shared__ int s_nb, s_kept;
    const int n = min(*d_n, n_max);
    for (int j = threadIdx.x; j < n; j += kMergeThreads) dead[j] = 0;
    if (threadIdx.x == 0) { s_nb = 0; s_kept = 0; }
    __syncthreads();
    const double thr = (double)iou;
    for (int i = 0; i < n; ++i) {
        if (dead[i]) continue;              // same value in every thread: read after the last barrier
        const SortedBox a = sorted[i];
        const int64_t ax1 = (int64_t)a.x + a.size, ay1 = (int64_t)a.y + a.size;
        const int64_t aa = (int64_t)a.size * a.size;
        int cnt = 0;
        for (int j = i + 1 + threadIdx.x; j < n; j += kMergeThreads) {
            if (dead[j]) continue;
            const SortedBox b = sorted[j];
            const int64_t iw = min(ax1, (int64_t)b.x + b.size) - max((int64_t)a.x, (int64_t)b.x);
            const int64_t ih = min(ay1, (int64_t)b.y + b.size) - max((int64_t)a.y, (int64_t)b.y);
            if (iw <= 0 || ih <= 0) continue;
            const int64_t inter = iw * ih, uni = aa + (int64_t)b.size * b.size - inter;
            if ((double)inter > __dmul_rn(thr, (double)uni)) { dead[j] = 1; ++cnt; }
        }
        if (cnt) atomicAdd(&s_nb, cnt);
        __syncthreads();
        if (threadIdx.x == 0) {
            if (s_nb + 1 >= min_neighbors) {
                if (s_kept < det_cap) {
                    cnnc_det d;
                    d.x = a.x; d.y = a.y; d.size = a.size; d.score = a.score;
                    d.level = a.level; d.neighbors = s_nb; d.index = a.index; d.reserved = 0;
                    det[s_kept] = d;
                }
                ++s_kept;
            }
            s_nb = 0;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) *d_ndet = s_kept;
}

hipError_t launch_merge(const cnnc_ctx *c, hipStream_t st)
{
    SortedBox *sorted = static_cast<SortedBox *>(c->d_merge_ws);
    const int nb = (c->merge_cap + 255) / 256;
    hipLaunchKernelGGL(merge_rank_kernel, dim3(nb), dim3(256), 0, st, c->d_idx[2], c->d_sc[2], &c->d_cnt->n[2],
                       c->merge_cap, c->d_levels, c->n_levels, sorted);
    hipLaunchKernelGGL(merge_greedy_kernel, dim3(1), dim3(kMergeThreads), 0, st, sorted, &c->d_cnt->n[2],
                       c->merge_cap, c->params.merge_iou, c->params.min_neighbors, c->d_det, c->merge_cap,
                       &c->d_cnt->n[3]);
    return hipGetLastError();
}

}  // namespace cnnc
