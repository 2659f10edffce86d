// Merging of the windows accepted by the last stage (paper, Section 3.3, last paragraph:
// non-maximum suppression aggregates the found regions; Section 4.2: minNeighbors).
// Greedy rule: in order of descending score (ties: ascending flat window index) a box not yet
// absorbed is kept and absorbs every later box whose intersection exceeds merge_iou * union.
//
// The greedy rule is sequential as stated; here it is evaluated in parallel rounds that give the
// same result.  With O the symmetric "overlaps more than the threshold" relation of the sorted
// boxes, a box is KEPT once all earlier boxes overlapping it are known to be absorbed, and ABSORBED
// once one earlier overlapping box is known to be kept.  The earliest undecided box is decided in
// every round, so the rounds end; typical depth is a handful.  The neighbour count of a kept box
// is the number of absorbed boxes whose FIRST kept overlapping predecessor it is, which is what the
// sequential pass counts.
//
// Launches: rank (counting sort position of every box, n^2 comparisons spread over the chip),
// scatter into sorted order as frame-pixel boxes, overlap bit matrix, and the rounds + ordered
// output in one workgroup.
#include "cnnc_internal.h"

namespace cnnc {

namespace {
constexpr int kMergeCapMax = 32768;
constexpr int kResolveThreads = 1024;
constexpr int kRankSplit = 8;

struct SortedBox {
    int32_t x, y, size;
    float score;
    int32_t level, index;
};

struct MergeWs {
    SortedBox *sorted;
    int32_t *rank;     // zero between calls
    int32_t *nb;
    unsigned long long *overlap;   // [cap][words]
    int words;                      // 64-bit words per row
};

__host__ __device__ inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

inline MergeWs carve(void *base, int cap)
{
    MergeWs w;
    char *p = static_cast<char *>(base);
    w.sorted = reinterpret_cast<SortedBox *>(p); p += align256(sizeof(SortedBox) * (size_t)cap);
    w.rank = reinterpret_cast<int32_t *>(p); p += align256(sizeof(int32_t) * (size_t)cap);
    w.nb = reinterpret_cast<int32_t *>(p); p += align256(sizeof(int32_t) * (size_t)cap);
    w.overlap = reinterpret_cast<unsigned long long *>(p);
    w.words = (cap + 63) / 64;
    return w;
}

__device__ __forceinline__ int32_t round_half_up(double v) { return (int32_t)floor(__dadd_rn(v, 0.5)); }

__device__ __forceinline__ bool overlaps(const SortedBox &a, const SortedBox &b, double thr)
{
    const int64_t iw = min((int64_t)a.x + a.size, (int64_t)b.x + b.size) - max((int64_t)a.x, (int64_t)b.x);
    const int64_t ih = min((int64_t)a.y + a.size, (int64_t)b.y + b.size) - max((int64_t)a.y, (int64_t)b.y);
    if (iw <= 0 || ih <= 0) return false;
    const int64_t inter = iw * ih, uni = (int64_t)a.size * a.size + (int64_t)b.size * b.size - inter;
    return (double)inter > __dmul_rn(thr, (double)uni);   // exact: 24-bit threshold times an integer below 2^29
}
}  // namespace

size_t merge_workspace_bytes(int cap)
{
    return align256(sizeof(SortedBox) * (size_t)cap) + 2 * align256(sizeof(int32_t) * (size_t)cap) +
           sizeof(unsigned long long) * (size_t)cap * ((cap + 63) / 64);
}

// rank[i] += number of boxes in this block's share of j that sort before box i
__global__ __launch_bounds__(256)
void merge_rank_kernel(const float *__restrict__ sc, const int32_t *__restrict__ d_n, int n_max, int32_t *__restrict__ rank)
{
    __shared__ float sS[256];
    const int n = min(*d_n, n_max);
    if ((int)blockIdx.x * 256 >= n) return;
    const int i = blockIdx.x * 256 + threadIdx.x;
    const float s = i < n ? sc[i] : 0.0f;
    const int per = ((n + kRankSplit - 1) / kRankSplit + 255) & ~255;       // share of j, whole tiles of 256
    const int j0 = blockIdx.y * per, j1 = min(j0 + per, n);
    int r = 0;
    for (int jb = j0; jb < j1; jb += 256) {
        __syncthreads();
        sS[threadIdx.x] = jb + (int)threadIdx.x < n ? sc[jb + threadIdx.x] : -INFINITY;
        __syncthreads();
        const int m = min(256, j1 - jb);
        for (int q = 0; q < m; ++q) {
            const float t = sS[q];
            r += (t > s || (t == s && jb + q < i)) ? 1 : 0;
        }
    }
    if (i < n && r) atomicAdd(&rank[i], r);
}

// sorted[rank[i]] = frame-pixel box of survivor i; clears rank and the neighbour counts for the next call
__global__ __launch_bounds__(256)
void merge_scatter_kernel(const uint32_t *__restrict__ idx, const float *__restrict__ sc,
                          const int32_t *__restrict__ d_n, int n_max, const LevelDev *__restrict__ levels,
                          int n_levels, int32_t *__restrict__ rank, int32_t *__restrict__ nb,
                          SortedBox *__restrict__ sorted)
{
    const int n = min(*d_n, n_max);
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int r = rank[i];
    rank[i] = 0;
    nb[i] = 0;
    const uint32_t g = idx[i];
    int l = 0;
    while (l + 1 < n_levels && g >= (uint32_t)levels[l + 1].score_off) ++l;
    const uint32_t rem = g - (uint32_t)levels[l].score_off;
    const int ow = levels[l].ow;
    const double scale = levels[l].scale;
    SortedBox b;
    b.x = round_half_up(__dmul_rn((double)(rem % ow), scale));
    b.y = round_half_up(__dmul_rn((double)(rem / ow), scale));
    b.size = round_half_up(__dmul_rn((double)kWin, scale));
    b.score = sc[i];
    b.level = l;
    b.index = (int32_t)g;
    sorted[r] = b;
}

// overlap[j][w] bit b = box j overlaps box 64 w + b beyond the threshold (j itself excluded).
// Workgroups stride over the (64-row block, word) pairs that exist for the current n.
__global__ __launch_bounds__(64)
void merge_overlap_kernel(const SortedBox *__restrict__ sorted, const int32_t *__restrict__ d_n, int n_max, float iou,
                          unsigned long long *__restrict__ overlap, int words)
{
    __shared__ SortedBox sCol[64];
    const int n = min(*d_n, n_max);
    const int nb64 = (n + 63) / 64;
    const double thr = (double)iou;
    for (int p = blockIdx.x; p < nb64 * nb64; p += gridDim.x) {
        const int j = (p / nb64) * 64 + threadIdx.x, w = p % nb64;
        const int c = w * 64 + threadIdx.x;
        __syncthreads();
        if (c < n) sCol[threadIdx.x] = sorted[c];
        __syncthreads();
        if (j < n) {
            const SortedBox a = sorted[j];
            const int m = min(64, n - w * 64);
            unsigned long long bits = 0;
            for (int b = 0; b < m; ++b)
                if (w * 64 + b != j && overlaps(a, sCol[b], thr)) bits |= 1ull << b;
            overlap[(size_t)j * words + w] = bits;
        }
    }
}

__global__ __launch_bounds__(kResolveThreads)
void merge_resolve_kernel(const SortedBox *__restrict__ sorted, const unsigned long long *__restrict__ overlap,
                          int words, const int32_t *__restrict__ d_n, int n_max, int min_neighbors,
                          int32_t *__restrict__ nb, cnnc_det *__restrict__ det, int det_cap,
                          int32_t *__restrict__ d_ndet)
{
    __shared__ unsigned long long keptS[kMergeCapMax / 64], remS[kMergeCapMax / 64];
    __shared__ int s_flag, s_wsum[kResolveThreads / 64], s_base;
    const int tid = threadIdx.x;
    const int n = min(*d_n, n_max);
    const int W = (n + 63) / 64;
    for (int w = tid; w < W; w += kResolveThreads) { keptS[w] = 0; remS[w] = 0; }
    uint32_t und = 0;                                   // bit q: box tid + 1024 q is still undecided
    for (int q = 0; q < kMergeCapMax / kResolveThreads; ++q)
        if (tid + kResolveThreads * q < n) und |= 1u << q;
    if (tid == 0) s_flag = 0;
    __syncthreads();

    for (;;) {
        uint32_t todo = und;
        while (todo) {
            const int q = __ffs(todo) - 1;
            todo &= todo - 1;
            const int j = tid + kResolveThreads * q, wj = j >> 6;
            const unsigned long long *row = overlap + (size_t)j * words;
            bool any_kept = false, all_removed = true;
            for (int w = 0; w <= wj; ++w) {
                unsigned long long p = row[w];
                if (w == wj) p &= (1ull << (j & 63)) - 1ull;
                if (p & keptS[w]) { any_kept = true; break; }
                if (p & ~remS[w]) all_removed = false;
            }
            if (any_kept) { atomicOr(&remS[wj], 1ull << (j & 63)); und &= ~(1u << q); }
            else if (all_removed) { atomicOr(&keptS[wj], 1ull << (j & 63)); und &= ~(1u << q); }
        }
        if (und) s_flag = 1;
        __syncthreads();
        const int more = s_flag;
        __syncthreads();
        if (tid == 0) s_flag = 0;
        if (!more) break;
        __syncthreads();
    }
    __syncthreads();

    // neighbours: an absorbed box counts for its first kept overlapping predecessor
    for (int j = tid; j < n; j += kResolveThreads) {
        const int wj = j >> 6;
        if (!((remS[wj] >> (j & 63)) & 1ull)) continue;
        const unsigned long long *row = overlap + (size_t)j * words;
        for (int w = 0; w <= wj; ++w) {
            unsigned long long p = row[w] & keptS[w];
            if (w == wj) p &= (1ull << (j & 63)) - 1ull;
            if (p) { atomicAdd(&nb[w * 64 + __ffsll((long long)p) - 1], 1); break; }
        }
    }
    __threadfence();
    if (tid == 0) s_base = 0;
    __syncthreads();

    // ordered output of the kept boxes that have enough neighbours
    const int lane = tid & 63, wave = tid >> 6;
    for (int j0 = 0; j0 < n; j0 += kResolveThreads) {
        const int j = j0 + tid;
        int cnt = 0;
        bool out = false;
        if (j < n && ((keptS[j >> 6] >> (j & 63)) & 1ull)) {
            cnt = __atomic_load_n(&nb[j], __ATOMIC_RELAXED);
            out = cnt + 1 >= min_neighbors;
        }
        const unsigned long long ball = __ballot(out);
        if (lane == 0) s_wsum[wave] = __popcll(ball);
        __syncthreads();
        int pos = s_base;
        for (int w = 0; w < wave; ++w) pos += s_wsum[w];
        pos += __popcll(ball & ((1ull << lane) - 1ull));
        if (out && pos < det_cap) {
            const SortedBox b = sorted[j];
            cnnc_det d;
            d.x = b.x; d.y = b.y; d.size = b.size; d.score = b.score;
            d.level = b.level; d.neighbors = cnt; d.index = b.index; d.reserved = 0;
            det[pos] = d;
        }
        __syncthreads();
        if (tid == 0) {
            int tot = 0;
            for (int w = 0; w < kResolveThreads / 64; ++w) tot += s_wsum[w];
            s_base += tot;
        }
        __syncthreads();
    }
    if (tid == 0) *d_ndet = s_base;
}

hipError_t merge_init_workspace(const cnnc_ctx *c)
{
    const MergeWs w = carve(c->d_merge_ws, c->merge_cap);
    return hipMemset(w.rank, 0, sizeof(int32_t) * (size_t)c->merge_cap);
}

hipError_t launch_merge(const cnnc_ctx *c, hipStream_t st)
{
    const MergeWs w = carve(c->d_merge_ws, c->merge_cap);
    const int cap = c->merge_cap;
    const int32_t *d_n = &c->d_cnt->n[2];
    hipLaunchKernelGGL(merge_rank_kernel, dim3((cap + 255) / 256, kRankSplit), dim3(256), 0, st, c->d_sc[2], d_n, cap, w.rank);
    hipLaunchKernelGGL(merge_scatter_kernel, dim3((cap + 255) / 256), dim3(256), 0, st, c->d_idx[2], c->d_sc[2], d_n, cap,
                       c->d_levels, c->n_levels, w.rank, w.nb, w.sorted);
    const int pairs = ((cap + 63) / 64) * ((cap + 63) / 64);
    hipLaunchKernelGGL(merge_overlap_kernel, dim3(pairs < 4096 ? pairs : 4096), dim3(64), 0, st, w.sorted, d_n, cap,
                       c->params.merge_iou, w.overlap, w.words);
    hipLaunchKernelGGL(merge_resolve_kernel, dim3(1), dim3(kResolveThreads), 0, st, w.sorted, w.overlap, w.words, d_n, cap,
                       c->params.min_neighbors, w.nb, c->d_det, cap, &c->d_cnt->n[3]);
    return hipGetLastError();
}

}  // namespace cnnc
