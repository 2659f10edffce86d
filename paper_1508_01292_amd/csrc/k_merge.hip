// Merging of the windows accepted by the last stage (paper, Section 3.3, last paragraph:
// non-maximum suppression aggregates the found regions; Section 4.2: minNeighbors).
// Greedy rule: in order of descending score (ties: ascending flat window index) a box not yet
// absorbed is kept and absorbs every later box whose intersection exceeds merge_iou * union.
//
// The greedy rule is sequential as stated; here it is evaluated in parallel in a way that gives the same
// result.  With O the symmetric "overlaps more than the threshold" relation of the sorted boxes, a box is
// KEPT once all earlier boxes overlapping it are known to be absorbed, and ABSORBED once one earlier
// overlapping box is known to be kept.  The sorted list is taken in chunks of 1024 boxes, one per thread of a
// single workgroup.  When a chunk starts every earlier chunk is final, so the chunk first looks for kept boxes
// among the overlapping predecessors that lie in earlier chunks: the overlap kernel leaves them as one flat
// array of (row, predecessor) pairs per chunk, which the threads share out evenly whatever the spread of pairs
// over the rows (the bit rows themselves when a chunk has more pairs than the array holds).  What is left
// depends on boxes of the same chunk only: the 16 words
// of the chunk's diagonal block of the bit matrix sit in registers, the chunk's kept / absorbed bits in LDS,
// and rounds repeat until no box of the chunk is undecided (the earliest undecided one is decided in every
// round).  The neighbour count of a kept box is the number of absorbed boxes whose FIRST kept overlapping
// predecessor it is, which is what the sequential pass counts.
//
// Launches: rank (counting sort position of every box, n^2 comparisons spread over the chip), scatter into
// sorted order as frame-pixel boxes, overlap bits (lower triangle) + predecessor lists, and the chunks +
// ordered output in one workgroup.
#include <climits>

#include "cnnc_internal.h"

namespace cnnc {

namespace {
constexpr int kMergeCapMax = 32768;
constexpr int kResolveThreads = 1024;
constexpr int kRankSplit = 8;
constexpr int kChunk = kResolveThreads;          // boxes decided together
constexpr int kChunkWords = kChunk / 64;
constexpr int kMaxChunks = kMergeCapMax / kChunk;
constexpr int kPairCap = 128 * 1024;             // (row, predecessor in an earlier chunk) pairs held per chunk

struct SortedBox {
    int32_t x, y, w, h;
    float score;
    int32_t level, index, pad;
};

struct MergeWs {
    SortedBox *sorted;
    int32_t *rank;     // zero between calls
    int32_t *nb;
    int32_t *npair;                 // [kMaxChunks] pairs of each chunk (may exceed kPairCap); zero between calls
    uint32_t *pairs;                // [chunks of cap][kPairCap] row inside the chunk << 16 | predecessor, in no order
    unsigned long long *overlap;   // [words][cap]: word w of row j at w * cap + j, for the words up to the row's own
};

__host__ __device__ inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

inline MergeWs carve(void *base, int cap)
{
    MergeWs w;
    char *p = static_cast<char *>(base);
    w.sorted = reinterpret_cast<SortedBox *>(p); p += align256(sizeof(SortedBox) * (size_t)cap);
    w.rank = reinterpret_cast<int32_t *>(p); p += align256(sizeof(int32_t) * (size_t)cap);
    w.nb = reinterpret_cast<int32_t *>(p); p += align256(sizeof(int32_t) * (size_t)cap);
    w.npair = reinterpret_cast<int32_t *>(p); p += align256(sizeof(int32_t) * kMaxChunks);
    w.pairs = reinterpret_cast<uint32_t *>(p); p += align256(sizeof(uint32_t) * (size_t)((cap + kChunk - 1) / kChunk) * kPairCap);
    w.overlap = reinterpret_cast<unsigned long long *>(p);
    return w;
}

__device__ __forceinline__ int32_t round_half_up(double v) { return (int32_t)floor(__dadd_rn(v, 0.5)); }

// Frames are at most 16384 pixels a side, so a box area stays below 2^29 and a union below 2^30.
struct Rect { int32_t x0, y0, x1, y1; };

__device__ __forceinline__ Rect rect_of(const SortedBox &b) { return {b.x, b.y, b.x + b.w, b.y + b.h}; }

__device__ __forceinline__ bool overlaps(const Rect &a, const Rect &b, double thr)
{
    const int32_t iw = min(a.x1, b.x1) - max(a.x0, b.x0), ih = min(a.y1, b.y1) - max(a.y0, b.y0);
    if (iw <= 0 || ih <= 0) return false;
    const int32_t inter = iw * ih, uni = (a.x1 - a.x0) * (a.y1 - a.y0) + (b.x1 - b.x0) * (b.y1 - b.y0) - inter;
    return (double)inter > __dmul_rn(thr, (double)uni);   // exact: 24-bit threshold times an integer below 2^30
}
}  // namespace

size_t merge_workspace_bytes(int cap)
{
    return align256(sizeof(SortedBox) * (size_t)cap) + 2 * align256(sizeof(int32_t) * (size_t)cap) +
           align256(sizeof(int32_t) * kMaxChunks) + align256(sizeof(uint32_t) * (size_t)((cap + kChunk - 1) / kChunk) * kPairCap) +
           sizeof(unsigned long long) * (size_t)cap * ((cap + 63) / 64);
}

// rank[i] += number of boxes in this block's share of j that sort before box i
__global__ __launch_bounds__(256)
void merge_rank_kernel(const float *__restrict__ sc, const int32_t *__restrict__ d_n, int n_max, int32_t *__restrict__ rank)
{
    __shared__ __attribute__((aligned(16))) float sS[256];
    const int n = min(*d_n, n_max);
    if ((int)blockIdx.x * 256 >= n) return;
    const int i = blockIdx.x * 256 + threadIdx.x;
    const float s = i < n ? sc[i] : 0.0f;
    const int per = ((n + kRankSplit - 1) / kRankSplit + 255) & ~255;       // share of j, whole tiles of 256
    const int j0 = blockIdx.y * per, j1 = min(j0 + per, n);
    int r = 0;
    for (int jb = j0; jb < j1; jb += 256) {
        __syncthreads();
        sS[threadIdx.x] = jb + (int)threadIdx.x < n ? sc[jb + threadIdx.x] : -INFINITY;   // the padding sorts after all
        __syncthreads();
        const int ties = i - jb;                                  // entries q < ties of this tile win a tie with box i
#pragma unroll 4
        for (int q = 0; q < 256; q += 4) {
            const float4 t = *reinterpret_cast<const float4 *>(&sS[q]);
            r += (t.x > s || (t.x == s && q + 0 < ties)) ? 1 : 0;
            r += (t.y > s || (t.y == s && q + 1 < ties)) ? 1 : 0;
            r += (t.z > s || (t.z == s && q + 2 < ties)) ? 1 : 0;
            r += (t.w > s || (t.w == s && q + 3 < ties)) ? 1 : 0;
        }
    }
    if (i < n && r) atomicAdd(&rank[i], r);
}

// sorted[rank[i]] = frame-pixel box of survivor i; clears rank and the neighbour counts for the next call
__global__ __launch_bounds__(256)
void merge_scatter_kernel(const uint32_t *__restrict__ idx, const float *__restrict__ sc,
                          const int32_t *__restrict__ d_n, int n_max, const LevelDev *__restrict__ levels,
                          int n_levels, int32_t *__restrict__ rank, int32_t *__restrict__ nb,
                          int32_t *__restrict__ npair, SortedBox *__restrict__ sorted)
{
    const int n = min(*d_n, n_max);
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < kMaxChunks) npair[i] = 0;
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
    b.w = b.h = round_half_up(__dmul_rn((double)kWin, scale));
    b.score = sc[i];
    b.level = l;
    b.index = (int32_t)g;
    b.pad = 0;
    sorted[r] = b;
}

// ---- the regions the selective unit accepted (paper, Section 3.3: non-maximum suppression aggregates the found
// regions).  A region enters as its 27 x 31 window in frame pixels with the largest combined CNN_3 response as score.
// One workgroup lists them in ascending position order.
__global__ __launch_bounds__(kResolveThreads)
void merge_pick_faces_kernel(const cnnc_region *__restrict__ rec, const float *__restrict__ maps3,
                             const int32_t *__restrict__ d_nreg, int reg_max, int cap, float *__restrict__ sc,
                             uint32_t *__restrict__ pick, int32_t *__restrict__ d_nface)
{
    __shared__ int s_wsum[kResolveThreads / 64], s_base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = min(*d_nreg, reg_max);
    if (tid == 0) s_base = 0;
    __syncthreads();
    for (int i0 = 0; i0 < n; i0 += kResolveThreads) {
        const int i = i0 + tid;
        const bool f = i < n && rec[i].face != 0;
        const unsigned long long ball = __ballot(f);
        if (lane == 0) s_wsum[wave] = __popcll(ball);
        __syncthreads();
        int pos = s_base;
        for (int w = 0; w < wave; ++w) pos += s_wsum[w];
        pos += __popcll(ball & ((1ull << lane) - 1ull));
        if (f && pos < cap) {
            const float *m = maps3 + (size_t)i * 25;
            float best = m[0];
            for (int k = 1; k < 25; ++k) best = fmaxf(best, m[k]);
            sc[pos] = best;
            pick[pos] = (uint32_t)i;
        }
        __syncthreads();
        if (tid == 0) {
            int tot = 0;
            for (int w = 0; w < kResolveThreads / 64; ++w) tot += s_wsum[w];
            s_base += tot;
        }
        __syncthreads();
    }
    if (tid == 0) *d_nface = s_base;
}

// sorted[rank[i]] = frame-pixel rectangle of accepted region i; clears rank and the counters for the next call
__global__ __launch_bounds__(256)
void merge_scatter_rect_kernel(const cnnc_region *__restrict__ rec, const uint32_t *__restrict__ pick,
                               const float *__restrict__ sc, const int32_t *__restrict__ d_n, int n_max,
                               const LevelDev *__restrict__ levels, int32_t *__restrict__ rank, int32_t *__restrict__ nb,
                               int32_t *__restrict__ npair, SortedBox *__restrict__ sorted)
{
    const int n = min(*d_n, n_max);
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < kMaxChunks) npair[i] = 0;
    if (i >= n) return;
    const int r = rank[i];
    rank[i] = 0;
    nb[i] = 0;
    const cnnc_region g = rec[pick[i]];
    const double scale = levels[g.level].scale;
    SortedBox b;
    b.x = round_half_up(__dmul_rn((double)(kScanStep * g.i), scale));
    b.y = round_half_up(__dmul_rn((double)(kScanStep * g.j), scale));
    b.w = round_half_up(__dmul_rn((double)kScanWinW, scale));
    b.h = round_half_up(__dmul_rn((double)kScanWinH, scale));
    b.score = sc[i];
    b.level = g.level;
    b.index = g.index;
    b.pad = 0;
    sorted[r] = b;
}

// Word w of row j (at overlap[w * n_max + j]), bit b: box j overlaps box 64 w + b beyond the threshold (j itself
// excluded), for the words up to the one that holds j.  Overlapping boxes of earlier chunks are also appended to
// the pair array of the row's chunk.
// A work item is a block of 64 rows times a group of G consecutive words, G = 1, 4 or 16 (a whole chunk of
// columns) growing with n: its pairs take one reservation in the chunk's array, so that long lists do not queue
// on the chunk's counter, while short lists still spread over the chip.  Workgroups (one wave each) stride
// over the items.
__global__ __launch_bounds__(64)
void merge_overlap_kernel(const SortedBox *__restrict__ sorted, const int32_t *__restrict__ d_n, int n_max, float iou,
                          unsigned long long *__restrict__ overlap, int32_t *__restrict__ npair,
                          uint32_t *__restrict__ pairs)
{
    __shared__ Rect sCol[64];
    const int n = min(*d_n, n_max);
    const int nb64 = (n + 63) / 64;
    const int G = n <= 2048 ? 1 : (n <= 8192 ? 4 : kChunkWords);
    const int lane = threadIdx.x;
    const double thr = (double)iou;
    // Row block rb has rb / G + 1 groups.  The items are numbered row block by row block: the G row blocks
    // q G .. q G + G - 1 have q + 1 groups each and start at item G q (q + 1) / 2.
    const int qn = (nb64 + G - 1) / G;                            // number of such sets of row blocks, the last may be short
    const int n_items = G * (qn - 1) * qn / 2 + (nb64 - (qn - 1) * G) * qn;
    for (int p = blockIdx.x; p < n_items; p += gridDim.x) {
        int q = (int)((sqrtf(8.0f * (float)p / (float)G + 1.0f) - 1.0f) * 0.5f);
        while (G * q * (q + 1) / 2 > p) --q;
        while (G * (q + 1) * (q + 2) / 2 <= p) ++q;
        const int r = p - G * q * (q + 1) / 2;
        const int rb = q * G + r / (q + 1), g0 = (r % (q + 1)) * G;
        const int j = rb * 64 + lane;
        Rect a = {0, 0, 0, 0};
        if (j < n) {
            a = rect_of(sorted[j]);
        }
        // column box of this lane in word w; beyond the list an empty box, which overlaps nothing
        auto column = [&](int w) -> Rect {
            const int c = w * 64 + lane;
            if (c >= n) return {0, 0, 0, 0};
            return rect_of(sorted[c]);
        };
        unsigned long long bits[kChunkWords];
        int cnt = 0;
        Rect next = column(g0);
#pragma unroll
        for (int g = 0; g < kChunkWords; ++g) {
            bits[g] = 0;
            const int w = g0 + g;
            if (g >= G || w > rb) continue;                       // uniform
            const Rect col = next;
            if (g + 1 < G && w + 1 <= rb) next = column(w + 1);   // in flight during this word's comparisons
            __syncthreads();
            sCol[lane] = col;
            __syncthreads();
            if (j < n) {
                unsigned long long v = 0;
                for (int b = 0; b < 64; b += 8) {                // eight column boxes read together, then compared
                    Rect r[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) r[u] = sCol[b + u];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (overlaps(a, r[u], thr)) v |= 1ull << (b + u);
                }
                if (w == rb) v &= ~(1ull << lane);
                overlap[(size_t)w * n_max + j] = v;
                bits[g] = v;
                cnt += __popcll(v);
            }
        }
        const int chunk = rb / kChunkWords;
        if (g0 / kChunkWords < chunk && __ballot(cnt != 0)) {
            int incl = cnt;                                       // inclusive prefix sum over the wave
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(incl, o);
                if (lane >= o) incl += t;
            }
            int base = 0;
            if (lane == 63) base = atomicAdd(&npair[chunk], incl);
            base = __shfl(base, 63);
            uint32_t *out = pairs + (size_t)chunk * kPairCap;
            const uint32_t row = (uint32_t)(j & (kChunk - 1)) << 16;
            int pos = base + incl - cnt;
#pragma unroll
            for (int g = 0; g < kChunkWords; ++g)
                for (unsigned long long v = bits[g]; v && pos < kPairCap; v &= v - 1ull, ++pos)
                    out[pos] = row | (uint32_t)((g0 + g) * 64 + __ffsll((long long)v) - 1);
        }
    }
}

template <typename DET> __device__ __forceinline__ DET make_det(const SortedBox &b, int neighbors);
template <> __device__ __forceinline__ cnnc_det make_det<cnnc_det>(const SortedBox &b, int neighbors)
{
    cnnc_det d;
    d.x = b.x; d.y = b.y; d.size = b.w; d.score = b.score;
    d.level = b.level; d.neighbors = neighbors; d.index = b.index; d.reserved = 0;
    return d;
}
template <> __device__ __forceinline__ cnnc_rdet make_det<cnnc_rdet>(const SortedBox &b, int neighbors)
{
    cnnc_rdet d;
    d.x = b.x; d.y = b.y; d.w = b.w; d.h = b.h; d.score = b.score;
    d.level = b.level; d.neighbors = neighbors; d.index = b.index;
    return d;
}

// DET = cnnc_det (square windows of the cascade) or cnnc_rdet (rectangles of the selective unit)
template <typename DET>
__global__ __launch_bounds__(kResolveThreads)
void merge_resolve_kernel(const SortedBox *__restrict__ sorted, const unsigned long long *__restrict__ overlap,
                          const int32_t *__restrict__ npair, const uint32_t *__restrict__ pairs,
                          const int32_t *__restrict__ d_n, int n_max, int min_neighbors,
                          int32_t *__restrict__ nb, DET *__restrict__ det, int det_cap,
                          int32_t *__restrict__ d_ndet)
{
    __shared__ unsigned long long keptS[kMergeCapMax / 64], remC[kChunkWords];
    __shared__ int firstS[kChunk], s_npair[kMaxChunks];
    __shared__ int s_wsum[kResolveThreads / 64], s_base;
    const int tid = threadIdx.x;
    const int n = min(*d_n, n_max);
    for (int w = tid; w < kMergeCapMax / 64; w += kResolveThreads) keptS[w] = 0;
    if (tid < kMaxChunks) s_npair[tid] = npair[tid];
    const int tw = tid >> 6;                                      // word of this thread's box inside its chunk
    const unsigned long long tbit = 1ull << (tid & 63);

    for (int c0 = 0; c0 < n; c0 += kChunk) {
        const int j = c0 + tid, w0 = c0 >> 6;
        const bool live = j < n;
        __syncthreads();                                          // keptS of the earlier chunks is final (or cleared)
        if (tid < kChunkWords) remC[tid] = 0;
        firstS[tid] = INT_MAX;

        // this box's words of the chunk's diagonal block, bits of earlier boxes only
        unsigned long long d[kChunkWords];
#pragma unroll
        for (int k = 0; k < kChunkWords; ++k) d[k] = 0;
        if (live) {
#pragma unroll
            for (int k = 0; k < kChunkWords; ++k)
                if (k <= tw) d[k] = overlap[(size_t)(w0 + k) * n_max + j];
#pragma unroll
            for (int k = 0; k < kChunkWords; ++k)
                if (k == tw) d[k] &= tbit - 1ull;
        }
        __syncthreads();

        // kept predecessors in earlier chunks: the lowest one of every row, or none
        const int np = c0 ? s_npair[c0 / kChunk] : 0;
        int first = INT_MAX;
        if (np <= kPairCap) {
            const uint32_t *pp = pairs + (size_t)(c0 / kChunk) * kPairCap;
            for (int t0 = tid; t0 < np; t0 += 8 * kResolveThreads) {       // eight loads of a thread in flight together
                uint32_t pr[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int t = t0 + u * kResolveThreads;
                    pr[u] = t < np ? pp[t] : 0xFFFFFFFFu;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = (int)(pr[u] & 0xFFFFu), r = (int)(pr[u] >> 16);
                    if (pr[u] != 0xFFFFFFFFu && ((keptS[e >> 6] >> (e & 63)) & 1ull)) atomicMin(&firstS[r], e);
                }
            }
        } else {
            // more pairs than the array holds: every wave reads the bit rows of its boxes, 64 words of a row a step
            for (int src = 0; src < 64 && c0 + (tid & ~63) + src < n; ++src) {
                const unsigned long long *row = overlap + (c0 + (tid & ~63) + src);
                int lowest = INT_MAX;
                for (int w = w0 - 1 - (tid & 63); w >= 0; w -= 64) {
                    const unsigned long long p = row[(size_t)w * n_max] & keptS[w];
                    if (p) lowest = w * 64 + __ffsll((long long)p) - 1;
                }
#pragma unroll
                for (int o = 32; o; o >>= 1) lowest = min(lowest, __shfl_xor(lowest, o));
                if ((tid & 63) == src) first = lowest;
            }
        }
        __syncthreads();
        first = min(first, firstS[tid]);
        bool und = live && first == INT_MAX;
        if (live && !und) atomicOr(&remC[tw], tbit);

        // Rounds inside the chunk.  A wave repeats its step while one of its boxes gets decided: what its own
        // lanes wrote to LDS is visible to its next read, so chains inside a 64-box word need no barrier; the
        // barrier rounds only carry decisions from one wave to another.
        for (;;) {
            __syncthreads();
            bool progress;
            do {
                asm volatile("" ::: "memory");                    // read the LDS words again
                progress = false;
                if (und) {
                    bool any_kept = false, all_removed = true;
#pragma unroll
                    for (int k = 0; k < kChunkWords; ++k) {
                        if (d[k] & keptS[w0 + k]) any_kept = true;
                        if (d[k] & ~remC[k]) all_removed = false;
                    }
                    if (any_kept) { atomicOr(&remC[tw], tbit); und = false; progress = true; }
                    else if (all_removed) { atomicOr(&keptS[w0 + tw], tbit); und = false; progress = true; }
                }
            } while (__ballot(progress));
            if (!__syncthreads_or(und)) break;
        }

        // an absorbed box counts for its first kept overlapping predecessor
        if (live && !((keptS[w0 + tw] >> (tid & 63)) & 1ull)) {
            if (first == INT_MAX) {
#pragma unroll
                for (int k = kChunkWords - 1; k >= 0; --k) {
                    const unsigned long long p = d[k] & keptS[w0 + k];
                    if (p) first = (w0 + k) * 64 + __ffsll((long long)p) - 1;
                }
            }
            atomicAdd(&nb[first], 1);
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
            det[pos] = make_det<DET>(sorted[j], cnt);
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
    hipError_t e = hipMemset(w.rank, 0, sizeof(int32_t) * (size_t)c->merge_cap);
    if (e == hipSuccess) e = hipMemset(w.npair, 0, sizeof(int32_t) * kMaxChunks);
    return e;
}

namespace {
template <typename DET>
void launch_overlap_resolve(const cnnc_ctx *c, const MergeWs &w, const int32_t *d_n, float iou, int min_neighbors,
                            DET *det, int32_t *d_ndet, hipStream_t st)
{
    const int cap = c->merge_cap;
    const int tiles = ((cap + 63) / 64) * ((cap + 63) / 64);
    hipLaunchKernelGGL(merge_overlap_kernel, dim3(tiles < 4096 ? tiles : 4096), dim3(64), 0, st, w.sorted, d_n, cap,
                       iou, w.overlap, w.npair, w.pairs);
    hipLaunchKernelGGL(merge_resolve_kernel<DET>, dim3(1), dim3(kResolveThreads), 0, st, w.sorted, w.overlap, w.npair, w.pairs,
                       d_n, cap, min_neighbors, w.nb, det, cap, d_ndet);
}
}  // namespace

hipError_t launch_merge(const cnnc_ctx *c, hipStream_t st)
{
    const MergeWs w = carve(c->d_merge_ws, c->merge_cap);
    const int cap = c->merge_cap;
    const int32_t *d_n = &c->d_cnt->n[2];
    hipLaunchKernelGGL(merge_rank_kernel, dim3((cap + 255) / 256, kRankSplit), dim3(256), 0, st, c->d_sc[2], d_n, cap, w.rank);
    hipLaunchKernelGGL(merge_scatter_kernel, dim3((cap + 255) / 256), dim3(256), 0, st, c->d_idx[2], c->d_sc[2], d_n, cap,
                       c->d_levels, c->n_levels, w.rank, w.nb, w.npair, w.sorted);
    launch_overlap_resolve<cnnc_det>(c, w, d_n, c->params.merge_iou, c->params.min_neighbors, c->d_det, &c->d_cnt->n[3], st);
    return hipGetLastError();
}

// Accepted regions of the last selective-unit pass -> d_sel_det, counts in d_sel_cnt[1] (accepted) and [2] (merged).
hipError_t launch_merge_regions(const cnnc_ctx *c, float iou, int min_neighbors, hipStream_t st)
{
    const MergeWs w = carve(c->d_merge_ws, c->merge_cap);
    const int cap = c->merge_cap;
    const int32_t *d_n = &c->d_sel_cnt[1];
    hipLaunchKernelGGL(merge_pick_faces_kernel, dim3(1), dim3(kResolveThreads), 0, st, c->d_sel_rec,
                       c->d_sel_maps + (size_t)25 * c->max_surv, &c->d_sel_cnt[0], c->max_surv, cap, c->d_sel_fsc,
                       c->d_sel_pick, &c->d_sel_cnt[1]);
    hipLaunchKernelGGL(merge_rank_kernel, dim3((cap + 255) / 256, kRankSplit), dim3(256), 0, st, c->d_sel_fsc, d_n, cap, w.rank);
    hipLaunchKernelGGL(merge_scatter_rect_kernel, dim3((cap + 255) / 256), dim3(256), 0, st, c->d_sel_rec, c->d_sel_pick,
                       c->d_sel_fsc, d_n, cap, c->d_levels, w.rank, w.nb, w.npair, w.sorted);
    launch_overlap_resolve<cnnc_rdet>(c, w, d_n, iou, min_neighbors, c->d_sel_det, &c->d_sel_cnt[2], st);
    return hipGetLastError();
}

}  // namespace cnnc
