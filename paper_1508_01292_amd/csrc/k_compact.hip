// Survivor compaction (paper, Section 3.3: the coordinates of the windows whose response exceeded
// the threshold are handed on).  Deterministic: the output keeps ascending input order, so no
// atomics on the output position.  Two small launches: per-workgroup counts, and the scatter, in
// which every workgroup first adds up the counts of the workgroups before it (a separate scan
// launch takes over for very long inputs); inside a workgroup each wave owns a contiguous run of
// the input and ranks its survivors with ballots.
#include <mutex>

#include "cnnc_internal.h"

namespace cnnc {

namespace {
constexpr int kWaves = kCompactBlock / 64;
constexpr int kPerWave = kCompactPerBlock / kWaves;   // contiguous values per wave
constexpr int kIters = kPerWave / 64;

// The part of the source this call covers: elements [begin, begin + n).  With device counters (d_end != nullptr) it
// is the list range [*d_begin, *d_end) clamped to the list's capacity n_max; otherwise the first n_literal values.
struct SourceRange { int64_t begin, n; };
__device__ __forceinline__ SourceRange source_range(const int32_t *d_begin, const int32_t *d_end, int64_t n_literal, int64_t n_max)
{
    if (d_end == nullptr) return {0, n_literal};
    const int64_t b = d_begin ? min((int64_t)*d_begin, n_max) : 0, e = min((int64_t)*d_end, n_max);
    return {b, e > b ? e - b : 0};
}
}  // namespace

__global__ __launch_bounds__(kCompactBlock)
void compact_count_kernel(const float *__restrict__ vals, const int32_t *__restrict__ d_begin,
                          const int32_t *__restrict__ d_end, int64_t n_literal, int64_t n_max, float thr,
                          int32_t *__restrict__ blockcnt)
{
    __shared__ int wsum[kWaves];
    const SourceRange R = source_range(d_begin, d_end, n_literal, n_max);
    const int64_t n = R.n;
    vals += R.begin;
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int64_t base = (int64_t)blockIdx.x * kCompactPerBlock + (int64_t)wave * kPerWave;
    int cnt = 0;
    for (int it = 0; it < kIters; ++it) {
        const int64_t e = base + it * 64 + lane;
        const bool pass = e < n && vals[e] > thr;
        cnt += __popcll(__ballot(pass));
    }
    if (lane == 0) wsum[wave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        int s = 0;
        for (int w = 0; w < kWaves; ++w) s += wsum[w];
        blockcnt[blockIdx.x] = s;
    }
}

// Exclusive scan of the per-workgroup counts (one workgroup, chunks of 1024 with a carry) and the
// total, plus the entries already in the output list (*d_base, if given), into *d_count (and *d_count2).
__global__ __launch_bounds__(1024)
void compact_scan_kernel(int32_t *__restrict__ blockcnt, int nblocks, const int32_t *__restrict__ d_base,
                         int32_t *__restrict__ d_count, int32_t *__restrict__ d_count2)
{
    __shared__ int wtot[16];
    __shared__ int carry_s;
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int base = 0; base < nblocks; base += 1024) {
        const int i = base + threadIdx.x;
        const int v = i < nblocks ? blockcnt[i] : 0;
        int incl = v;
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(incl, d, 64);
            if (lane >= d) incl += o;
        }
        if (lane == 63) wtot[wave] = incl;
        __syncthreads();
        int woff = 0, total = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < wave) woff += wtot[w];
            total += wtot[w];
        }
        const int carry = carry_s;
        if (i < nblocks) blockcnt[i] = carry + woff + incl - v;
        __syncthreads();
        if (threadIdx.x == 0) carry_s = carry + total;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const int total = carry_s + (d_base ? *d_base : 0);
        *d_count = total;
        if (d_count2) *d_count2 = total;
    }
}

__global__ __launch_bounds__(kCompactBlock)
void compact_scatter_kernel(const float *__restrict__ vals, const uint32_t *__restrict__ src_idx, uint32_t idx_base,
                            const int32_t *__restrict__ d_begin, const int32_t *__restrict__ d_end, int64_t n_literal,
                            int64_t n_max, float thr, const int32_t *__restrict__ blockoff,
                            uint32_t *__restrict__ out_idx, float *__restrict__ out_sc, int cap,
                            const int32_t *__restrict__ d_base, int32_t *__restrict__ d_count_if_unscanned,
                            int32_t *__restrict__ d_count2)
{
    __shared__ int wsum[kWaves], wpre[kWaves];
    const SourceRange R = source_range(d_begin, d_end, n_literal, n_max);
    const int64_t n = R.n;
    vals += R.begin;
    if (src_idx) src_idx += R.begin;
    const int base_out = d_base ? *d_base : 0;       // entries already in the output list (appending a later chunk)
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int64_t base = (int64_t)blockIdx.x * kCompactPerBlock + (int64_t)wave * kPerWave;
    float v[kIters];
    uint64_t mask[kIters];
    int cnt = 0;
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const int64_t e = base + it * 64 + lane;
        v[it] = e < n ? vals[e] : 0.0f;
        mask[it] = __ballot(e < n && v[it] > thr);
        cnt += __popcll(mask[it]);
    }
    int pos;
    if (d_count_if_unscanned) {
        // blockoff holds the raw counts of the workgroups: this one sums those before it (a few KB from L2), and
        // the last one also leaves the total
        int before = 0;
        for (int b = threadIdx.x; b < (int)blockIdx.x; b += kCompactBlock) before += blockoff[b];
        for (int d = 32; d >= 1; d >>= 1) before += __shfl_xor(before, d, 64);
        if (lane == 0) { wsum[wave] = cnt; wpre[wave] = before; }
        __syncthreads();
        pos = 0;
        int own = 0;
        for (int w = 0; w < kWaves; ++w) { pos += wpre[w]; own += wsum[w]; }
        if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
            *d_count_if_unscanned = base_out + pos + own;
            if (d_count2) *d_count2 = base_out + pos + own;
        }
    } else {
        if (lane == 0) wsum[wave] = cnt;
        __syncthreads();
        pos = blockoff[blockIdx.x];
    }
    for (int w = 0; w < wave; ++w) pos += wsum[w];
    pos += base_out;
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const uint64_t m = mask[it];
        if ((m >> lane) & 1ull) {
            const int p = pos + __popcll(m & ((1ull << lane) - 1ull));
            if (p < cap) {
                const int64_t e = base + it * 64 + lane;
                out_idx[p] = src_idx ? src_idx[e] : idx_base + (uint32_t)e;
                out_sc[p] = v[it];
            }
        }
        pos += __popcll(m);
    }
}

// ---- the same list from the bit mask the fused stage-1 kernel leaves: one thread per mask word ------------
__global__ __launch_bounds__(kCompactBlock)
void mask_count_kernel(const uint32_t *__restrict__ mask, int n_words, int32_t *__restrict__ blockcnt)
{
    __shared__ int wsum[kWaves];
    const int w = blockIdx.x * kCompactBlock + threadIdx.x;
    int cnt = w < n_words ? __popc(mask[w]) : 0;
    for (int d = 32; d >= 1; d >>= 1) cnt += __shfl_xor(cnt, d, 64);
    if (threadIdx.x % 64 == 0) wsum[threadIdx.x / 64] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        int s = 0;
        for (int k = 0; k < kWaves; ++k) s += wsum[k];
        blockcnt[blockIdx.x] = s;
    }
}

__global__ __launch_bounds__(kCompactBlock)
void mask_scatter_kernel(const uint32_t *__restrict__ mask, int n_words, const float *__restrict__ score,
                         const LevelDev *__restrict__ levels, int n_levels, const int32_t *__restrict__ blockoff,
                         uint32_t *__restrict__ out_idx, float *__restrict__ out_sc, int cap)
{
    __shared__ int wsum[kWaves];
    const int w = blockIdx.x * kCompactBlock + threadIdx.x, wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    uint32_t m = w < n_words ? mask[w] : 0u;
    const int cnt = __popc(m);
    int incl = cnt;
    for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int pos = blockoff[blockIdx.x] + incl - cnt;
    for (int k = 0; k < wave; ++k) pos += wsum[k];
    if (m == 0u) return;
    // word -> first window of its 32-window run: level, row, run within the row
    int l = 0;
    while (l + 1 < n_levels && w >= levels[l + 1].word_off) ++l;
    const int rel = w - levels[l].word_off, wpr = levels[l].words_per_row;
    const uint32_t g0 = (uint32_t)levels[l].score_off + (uint32_t)(rel / wpr) * (uint32_t)levels[l].ow + 32u * (uint32_t)(rel % wpr);
    while (m) {
        const int b = __ffs(m) - 1;
        m &= m - 1;
        if (pos < cap) {
            out_idx[pos] = g0 + b;
            out_sc[pos] = score[g0 + b];
        }
        ++pos;
    }
}

hipError_t launch_compact_mask(const cnnc_ctx *c, uint32_t *out_idx, float *out_sc, int32_t *d_count, hipStream_t st)
{
    const int n_words = (int)c->n_words;
    const int nblocks = (n_words + kCompactBlock - 1) / kCompactBlock;
    hipLaunchKernelGGL(mask_count_kernel, dim3(nblocks), dim3(kCompactBlock), 0, st, c->d_mask1, n_words, c->d_blockcnt[0]);
    hipLaunchKernelGGL(compact_scan_kernel, dim3(1), dim3(1024), 0, st, c->d_blockcnt[0], nblocks, (const int32_t *)nullptr,
                       d_count, (int32_t *)nullptr);
    hipLaunchKernelGGL(mask_scatter_kernel, dim3(nblocks), dim3(kCompactBlock), 0, st, c->d_mask1, n_words, c->d_score1,
                       c->d_levels, c->n_levels, c->d_blockcnt[0], out_idx, out_sc, c->max_surv);
    return hipGetLastError();
}

hipError_t launch_compact(const cnnc_ctx *c, const CompactJob &job, hipStream_t st)
{
    const int64_t n_max = job.d_end ? (int64_t)c->max_surv : job.n_literal;
    int nblocks = (int)((n_max + kCompactPerBlock - 1) / kCompactPerBlock);
    if (nblocks < 1) nblocks = 1;   // an empty input still has to write a zero count
    int32_t *blockcnt = c->d_blockcnt[job.slot];
    hipLaunchKernelGGL(compact_count_kernel, dim3(nblocks), dim3(kCompactBlock), 0, st, job.vals, job.d_begin, job.d_end,
                       job.n_literal, n_max, job.thr, blockcnt);
    // Up to a few thousand workgroups each scatter workgroup adds up the counts before it by itself, which saves
    // the launch of the scan in between; beyond that the scan kernel is cheaper than the repeated sums.
    const bool scan_in_scatter = nblocks <= 4096;
    if (!scan_in_scatter)
        hipLaunchKernelGGL(compact_scan_kernel, dim3(1), dim3(1024), 0, st, blockcnt, nblocks, job.d_base, job.d_count, job.d_count2);
    hipLaunchKernelGGL(compact_scatter_kernel, dim3(nblocks), dim3(kCompactBlock), 0, st, job.vals, job.src_idx, job.idx_base,
                       job.d_begin, job.d_end, job.n_literal, n_max, job.thr, blockcnt, job.out_idx, job.out_sc, c->max_surv,
                       job.d_base, scan_in_scatter ? job.d_count : (int32_t *)nullptr,
                       scan_in_scatter ? job.d_count2 : (int32_t *)nullptr);
    return hipGetLastError();
}

}  // namespace cnnc

// ---- the compaction for callers that must not allocate ------------------------------------------------------------
// Per-workgroup counts live in a fixed array in the library's device image instead of a context's buffer.  Every GPU
// holds its own copy at its own address; the name below is only the host-side handle of the symbol, the address that
// kernels and copies may use comes from hipGetSymbolAddress with that GPU current.
namespace {
constexpr int kStaticMaxBlocks = CNNC_NOALLOC_MAX_VALUES / cnnc::kCompactPerBlock;
static_assert(CNNC_NOALLOC_MAX_VALUES % cnnc::kCompactPerBlock == 0, "the limit is a whole number of workgroups");
constexpr int kMaxDevices = 64;
static __device__ __align__(256) __attribute__((used)) int32_t scratch[kStaticMaxBlocks];     // 32 KiB per GPU, held until the process ends

std::mutex g_scratch_mutex;
int32_t *g_scratch_ptr[kMaxDevices];       // device address of `scratch` on each GPU, looked up once

// Device address of the scratch array on the current GPU (nullptr on failure).
int32_t *scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = static_cast<int32_t *>(p);
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" int cnnc_compact_noalloc(const float *d_values, int64_t n, float thr, uint32_t *d_index, float *d_score,
                                    int32_t cap, int32_t *d_count, void *stream)
{
    if (!d_count || n < 0 || cap < 0 || (n > 0 && !d_values) || (cap > 0 && (!d_index || !d_score)) || thr != thr)
        return CNNC_E_INVAL;
    if (n > CNNC_NOALLOC_MAX_VALUES) return CNNC_E_TOOBIG;
    int32_t *blockcnt = scratch_on_current_device();
    if (!blockcnt) return CNNC_E_HIP;
    hipStream_t st = (hipStream_t)stream;
    int nblocks = (int)((n + cnnc::kCompactPerBlock - 1) / cnnc::kCompactPerBlock);
    if (nblocks < 1) nblocks = 1;           // an empty input still writes a zero count
    // every entry of blockcnt[0, nblocks) is written by the count kernel before it is read: nothing to clear
    hipLaunchKernelGGL(cnnc::compact_count_kernel, dim3(nblocks), dim3(cnnc::kCompactBlock), 0, st, d_values,
                       (const int32_t *)nullptr, (const int32_t *)nullptr, n, n, thr, blockcnt);
    const bool scan_in_scatter = nblocks <= 4096;
    if (!scan_in_scatter)
        hipLaunchKernelGGL(cnnc::compact_scan_kernel, dim3(1), dim3(1024), 0, st, blockcnt, nblocks, (const int32_t *)nullptr,
                           d_count, (int32_t *)nullptr);
    hipLaunchKernelGGL(cnnc::compact_scatter_kernel, dim3(nblocks), dim3(cnnc::kCompactBlock), 0, st, d_values,
                       (const uint32_t *)nullptr, 0u, (const int32_t *)nullptr, (const int32_t *)nullptr, n, n, thr, blockcnt,
                       d_index, d_score, (int)cap, (const int32_t *)nullptr, scan_in_scatter ? d_count : (int32_t *)nullptr,
                       (int32_t *)nullptr);
    return hipGetLastError() == hipSuccess ? CNNC_OK : CNNC_E_HIP;
}

