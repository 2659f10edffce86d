// Machine probes used by the benchmark to put achieved rates beside what this GPU sustains in
// practice: dense fp32 MFMA, plain fp32 FMA on the vector ALU, an HBM copy; and the two measurements the
// kernels' designs lean on: how fast a vector instruction issues depending on where its operands sit, and what an
// LDS read costs for a given pattern of lane addresses.  Every kernel is a bounded loop over private registers,
// a bounds-checked copy, or reads of a workgroup's own LDS array at host-checked addresses.
#include "cnnc_internal.h"

namespace cnnc {

typedef float floatx4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256)
void peak_mfma_kernel(float *__restrict__ out, int iters)
{
    floatx4 acc[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] = floatx4{0, 0, 0, 0};
    const float a = 1.0f + threadIdx.x * 1e-6f, b = 1.0f - threadIdx.x * 1e-6f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[u], 0, 0, 0);
    }
    float s = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) s += acc[u][0] + acc[u][1] + acc[u][2] + acc[u][3];
    if (s == 12345.678f) out[0] = s;     // keeps the loop alive; practically never true
}

__global__ __launch_bounds__(256)
void peak_valu_kernel(float *__restrict__ out, int iters)
{
    float acc[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) acc[u] = threadIdx.x * 1e-3f + u;
    const float a = 0.999f, b = 1e-3f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 16; ++u) acc[u] = fmaf(acc[u], a, b);
    }
    float s = 0;
#pragma unroll
    for (int u = 0; u < 16; ++u) s += acc[u];
    if (s == 12345.678f) out[0] = s;
}

__global__ __launch_bounds__(256)
void peak_copy_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// ---- issue-rate probes: one kind of vector instruction back to back on sixteen independent registers ----------
// MODE 0: v_fmac_f32 with vector operands; 1: one operand in a scalar register; 2: a 32-bit literal; 3: v_rcp_f32
template <int MODE>
__global__ __launch_bounds__(256)
void issue_rate_kernel(float *__restrict__ out, int iters, float scalar_value)
{
    float acc[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) acc[u] = 1.0f + threadIdx.x * 1e-3f + u;
    float x = 0.5f + threadIdx.x * 1e-6f, w = 0.999f;
    asm volatile("" : "+v"(x), "+v"(w));
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            if (MODE == 0) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[u]) : "v"(w), "v"(x));
            else if (MODE == 1) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[u]) : "s"(scalar_value), "v"(x));
            else if (MODE == 2) asm volatile("v_fmac_f32 %0, 0x3f7fbe77, %1" : "+v"(acc[u]) : "v"(x));
            else asm volatile("v_rcp_f32 %0, %0" : "+v"(acc[u]));
        }
    }
    float s = 0;
#pragma unroll
    for (int u = 0; u < 16; ++u) s += acc[u];
    if (s == 12345.678f) out[0] = s;
}

// ---- LDS read probe: every lane reads W dwords at a dword address from a table, eight independent reads a batch
// (at offsets of 64 dwords, the same banks).  Lanes with a negative entry stay out.  The host checks the addresses.
constexpr int kLdsProbeDwords = 9216, kLdsProbeMaxAddr = 8704;
static_assert(kLdsProbeMaxAddr + 7 * 64 + 4 <= kLdsProbeDwords, "the last read of a batch stays inside the array");
template <int W>
__global__ __launch_bounds__(256)
void lds_read_kernel(const int32_t *__restrict__ tab, float *__restrict__ out, int iters)
{
    __shared__ __attribute__((aligned(16))) float lds[kLdsProbeDwords];
    for (int e = threadIdx.x; e < kLdsProbeDwords; e += 256) lds[e] = (float)(e & 7);
    __syncthreads();
    const int t = tab[threadIdx.x & 63];
    float s = 0.0f;
    if (t >= 0) {
        const uint32_t a = (uint32_t)(size_t)(&lds[0]) + 4u * (uint32_t)t;
        for (int i = 0; i < iters; ++i) {
            if (W == 1) {
                float v0, v1, v2, v3, v4, v5, v6, v7;
                asm volatile("ds_read_b32 %0, %8\n ds_read_b32 %1, %8 offset:256\n ds_read_b32 %2, %8 offset:512\n ds_read_b32 %3, %8 offset:768\n"
                             "ds_read_b32 %4, %8 offset:1024\n ds_read_b32 %5, %8 offset:1280\n ds_read_b32 %6, %8 offset:1536\n"
                             "ds_read_b32 %7, %8 offset:1792\n s_waitcnt lgkmcnt(0)"
                             : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7) : "v"(a) : "memory");
                s += v0 + v1 + v2 + v3 + v4 + v5 + v6 + v7;
            } else if (W == 2) {
                float2 v0, v1, v2, v3, v4, v5, v6, v7;
                asm volatile("ds_read_b64 %0, %8\n ds_read_b64 %1, %8 offset:256\n ds_read_b64 %2, %8 offset:512\n ds_read_b64 %3, %8 offset:768\n"
                             "ds_read_b64 %4, %8 offset:1024\n ds_read_b64 %5, %8 offset:1280\n ds_read_b64 %6, %8 offset:1536\n"
                             "ds_read_b64 %7, %8 offset:1792\n s_waitcnt lgkmcnt(0)"
                             : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7) : "v"(a) : "memory");
                s += v0.x + v1.y + v2.x + v3.y + v4.x + v5.y + v6.x + v7.y;
            } else {
                float4 v0, v1, v2, v3, v4, v5, v6, v7;
                asm volatile("ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:256\n ds_read_b128 %2, %8 offset:512\n ds_read_b128 %3, %8 offset:768\n"
                             "ds_read_b128 %4, %8 offset:1024\n ds_read_b128 %5, %8 offset:1280\n ds_read_b128 %6, %8 offset:1536\n"
                             "ds_read_b128 %7, %8 offset:1792\n s_waitcnt lgkmcnt(0)"
                             : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7) : "v"(a) : "memory");
                s += v0.x + v1.y + v2.z + v3.w + v4.x + v5.y + v6.z + v7.w;
            }
        }
    }
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace cnnc

extern "C" int cnnc_measure_issue_rates(double *ns, int n)
{
    using namespace cnnc;
    if (!ns || n < 1) return CNNC_E_INVAL;
    hipDeviceProp_t prop;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return CNNC_E_HIP;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return CNNC_E_HIP;
    float *d_out = nullptr;
    int rc = CNNC_OK;
    if (hipMalloc((void **)&d_out, 256) != hipSuccess) {
        rc = CNNC_E_NOMEM;
    } else {
        // four workgroups of four waves per compute unit: four waves on every SIMD
        const int grid = prop.multiProcessorCount * 4, iters = 20000;
        for (int mode = 0; mode < 4 && mode < n; ++mode) {
            float ms = 0;
            for (int rep = 0; rep < 2; ++rep) {      // first pass warms up
                (void)hipEventRecord(e0, nullptr);
                switch (mode) {
                case 0: hipLaunchKernelGGL(issue_rate_kernel<0>, dim3(grid), dim3(256), 0, nullptr, d_out, iters, 0.999f); break;
                case 1: hipLaunchKernelGGL(issue_rate_kernel<1>, dim3(grid), dim3(256), 0, nullptr, d_out, iters, 0.999f); break;
                case 2: hipLaunchKernelGGL(issue_rate_kernel<2>, dim3(grid), dim3(256), 0, nullptr, d_out, iters, 0.999f); break;
                default: hipLaunchKernelGGL(issue_rate_kernel<3>, dim3(grid), dim3(256), 0, nullptr, d_out, iters, 0.999f); break;
                }
                (void)hipEventRecord(e1, nullptr);
                (void)hipEventSynchronize(e1);
                (void)hipEventElapsedTime(&ms, e0, e1);
            }
            ns[mode] = (double)ms * 1e6 / ((double)iters * 16 * 4);   // per SIMD: 4 waves x iters x 16 instructions
        }
        if (hipGetLastError() != hipSuccess) rc = CNNC_E_HIP;
    }
    (void)hipFree(d_out);
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    return rc;
}

extern "C" int cnnc_measure_lds_read(const int32_t *addr, int width, double *ns_per_instruction)
{
    using namespace cnnc;
    if (!addr || !ns_per_instruction || (width != 1 && width != 2 && width != 4)) return CNNC_E_INVAL;
    for (int l = 0; l < 64; ++l)
        if (addr[l] >= 0 && (addr[l] % width != 0 || addr[l] > kLdsProbeMaxAddr)) return CNNC_E_INVAL;
    hipDeviceProp_t prop;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return CNNC_E_HIP;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return CNNC_E_HIP;
    const int per_cu = 4, grid = prop.multiProcessorCount * per_cu, iters = 2000;
    int32_t *d_tab = nullptr;
    float *d_out = nullptr;
    int rc = CNNC_OK;
    if (hipMalloc((void **)&d_tab, 64 * sizeof(int32_t)) != hipSuccess || hipMalloc((void **)&d_out, sizeof(float) * 256 * (size_t)grid) != hipSuccess) {
        rc = CNNC_E_NOMEM;
    } else if (hipMemcpy(d_tab, addr, 64 * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess) {
        rc = CNNC_E_HIP;
    } else {
        float ms = 0, best = 1e30f;
        for (int rep = 0; rep < 3; ++rep) {          // first pass warms up
            (void)hipEventRecord(e0, nullptr);
            if (width == 1) hipLaunchKernelGGL(lds_read_kernel<1>, dim3(grid), dim3(256), 0, nullptr, d_tab, d_out, iters);
            else if (width == 2) hipLaunchKernelGGL(lds_read_kernel<2>, dim3(grid), dim3(256), 0, nullptr, d_tab, d_out, iters);
            else hipLaunchKernelGGL(lds_read_kernel<4>, dim3(grid), dim3(256), 0, nullptr, d_tab, d_out, iters);
            (void)hipEventRecord(e1, nullptr);
            (void)hipEventSynchronize(e1);
            (void)hipEventElapsedTime(&ms, e0, e1);
            if (rep > 0 && ms < best) best = ms;
        }
        // wave instructions per compute unit: per_cu workgroups x 4 waves x iters x 8
        *ns_per_instruction = (double)best * 1e6 / ((double)per_cu * 4 * iters * 8);
        if (hipGetLastError() != hipSuccess) rc = CNNC_E_HIP;
    }
    (void)hipFree(d_tab); (void)hipFree(d_out);
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    return rc;
}

extern "C" int cnnc_measure_peaks(double *mfma_f32_tflops, double *valu_f32_tflops, double *hbm_copy_gbs)
{
    using namespace cnnc;
    if (!mfma_f32_tflops || !valu_f32_tflops || !hbm_copy_gbs) return CNNC_E_INVAL;
    hipDeviceProp_t prop;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return CNNC_E_HIP;
    const int cus = prop.multiProcessorCount;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return CNNC_E_HIP;
    float *d_out = nullptr;
    float4 *d_a = nullptr, *d_b = nullptr;
    const size_t n4 = (size_t)64 << 20;   // 1 GiB per buffer
    int rc = CNNC_OK;
    float ms = 0;
    if (hipMalloc((void **)&d_out, 256) != hipSuccess || hipMalloc((void **)&d_a, n4 * 16) != hipSuccess ||
        hipMalloc((void **)&d_b, n4 * 16) != hipSuccess) {
        rc = CNNC_E_NOMEM;
    } else if (hipMemset(d_a, 1, n4 * 16) != hipSuccess) {
        rc = CNNC_E_HIP;
    } else {
        const int grid = cus * 8, iters = 20000;
        for (int rep = 0; rep < 2; ++rep) {      // first pass warms up
            (void)hipEventRecord(e0, nullptr);
            hipLaunchKernelGGL(peak_mfma_kernel, dim3(grid), dim3(256), 0, nullptr, d_out, iters);
            (void)hipEventRecord(e1, nullptr);
            (void)hipEventSynchronize(e1);
            (void)hipEventElapsedTime(&ms, e0, e1);
        }
        *mfma_f32_tflops = (double)grid * 4 * iters * 8 * 2048.0 / (ms * 1e-3) / 1e12;
        for (int rep = 0; rep < 2; ++rep) {
            (void)hipEventRecord(e0, nullptr);
            hipLaunchKernelGGL(peak_valu_kernel, dim3(grid), dim3(256), 0, nullptr, d_out, iters);
            (void)hipEventRecord(e1, nullptr);
            (void)hipEventSynchronize(e1);
            (void)hipEventElapsedTime(&ms, e0, e1);
        }
        *valu_f32_tflops = (double)grid * 256 * iters * 16 * 2.0 / (ms * 1e-3) / 1e12;
        for (int rep = 0; rep < 3; ++rep) {
            (void)hipEventRecord(e0, nullptr);
            hipLaunchKernelGGL(peak_copy_kernel, dim3(cus * 16), dim3(256), 0, nullptr, d_a, d_b, n4);
            (void)hipEventRecord(e1, nullptr);
            (void)hipEventSynchronize(e1);
            (void)hipEventElapsedTime(&ms, e0, e1);
        }
        *hbm_copy_gbs = 2.0 * (double)n4 * 16 / (ms * 1e-3) / 1e9;
        if (hipGetLastError() != hipSuccess) rc = CNNC_E_HIP;
    }
    (void)hipFree(d_out); (void)hipFree(d_a); (void)hipFree(d_b);
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    return rc;
}
