// Machine-peak probes used by the benchmark to put achieved rates beside what this GPU sustains in
// practice: dense fp32 MFMA, plain fp32 FMA on the vector ALU, and an HBM copy.  Every kernel is a
// bounded loop over private registers or a bounds-checked copy.
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

}  // namespace cnnc

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
