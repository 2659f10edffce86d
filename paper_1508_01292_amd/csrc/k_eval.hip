// Stages 2 and 3 (paper, Section 3.3, selective unit: the regions that passed the previous stage
// are read from the original image, scaled to the network's input size and classified by the
// larger CNNs).  One workgroup takes one surviving window at a time: it gathers the crop from
// the uint8 frame (16.16 fixed-point bilinear, 8-bit weights), then runs the whole network with
// every intermediate map in LDS.  Workgroups stride over the survivor list, whose length is read
// from device memory, so no host round trip separates the stages.
//
// Max-pooling is applied to the pre-activations (the activation is non-decreasing, so
// f(max) = max(f)), which quarters the number of activations of the pooled layers.
#include "eval_common.h"

namespace cnnc {

namespace {
using namespace evalc;

// "valid" convolution, optional 2x2 max-pool of the pre-activations, activation.
// in: LDS [CIN][IN][IN]; out: LDS [COUT][PO][PO]; w: global [COUT][CIN][K][K].
template <int CIN, int COUT, int K, int IN, bool POOL, int ACT>
__device__ void conv_layer(const float *in, float *out, const float *__restrict__ w, const float *__restrict__ bias)
{
    constexpr int O = IN - K + 1, PO = POOL ? O / 2 : O, STEP = POOL ? 2 : 1, NA = POOL ? 4 : 1;
    for (int e = threadIdx.x; e < COUT * PO * PO; e += kThreads) {
        const int oc = e / (PO * PO), py = (e / PO) % PO, px = e % PO;
        float acc[NA];
#pragma unroll
        for (int q = 0; q < NA; ++q) acc[q] = 0.0f;
        const float *wp = w + (size_t)oc * CIN * K * K;
        for (int ic = 0; ic < CIN; ++ic) {
            const float *ip = in + (ic * IN + py * STEP) * IN + px * STEP;
#pragma unroll
            for (int a = 0; a < K; ++a)
#pragma unroll
                for (int b = 0; b < K; ++b) {
                    const float wv = wp[(ic * K + a) * K + b];
                    acc[0] = fmaf(wv, ip[a * IN + b], acc[0]);
                    if (POOL) {
                        acc[1] = fmaf(wv, ip[a * IN + b + 1], acc[1]);
                        acc[2] = fmaf(wv, ip[(a + 1) * IN + b], acc[2]);
                        acc[3] = fmaf(wv, ip[(a + 1) * IN + b + 1], acc[3]);
                    }
                }
        }
        float m = acc[0];
        if (POOL) m = fmaxf(fmaxf(acc[0], acc[1]), fmaxf(acc[2], acc[3]));
        out[e] = act_f<ACT>(m + bias[oc]);
    }
    __syncthreads();
}

// Fully connected layer: each wave takes outputs wave, wave+4, ...; lanes stride over the inputs.
template <int NIN, int NOUT, int ACT>
__device__ void fc_layer(const float *in, float *out, const float *__restrict__ w, const float *__restrict__ bias)
{
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    for (int o = wave; o < NOUT; o += kThreads / 64) {
        float acc = 0.0f;
        for (int i = lane; i < NIN; i += 64) acc = fmaf(w[(size_t)o * NIN + i], in[i], acc);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
        if (lane == 0) out[o] = act_f<ACT>(acc + bias[o]);
    }
    __syncthreads();
}

}  // namespace

template <int ACT>
__global__ __launch_bounds__(kThreads)
void eval2_kernel(const uint8_t *__restrict__ frame, int fw, int fh, int pitch, const LevelDev *__restrict__ levels,
                  int n_levels, const uint32_t *__restrict__ idx, const int32_t *__restrict__ d_begin,
                  const int32_t *__restrict__ d_n, int n_max, const float *__restrict__ wt, float *__restrict__ out)
{
    __shared__ uint32_t sTab[2 * kS2In];
    __shared__ float sCrop[24 * 24];
    __shared__ float sP1[8 * 10 * 10];
    __shared__ float sP2[16 * 4 * 4];
    __shared__ float sF[32];
    const int n = min(*d_n, n_max);
    for (int i = min(*d_begin, n_max) + blockIdx.x; i < n; i += gridDim.x) {
        const Survivor s = decode(idx[i], levels, n_levels);
        gather_crop<kS2In>(frame, fw, fh, pitch, s.x, s.y, levels[s.level].scale_q16, sTab, sCrop);
        conv_layer<1, 8, 5, 24, true, ACT>(sCrop, sP1, wt + s2::W1, wt + s2::B1);
        conv_layer<8, 16, 3, 10, true, ACT>(sP1, sP2, wt + s2::W2, wt + s2::B2);
        fc_layer<256, 32, ACT>(sP2, sF, wt + s2::W3, wt + s2::B3);
        if (threadIdx.x < 64) {
            float acc = threadIdx.x < 32 ? wt[s2::W4 + threadIdx.x] * sF[threadIdx.x] : 0.0f;
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
            if (threadIdx.x == 0) out[i] = acc + wt[s2::B4];
        }
        __syncthreads();
    }
}

template <int ACT>
__global__ __launch_bounds__(kThreads)
void eval3_kernel(const uint8_t *__restrict__ frame, int fw, int fh, int pitch, const LevelDev *__restrict__ levels,
                  int n_levels, const uint32_t *__restrict__ idx, const int32_t *__restrict__ d_begin,
                  const int32_t *__restrict__ d_n, int n_max, const float *__restrict__ wt, float *__restrict__ out)
{
    __shared__ uint32_t sTab[2 * kS3In];
    __shared__ float sCrop[48 * 48];
    __shared__ float sP1[16 * 22 * 22];
    __shared__ float sP2[32 * 9 * 9];
    __shared__ float sP3[32 * 7 * 7];
    __shared__ float sF[64];
    const int n = min(*d_n, n_max);
    for (int i = min(*d_begin, n_max) + blockIdx.x; i < n; i += gridDim.x) {
        const Survivor s = decode(idx[i], levels, n_levels);
        gather_crop<kS3In>(frame, fw, fh, pitch, s.x, s.y, levels[s.level].scale_q16, sTab, sCrop);
        conv_layer<1, 16, 5, 48, true, ACT>(sCrop, sP1, wt + s3::W1, wt + s3::B1);
        conv_layer<16, 32, 5, 22, true, ACT>(sP1, sP2, wt + s3::W2, wt + s3::B2);
        conv_layer<32, 32, 3, 9, false, ACT>(sP2, sP3, wt + s3::W3, wt + s3::B3);
        fc_layer<1568, 64, ACT>(sP3, sF, wt + s3::W4, wt + s3::B4);
        if (threadIdx.x < 64) {
            float acc = wt[s3::W5 + threadIdx.x] * sF[threadIdx.x];
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
            if (threadIdx.x == 0) out[i] = acc + wt[s3::B5];
        }
        __syncthreads();
    }
}

namespace {
int eval_grid(const cnnc_ctx *c)
{
    const int g = 256 * 8;   // a few workgroups per compute unit; each strides over the list
    return c->max_surv < g ? c->max_surv : g;
}
}  // namespace

#define CNNC_EVAL(KERNEL, ACT, IDX, WT, OUT)                                                                 \
    hipLaunchKernelGGL(KERNEL<ACT>, dim3(eval_grid(c)), dim3(kThreads), 0, st, c->d_frame, c->fw, c->fh,     \
                       c->fpitch, c->d_levels, c->n_levels, IDX, r.d_begin, r.d_end, c->max_surv, WT, OUT)

hipError_t launch_eval2(const cnnc_ctx *c, ListRange r, hipStream_t st)
{
    switch (c->act) {
    case CNNC_ACT_RATIONAL: CNNC_EVAL(eval2_kernel, CNNC_ACT_RATIONAL, c->d_idx[0], c->d_wt[1], c->d_eval[0]); break;
    case CNNC_ACT_SCALED_TANH: CNNC_EVAL(eval2_kernel, CNNC_ACT_SCALED_TANH, c->d_idx[0], c->d_wt[1], c->d_eval[0]); break;
    default: CNNC_EVAL(eval2_kernel, CNNC_ACT_TANH, c->d_idx[0], c->d_wt[1], c->d_eval[0]); break;
    }
    return hipGetLastError();
}

hipError_t launch_eval3(const cnnc_ctx *c, ListRange r, hipStream_t st)
{
    switch (c->act) {
    case CNNC_ACT_RATIONAL: CNNC_EVAL(eval3_kernel, CNNC_ACT_RATIONAL, c->d_idx[1], c->d_wt[2], c->d_eval[1]); break;
    case CNNC_ACT_SCALED_TANH: CNNC_EVAL(eval3_kernel, CNNC_ACT_SCALED_TANH, c->d_idx[1], c->d_wt[2], c->d_eval[1]); break;
    default: CNNC_EVAL(eval3_kernel, CNNC_ACT_TANH, c->d_idx[1], c->d_wt[2], c->d_eval[1]); break;
    }
    return hipGetLastError();
}

}  // namespace cnnc
