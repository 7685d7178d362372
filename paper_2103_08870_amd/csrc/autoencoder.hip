// Autoencoder layers (Sec. IV-C, Tables I and II: 1-D convolutions / transposed convolutions,
// kernel size 1 or 3, stride 1 or 2, padding (ksize-1)/2) and the scatter/average step
// (Sec. V-B), for gfx950.  Generic per-layer kernels: one thread computes COT output channels
// at one output position; weights are wave-uniform and come through the scalar cache.
#include "lgc_internal.h"

namespace lgc {

__device__ __forceinline__ float leaky(float x, float slope) { return x > 0.f ? x : slope * x; }

// out[b][co][p] = bias[co] + sum_ci sum_t w[co][ci][t] * in[b][ci][p*stride - pad + t]
template <int COT, int KS>
__global__ __launch_bounds__(256) void k_conv1d(const float *__restrict__ in, float *__restrict__ out,
                                                const float *__restrict__ w, const float *__restrict__ bias,
                                                int c_in, int c_out, int stride, uint32_t l_in,
                                                uint32_t l_out, int act, float slope) {
    const uint32_t p = blockIdx.x * 256 + threadIdx.x;
    if (p >= l_out) return;
    const int co0 = blockIdx.y * COT;
    const int b = blockIdx.z;
    constexpr int PAD = (KS - 1) / 2;
    in += (size_t)b * c_in * l_in;
    out += (size_t)b * c_out * l_out;
    float acc[COT];
#pragma unroll
    for (int c = 0; c < COT; ++c) acc[c] = (co0 + c < c_out) ? bias[co0 + c] : 0.f;
    const long long q0 = (long long)p * stride - PAD;
    for (int ci = 0; ci < c_in; ++ci) {
        float x[KS];
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            const long long q = q0 + t;
            x[t] = (q >= 0 && q < (long long)l_in) ? in[(size_t)ci * l_in + q] : 0.f;
        }
#pragma unroll
        for (int c = 0; c < COT; ++c) {
            if (co0 + c < c_out) {
#pragma unroll
                for (int t = 0; t < KS; ++t) acc[c] = fmaf(w[((size_t)(co0 + c) * c_in + ci) * KS + t], x[t], acc[c]);
            }
        }
    }
#pragma unroll
    for (int c = 0; c < COT; ++c)
        if (co0 + c < c_out) out[(size_t)(co0 + c) * l_out + p] = act ? leaky(acc[c], slope) : acc[c];
}

// out[b][co][q] = bias[co] + sum_ci sum_{(p,t): p*stride - pad + t = q} w[ci][co][t] * in[b][ci][p]
template <int COT, int KS>
__global__ __launch_bounds__(256) void k_conv_transpose1d(const float *__restrict__ in, float *__restrict__ out,
                                                          const float *__restrict__ w,
                                                          const float *__restrict__ bias, int c_in, int c_out,
                                                          int stride, uint32_t l_in, uint32_t l_out, int act,
                                                          float slope) {
    const uint32_t q = blockIdx.x * 256 + threadIdx.x;
    if (q >= l_out) return;
    const int co0 = blockIdx.y * COT;
    const int b = blockIdx.z;
    constexpr int PAD = (KS - 1) / 2;
    in += (size_t)b * c_in * l_in;
    out += (size_t)b * c_out * l_out;
    float acc[COT];
#pragma unroll
    for (int c = 0; c < COT; ++c) acc[c] = (co0 + c < c_out) ? bias[co0 + c] : 0.f;
    // which taps reach q, and from which input position
    bool hit[KS];
    uint32_t src[KS];
#pragma unroll
    for (int t = 0; t < KS; ++t) {
        const long long num = (long long)q + PAD - t;
        hit[t] = num >= 0 && (num % stride) == 0 && (num / stride) < (long long)l_in;
        src[t] = hit[t] ? (uint32_t)(num / stride) : 0u;
    }
    for (int ci = 0; ci < c_in; ++ci) {
        float x[KS];
#pragma unroll
        for (int t = 0; t < KS; ++t) x[t] = hit[t] ? in[(size_t)ci * l_in + src[t]] : 0.f;
#pragma unroll
        for (int c = 0; c < COT; ++c) {
            if (co0 + c < c_out) {
#pragma unroll
                for (int t = 0; t < KS; ++t) acc[c] = fmaf(w[((size_t)ci * c_out + co0 + c) * KS + t], x[t], acc[c]);
            }
        }
    }
#pragma unroll
    for (int c = 0; c < COT; ++c)
        if (co0 + c < c_out) out[(size_t)(co0 + c) * l_out + q] = act ? leaky(acc[c], slope) : acc[c];
}

constexpr int kCot = 8;

void launch_conv1d(const float *in, float *out, const LayerDev &l, uint32_t l_in, uint32_t l_out, int batch,
                   bool act, float slope, hipStream_t st) {
    if (l_out == 0) return;
    dim3 grid((l_out + 255) / 256, (l.c_out + kCot - 1) / kCot, batch);
    if (l.ksize == 3)
        hipLaunchKernelGGL((k_conv1d<kCot, 3>), grid, dim3(256), 0, st, in, out, l.w, l.b, l.c_in, l.c_out,
                           l.stride, l_in, l_out, (int)act, slope);
    else
        hipLaunchKernelGGL((k_conv1d<kCot, 1>), grid, dim3(256), 0, st, in, out, l.w, l.b, l.c_in, l.c_out,
                           l.stride, l_in, l_out, (int)act, slope);
}

void launch_conv_transpose1d(const float *in, float *out, const LayerDev &l, uint32_t l_in, uint32_t l_out,
                             int batch, bool act, float slope, hipStream_t st) {
    if (l_out == 0) return;
    dim3 grid((l_out + 255) / 256, (l.c_out + kCot - 1) / kCot, batch);
    if (l.ksize == 3)
        hipLaunchKernelGGL((k_conv_transpose1d<kCot, 3>), grid, dim3(256), 0, st, in, out, l.w, l.b, l.c_in,
                           l.c_out, l.stride, l_in, l_out, (int)act, slope);
    else
        hipLaunchKernelGGL((k_conv_transpose1d<kCot, 1>), grid, dim3(256), 0, st, in, out, l.w, l.b, l.c_in,
                           l.c_out, l.stride, l_in, l_out, (int)act, slope);
}

// dense[idx[j]] <- dense[idx[j]] + scale*vals[j]; indices are distinct within one launch, so no
// atomics are needed and the result does not depend on scheduling.
__global__ __launch_bounds__(256) void k_scatter(const float *__restrict__ vals, const uint32_t *__restrict__ idx,
                                                 uint32_t k, float scale, float *__restrict__ dense, uint32_t n,
                                                 Stats *stats) {
    const uint32_t j = blockIdx.x * 256 + threadIdx.x;
    if (j >= k) return;
    const uint32_t i = idx[j];
    if (i >= n) { atomicAdd(&stats->errors, 1u); return; }
    dense[i] = __fadd_rn(dense[i], __fmul_rn(scale, vals[j]));
}

void launch_scatter(const float *vals, const uint32_t *idx, uint32_t k, float scale, float *dense, uint32_t n,
                    Stats *stats, hipStream_t st) {
    if (k == 0) return;
    hipLaunchKernelGGL(k_scatter, dim3((k + 255) / 256), dim3(256), 0, st, vals, idx, k, scale, dense, n, stats);
}

}  // namespace lgc
