// Small device-side helpers shared by the selection kernels (gfx950, wave64).
#pragma once
#include "lgc_internal.h"

namespace lgc {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------ small helpers

__device__ __forceinline__ uint32_t key_of(float x) { return __float_as_uint(x) & 0x7fffffffu; }

__device__ __forceinline__ uint32_t lanes_below(unsigned long long m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t x) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}

__device__ __forceinline__ unsigned long long ld_agent(const unsigned long long *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(unsigned long long *p, unsigned long long x) {
    __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t ld_agent32(const uint32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// accumulation step: three separately rounded fp32 operations, never contracted
__device__ __forceinline__ void accum1(float g, float &u, float &v, float m) {
    u = __fadd_rn(__fmul_rn(m, u), g);
    v = __fadd_rn(v, u);
}

// Block-wide search in a histogram held in LDS: finds the bin b such that
// count(bins > b) < rank <= count(bins >= b).  Every thread owns NB/blockDim.x consecutive bins.
// Result through LDS: res[0] = b (or 0xffffffff if the histogram holds fewer than rank), res[1] =
// count(bins > b).  All threads must call; contains barriers.
template <int NB>
__device__ inline void find_rank_bin(const uint32_t *hist, uint32_t rank, uint32_t *wave_tmp, uint32_t *res) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    const int per = NB / blockDim.x;
    uint32_t part = 0;
    for (int i = 0; i < per; ++i) part += hist[tid * per + i];
    // inclusive suffix sum inside the wave
    uint32_t incl = part;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t y = __shfl_down(incl, d, 64);
        if (lane + d < 64) incl += y;
    }
    if (tid == 0) { res[0] = 0xffffffffu; res[1] = 0; }
    if (lane == 0) wave_tmp[wave] = incl;
    __syncthreads();
    uint32_t above = incl - part;
    for (int w = wave + 1; w < nw; ++w) above += wave_tmp[w];
    if (above < rank && rank <= above + part) {
        uint32_t acc = above;
        for (int i = per - 1; i >= 0; --i) {
            uint32_t h = hist[tid * per + i];
            if (acc + h >= rank) { res[0] = tid * per + i; res[1] = acc; break; }
            acc += h;
        }
    }
    __syncthreads();
}

}  // namespace lgc
