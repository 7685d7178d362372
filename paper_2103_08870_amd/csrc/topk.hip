// Accumulation and exact top-k selection kernels for gfx950 (wave64).
//
// What is computed (paper: Alg. 1 / Alg. 2, layer loop; Sec. V-A):
//   u <- m*u + g ; v <- v + u                     accumulation with momentum correction
//   S = first k positions in (|v| desc, index asc)  top-k magnitude selection, exact
//   vals/idx <- v at S (ascending index) ; v[S] <- 0 ; u[S] <- 0     g~ and the kept residual
//
// How: magnitudes are compared through the key bits(v) & 0x7fffffff.
//  * fast path: a sampled order statistic gives a key t_est with a few more than k elements
//    above it; ONE streaming pass over g,u,v writes u,v and extracts, in index order, every
//    element with key >= t_est ("candidates") plus a histogram of their keys.  The exact k-th
//    key T* and the number of ties to take are then found among the candidates alone, and the
//    output is compacted from them.  The result is exact whenever count(candidates) >= k; if
//    not (or if the candidate buffer would overflow) the device itself falls back to
//  * exact path: a 3-pass (11+10+10 bit) radix select over all of v, then an ordered
//    compaction of v with the exact threshold.
//  Ordered compaction uses one look-back chain over 4096-element chunks (chunk ids are handed
//  out by an atomic ticket, so a chunk only ever waits for chunks that already run).
#include "lgc_internal.h"

namespace lgc {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

enum { SRC_FUSED = 0, SRC_PLAIN = 1, SRC_CAND = 2 };

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
__device__ void find_rank_bin(const uint32_t *hist, uint32_t rank, uint32_t *wave_tmp, uint32_t *res) {
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

// ------------------------------------------------------------------ plain accumulation

template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_accumulate(const float *__restrict__ g, float *__restrict__ u,
                                                       float *__restrict__ v, uint32_t n, uint64_t stride,
                                                       float m) {
    const size_t off = (size_t)blockIdx.y * stride;
    g += off; u += off; v += off;
    const uint32_t tid = blockIdx.x * kBlock + threadIdx.x, nthreads = gridDim.x * kBlock;
    if (VEC) {
        const uint32_t n4 = n >> 2;
        for (uint32_t i = tid; i < n4; i += nthreads) {
            f4 gg = __builtin_nontemporal_load((const f4 *)g + i);
            f4 uu = ((const f4 *)u)[i], vv = ((const f4 *)v)[i];
#pragma unroll
            for (int j = 0; j < 4; ++j) { float x = uu[j], y = vv[j]; accum1(gg[j], x, y, m); uu[j] = x; vv[j] = y; }
            ((f4 *)u)[i] = uu; ((f4 *)v)[i] = vv;
        }
        for (uint32_t i = (n4 << 2) + tid; i < n; i += nthreads) {
            float uu = u[i], vv = v[i];
            accum1(g[i], uu, vv, m);
            u[i] = uu; v[i] = vv;
        }
    } else {
        for (uint32_t i = tid; i < n; i += nthreads) {
            float uu = u[i], vv = v[i];
            accum1(g[i], uu, vv, m);
            u[i] = uu; v[i] = vv;
        }
    }
}

void launch_accumulate(const float *g, float *u, float *v, uint32_t n, int batch, uint64_t stride,
                       float momentum, bool vec, hipStream_t st) {
    uint32_t blocks = (uint32_t)(((uint64_t)n + kChunk - 1) / kChunk);
    if (blocks > 8192) blocks = 8192;
    if (blocks == 0) blocks = 1;
    dim3 grid(blocks, batch);
    if (vec) hipLaunchKernelGGL(k_accumulate<true>, grid, dim3(kBlock), 0, st, g, u, v, n, stride, momentum);
    else hipLaunchKernelGGL(k_accumulate<false>, grid, dim3(kBlock), 0, st, g, u, v, n, stride, momentum);
}

// ------------------------------------------------------------------ clearing of the scratch

__global__ __launch_bounds__(kBlock) void k_clear(SelArgs a, uint32_t chunks_n, uint32_t chunks_cand) {
    const int node = blockIdx.y;
    const uint32_t tid = blockIdx.x * kBlock + threadIdx.x, nthreads = gridDim.x * kBlock;
    unsigned long long *s0 = a.status[0] + (size_t)node * a.status_stride;
    unsigned long long *s1 = a.status[1] + (size_t)node * a.status_stride;
    unsigned long long *s2 = a.status[2] + (size_t)node * a.status_stride;
    for (uint32_t i = tid; i < chunks_n; i += nthreads) { s0[i] = 0; s2[i] = 0; }
    for (uint32_t i = tid; i < chunks_cand; i += nthreads) s1[i] = 0;
    for (uint32_t i = tid; i < (uint32_t)kSampleBins; i += nthreads) a.sample_hist[node * kSampleBins + i] = 0;
    for (uint32_t i = tid; i < (uint32_t)kFineBins; i += nthreads) a.fine_hist[node * kFineBins + i] = 0;
    for (uint32_t i = tid; i < 3u * kRadixBins; i += nthreads) a.radix_hist[node * 3 * kRadixBins + i] = 0;
    if (tid < sizeof(Sel) / 4) ((uint32_t *)(a.sel + node))[tid] = 0;
}

void launch_clear(const SelArgs &a, int batch, uint32_t chunks_n, uint32_t chunks_cand, hipStream_t st) {
    uint32_t work = chunks_n > (uint32_t)(3 * kRadixBins) ? chunks_n : 3 * kRadixBins;
    uint32_t blocks = (work + kBlock - 1) / kBlock;
    if (blocks > 64) blocks = 64;
    hipLaunchKernelGGL(k_clear, dim3(blocks, batch), dim3(kBlock), 0, st, a, chunks_n, chunks_cand);
}

// ------------------------------------------------------------------ sampled threshold estimate

__device__ __forceinline__ uint32_t mix32(uint32_t h) {
    h *= 0x9E3779B1u; h ^= h >> 15; h *= 0x85EBCA77u; h ^= h >> 13; h *= 0xC2B2AE3Du; h ^= h >> 16;
    return h;
}

// One group of four neighbouring elements per thread, at a jittered position inside the thread's
// own stratum of the vector.  The keys that the accumulation WILL produce are sampled (the fused
// source recomputes v + (m*u + g) without storing it).  The last block to finish picks the key
// t_est = (roughly) the rank-th largest sampled key.
template <bool FUSED>
__global__ __launch_bounds__(kBlock) void k_sample(SelArgs a) {
    __shared__ uint32_t hist[kSampleBins];
    __shared__ uint32_t wave_tmp[kWaves], res[2];
    __shared__ uint32_t is_last;
    const int node = blockIdx.y, tid = threadIdx.x;
    const size_t off = (size_t)node * a.stride;
    const uint32_t j = blockIdx.x * kBlock + tid;  // < kSampleGroups
    const uint32_t stratum = (a.n >> 2) / kSampleGroups;
    const uint32_t e = (j * stratum + mix32(j + 0x5bd1e995u * (uint32_t)node) % stratum) << 2;
    uint32_t *smp = a.samples + (size_t)node * kSample;
    uint32_t *sh = a.sample_hist + node * kSampleBins;
    for (int i = tid; i < kSampleBins; i += kBlock) hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float vv = a.v[off + e + i];
        if (FUSED) {
            float uu = a.u[off + e + i];
            accum1(a.g[off + e + i], uu, vv, a.momentum);
        }
        uint32_t key = key_of(vv);
        smp[j * 4 + i] = key;
        atomicAdd(&hist[key >> 20], 1u);
    }
    __syncthreads();
    for (int i = tid; i < kSampleBins; i += kBlock) { uint32_t h = hist[i]; if (h) atomicAdd(&sh[i], h); }
    __threadfence();
    __syncthreads();
    if (tid == 0) is_last = (atomicAdd(&a.sel[node].done[0], 1u) == gridDim.x - 1);
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    for (int i = tid; i < kSampleBins; i += kBlock) hist[i] = ld_agent32(&sh[i]);
    __syncthreads();
    find_rank_bin<kSampleBins>(hist, a.rank, wave_tmp, res);
    const uint32_t b1 = res[0], need = a.rank - res[1];
    __syncthreads();
    if (b1 == 0xffffffffu) {  // cannot happen (rank <= kSample); leave t_est = 0: everything is a candidate
        return;
    }
    for (int i = tid; i < 1024; i += kBlock) hist[i] = 0;
    __syncthreads();
    for (uint32_t i = tid; i < kSample; i += kBlock) {
        uint32_t key = ld_agent32(&smp[i]);
        if ((key >> 20) == b1) atomicAdd(&hist[(key >> 10) & 1023u], 1u);
    }
    __syncthreads();
    find_rank_bin<1024>(hist, need, wave_tmp, res);
    if (tid == 0) a.sel[node].t_est = (b1 << 20) | ((res[0] == 0xffffffffu ? 0u : res[0]) << 10);
}

void launch_sample(const SelArgs &a, int batch, bool fused, hipStream_t st) {
    dim3 grid(kSampleGroups / kBlock, batch);
    if (fused) hipLaunchKernelGGL(k_sample<true>, grid, dim3(kBlock), 0, st, a);
    else hipLaunchKernelGGL(k_sample<false>, grid, dim3(kBlock), 0, st, a);
}

// ------------------------------------------------------------------ ordered compaction

// status word of a chunk: [63:62] 0 = nothing yet, 1 = this chunk's own counts, 2 = counts of all
// chunks up to and including this one; [61:31] count of "greater", [30:0] count of "equal".
__device__ __forceinline__ unsigned long long pack_status(uint32_t st, uint32_t gt, uint32_t eq) {
    return ((unsigned long long)st << 62) | ((unsigned long long)gt << 31) | (unsigned long long)eq;
}

// SRC_FUSED: reads g,u,v, writes u,v (accumulation) and classifies the new v.
// SRC_PLAIN: reads v.   SRC_CAND: reads the candidate list.
// EXACT = false: "greater" means key >= t_est; such elements are appended, in index order, to
//                the candidate list and counted in the fine histogram.
// EXACT = true : threshold T* and tie quota are known; the selected elements are written to the
//                output in index order and zeroed in v (and u).
template <int SRC, bool EXACT, bool VEC>
__global__ __launch_bounds__(kBlock) void k_emit(SelArgs a) {
    constexpr int SLOT = (SRC == SRC_CAND) ? 1 : (EXACT ? 2 : 0);
    __shared__ uint32_t sh_chunk;
    __shared__ uint32_t sh_gt[kRows][kWaves], sh_eq[kRows][kWaves];
    __shared__ uint32_t sh_prefix[2];

    const int node = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    Sel *s = a.sel + node;
    if (SRC == SRC_CAND) { if (!s->fast_ok) return; }
    if (SRC == SRC_PLAIN && EXACT) { if (!a.force && s->fast_ok) return; }

    if (tid == 0) sh_chunk = atomicAdd(&s->ticket[SLOT], 1u);
    __syncthreads();
    const uint32_t chunk = sh_chunk;
    const uint32_t n_src = (SRC == SRC_CAND) ? s->cand_total : a.n;
    const uint32_t base = chunk * (uint32_t)kChunk;
    if (base >= n_src) return;
    const uint32_t nchunks = (n_src + kChunk - 1) / kChunk;

    const size_t off = (size_t)node * a.stride;
    const float *g = a.g + off;
    float *u = a.u ? a.u + off : nullptr;
    float *v = a.v + off;
    const uint32_t *cidx = a.cand_idx + (size_t)node * a.cap;
    const uint32_t *cval = a.cand_val + (size_t)node * a.cap;

    const uint32_t thr = EXACT ? s->thr : s->t_est;
    const uint32_t quota = EXACT ? s->quota : 0u;

    uint32_t bits[kRows][4];   // value bits of my 16 elements
    uint32_t pos[kRows][4];    // original index (SRC_CAND only)
    uint32_t gtm = 0, eqm = 0; // flag bit r*4+j

#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const uint32_t e0 = base + r * kRowElems + tid * 4;
        if (SRC == SRC_CAND) {
            u4 ci = {0, 0, 0, 0}, cv = {0, 0, 0, 0};
            if (e0 + 3 < n_src) { ci = *(const u4 *)(cidx + e0); cv = *(const u4 *)(cval + e0); }
            else {
                for (int j = 0; j < 4; ++j) if (e0 + j < n_src) { ci[j] = cidx[e0 + j]; cv[j] = cval[e0 + j]; }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) { pos[r][j] = ci[j]; bits[r][j] = cv[j]; }
        } else if (SRC == SRC_PLAIN) {
            f4 vv = {0.f, 0.f, 0.f, 0.f};
            if (VEC && e0 + 3 < n_src) vv = *(const f4 *)(v + e0);
            else { for (int j = 0; j < 4; ++j) if (e0 + j < n_src) vv[j] = v[e0 + j]; }
#pragma unroll
            for (int j = 0; j < 4; ++j) bits[r][j] = __float_as_uint(vv[j]);
        } else {
            f4 vv = {0.f, 0.f, 0.f, 0.f};
            if (VEC && e0 + 3 < n_src) {
                f4 gg = __builtin_nontemporal_load((const f4 *)(g + e0));
                f4 uu = *(const f4 *)(u + e0);
                vv = *(const f4 *)(v + e0);
#pragma unroll
                for (int j = 0; j < 4; ++j) { float x = uu[j], y = vv[j]; accum1(gg[j], x, y, a.momentum); uu[j] = x; vv[j] = y; }
                *(f4 *)(u + e0) = uu;
                *(f4 *)(v + e0) = vv;
            } else {
                for (int j = 0; j < 4; ++j) if (e0 + j < n_src) {
                    float x = u[e0 + j], y = v[e0 + j];
                    accum1(g[e0 + j], x, y, a.momentum);
                    u[e0 + j] = x; v[e0 + j] = y; vv[j] = y;
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) bits[r][j] = __float_as_uint(vv[j]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool valid = e0 + j < n_src;
            const uint32_t key = bits[r][j] & 0x7fffffffu;
            const bool fg = valid && (EXACT ? key > thr : key >= thr);
            const bool fe = EXACT && valid && key == thr;
            gtm |= (uint32_t)fg << (r * 4 + j);
            eqm |= (uint32_t)fe << (r * 4 + j);
        }
    }

    // position of my flagged elements inside the block, in index order (row, wave, lane, j)
    uint32_t lane_gt[kRows], lane_eq[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        uint32_t lg = 0, le = 0, tg = 0, te = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            unsigned long long m = __ballot((gtm >> (r * 4 + j)) & 1u);
            lg += lanes_below(m); tg += __popcll(m);
            if (EXACT) {
                unsigned long long me = __ballot((eqm >> (r * 4 + j)) & 1u);
                le += lanes_below(me); te += __popcll(me);
            }
        }
        lane_gt[r] = lg; lane_eq[r] = le;
        if (lane == 0) { sh_gt[r][wave] = tg; sh_eq[r][wave] = te; }
    }
    __syncthreads();
    uint32_t off_gt[kRows], off_eq[kRows], blk_gt = 0, blk_eq = 0;
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            if (w == wave) { off_gt[r] = blk_gt; off_eq[r] = blk_eq; }
            blk_gt += sh_gt[r][w]; blk_eq += sh_eq[r][w];
        }
    }

    // look-back over the preceding chunks (first wave only)
    if (wave == 0) {
        unsigned long long *st = a.status[SLOT] + (size_t)node * a.status_stride;
        uint32_t pg = 0, pe = 0;
        if (chunk == 0) {
            if (lane == 0) st_agent(&st[0], pack_status(2, blk_gt, blk_eq));
        } else {
            if (lane == 0) st_agent(&st[chunk], pack_status(1, blk_gt, blk_eq));
            int first = (int)chunk - 1;
            uint32_t spins = 0;
            bool failed = false;
            while (first >= 0) {
                const int jn = first - lane;
                const bool valid = jn >= 0;
                unsigned long long w = 0;
                while (true) {
                    if (valid) w = ld_agent(&st[jn]);
                    const bool ready = !valid || (w >> 62) != 0;
                    if (__all(ready)) break;
                    if (++spins > a.spin_limit) { failed = true; break; }
                    __builtin_amdgcn_s_sleep(2);
                }
                if (failed) break;
                const unsigned long long incl = __ballot(valid && (w >> 62) == 2);
                const int nearest = incl ? (__ffsll((long long)incl) - 1) : 64;
                const bool take = valid && lane <= nearest;
                pg += wave_sum(take ? (uint32_t)((w >> 31) & 0x7fffffffu) : 0u);
                pe += wave_sum(take ? (uint32_t)(w & 0x7fffffffu) : 0u);
                if (incl) break;
                first -= 64;
            }
            if (failed && lane == 0) {
                atomicAdd(&a.stats->errors, 1u);
                s->wait_failed = 1;
            }
            if (lane == 0) st_agent(&st[chunk], pack_status(2, pg + blk_gt, pe + blk_eq));
        }
        if (lane == 0) { sh_prefix[0] = pg; sh_prefix[1] = pe; }
    }
    __syncthreads();
    const uint32_t pre_gt = sh_prefix[0], pre_eq = sh_prefix[1];

    if (tid == 0 && chunk == nchunks - 1) {
        if (!EXACT) s->cand_total = pre_gt + blk_gt;
        else {
            const uint32_t te = pre_eq + blk_eq;
            if (pre_gt + blk_gt + (te < quota ? te : quota) != a.k) atomicAdd(&a.stats->errors, 1u);
        }
    }

    if ((gtm | eqm) == 0) return;

    uint32_t *oidx = a.out_idx + (size_t)node * a.k;
    float *oval = a.out_vals + (size_t)node * a.k;
    uint32_t *widx = a.cand_idx + (size_t)node * a.cap;
    uint32_t *wval = a.cand_val + (size_t)node * a.cap;
    uint32_t *fine = a.fine_hist + node * kFineBins;

#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        uint32_t cg = pre_gt + off_gt[r] + lane_gt[r];
        uint32_t ce = pre_eq + off_eq[r] + lane_eq[r];
        const uint32_t e0 = base + r * kRowElems + tid * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool fg = (gtm >> (r * 4 + j)) & 1u, fe = (eqm >> (r * 4 + j)) & 1u;
            if (!EXACT) {
                if (fg) {
                    if (cg < a.cap) { widx[cg] = e0 + j; wval[cg] = bits[r][j]; }
                    uint32_t d = ((bits[r][j] & 0x7fffffffu) - thr) >> kFineShift;
                    atomicAdd(&fine[d < (uint32_t)kFineBins - 1 ? d : (uint32_t)kFineBins - 1], 1u);
                }
            } else {
                if (fg || (fe && ce < quota)) {
                    const uint32_t o = cg + (ce < quota ? ce : quota);
                    const uint32_t where = (SRC == SRC_CAND) ? pos[r][j] : e0 + j;
                    if (o < a.k) { oidx[o] = where; oval[o] = __uint_as_float(bits[r][j]); }
                    else atomicAdd(&a.stats->errors, 1u);
                    v[where] = 0.0f;
                    if (u) u[where] = 0.0f;
                }
            }
            cg += fg; ce += fe;
        }
    }
}

void launch_candidates(const SelArgs &a, int batch, bool fused, bool vec, hipStream_t st) {
    dim3 grid((a.n + kChunk - 1) / kChunk, batch);
    if (fused) {
        if (vec) hipLaunchKernelGGL((k_emit<SRC_FUSED, false, true>), grid, dim3(kBlock), 0, st, a);
        else hipLaunchKernelGGL((k_emit<SRC_FUSED, false, false>), grid, dim3(kBlock), 0, st, a);
    } else {
        if (vec) hipLaunchKernelGGL((k_emit<SRC_PLAIN, false, true>), grid, dim3(kBlock), 0, st, a);
        else hipLaunchKernelGGL((k_emit<SRC_PLAIN, false, false>), grid, dim3(kBlock), 0, st, a);
    }
}

void launch_output_from_candidates(const SelArgs &a, int batch, hipStream_t st) {
    dim3 grid((a.cap + kChunk - 1) / kChunk, batch);
    hipLaunchKernelGGL((k_emit<SRC_CAND, true, true>), grid, dim3(kBlock), 0, st, a);
}

void launch_exact_output(const SelArgs &a, int batch, bool vec, hipStream_t st) {
    dim3 grid((a.n + kChunk - 1) / kChunk, batch);
    if (vec) hipLaunchKernelGGL((k_emit<SRC_PLAIN, true, true>), grid, dim3(kBlock), 0, st, a);
    else hipLaunchKernelGGL((k_emit<SRC_PLAIN, true, false>), grid, dim3(kBlock), 0, st, a);
}

// ------------------------------------------------------------------ exact k-th key among the candidates

// One block per node.  Needs count(candidates) >= k and the list complete; otherwise the node is
// handed to the exact path (fast_ok stays 0).
__global__ __launch_bounds__(1024) void k_select_candidates(SelArgs a) {
    __shared__ uint32_t hist[kFineBins];
    __shared__ uint32_t wave_tmp[16], res[2];
    const int node = blockIdx.x, tid = threadIdx.x;
    Sel *s = a.sel + node;
    const uint32_t total = s->cand_total;
    if (s->wait_failed || total < a.k || total > a.cap) {
        if (tid == 0) { s->fast_ok = 0; atomicAdd(&a.stats->fallback, 1u); }
        return;
    }
    const uint32_t t_est = s->t_est;
    const uint32_t *cval = a.cand_val + (size_t)node * a.cap;
    for (int i = tid; i < kFineBins; i += 1024) hist[i] = a.fine_hist[node * kFineBins + i];
    __syncthreads();
    find_rank_bin<kFineBins>(hist, a.k, wave_tmp, res);
    const uint32_t bin = res[0];
    uint32_t need = a.k - res[1];
    __syncthreads();

    uint32_t thr;
    if (bin < (uint32_t)kFineBins - 1) {
        for (int i = tid; i < kFineBins; i += 1024) hist[i] = 0;
        __syncthreads();
        for (uint32_t i = tid; i < total; i += 1024) {
            const uint32_t d = (cval[i] & 0x7fffffffu) - t_est;
            if ((d >> kFineShift) == bin) atomicAdd(&hist[d & ((1u << kFineShift) - 1)], 1u);
        }
        __syncthreads();
        find_rank_bin<kFineBins>(hist, need, wave_tmp, res);
        thr = t_est + (bin << kFineShift) + res[0];
        need -= res[1];
    } else {
        // the k-th key lies beyond the histogram's range: radix select on (key - t_est) over the
        // candidates of the last bin, digits [31:20], [19:8], [7:0]
        const uint32_t lo = ((uint32_t)kFineBins - 1) << kFineShift;
        uint32_t prefix = 0;
        const int shifts[3] = {20, 8, 0};
        const uint32_t masks[3] = {0xfffu, 0xfffu, 0xffu};
        for (int p = 0; p < 3; ++p) {
            for (int i = tid; i < kFineBins; i += 1024) hist[i] = 0;
            __syncthreads();
            for (uint32_t i = tid; i < total; i += 1024) {
                const uint32_t d = (cval[i] & 0x7fffffffu) - t_est;
                const bool member = d >= lo && (p == 0 || (d >> (shifts[p - 1])) == prefix);
                if (member) atomicAdd(&hist[(d >> shifts[p]) & masks[p]], 1u);
            }
            __syncthreads();
            find_rank_bin<kFineBins>(hist, need, wave_tmp, res);
            need -= res[1];
            prefix = (p == 0) ? res[0] : ((prefix << (shifts[p - 1] - shifts[p])) | res[0]);
            __syncthreads();
        }
        thr = t_est + prefix;
    }
    if (tid == 0) {
        s->thr = thr;
        s->quota = need;
        s->fast_ok = 1;
        atomicAdd(&a.stats->fast, 1u);
    }
}

void launch_select_candidates(const SelArgs &a, int batch, hipStream_t st) {
    hipLaunchKernelGGL(k_select_candidates, dim3(batch), dim3(1024), 0, st, a);
}

// ------------------------------------------------------------------ exact path: radix select over v

// pass 0: digit = key >> 20 ; pass 1: (key >> 10) & 1023 under prefix key >> 20 ;
// pass 2: key & 1023 under prefix key >> 10.  The last block to finish a pass fixes the digit.
template <int PASS, bool VEC>
__global__ __launch_bounds__(kBlock) void k_radix_pass(SelArgs a) {
    __shared__ uint32_t hist[kRadixBins];
    __shared__ uint32_t wave_tmp[kWaves], res[2];
    __shared__ uint32_t is_last;
    const int node = blockIdx.y, tid = threadIdx.x;
    Sel *s = a.sel + node;
    if (!a.force && s->fast_ok) return;
    const float *v = a.v + (size_t)node * a.stride;
    uint32_t *gh = a.radix_hist + (node * 3 + PASS) * kRadixBins;
    const uint32_t prefix = s->prefix;
    const uint32_t rank = PASS == 0 ? a.k : s->need;
    constexpr int NB = PASS == 0 ? kRadixBins : 1024;

    for (int i = tid; i < NB; i += kBlock) hist[i] = 0;
    __syncthreads();
    auto count = [&](uint32_t key) {
        if (PASS == 0) atomicAdd(&hist[key >> 20], 1u);
        else if (PASS == 1) { if ((key >> 20) == prefix) atomicAdd(&hist[(key >> 10) & 1023u], 1u); }
        else { if ((key >> 10) == prefix) atomicAdd(&hist[key & 1023u], 1u); }
    };
    const uint32_t gtid = blockIdx.x * kBlock + tid, nthreads = gridDim.x * kBlock;
    if (VEC) {
        const uint32_t n4 = a.n >> 2;
        for (uint32_t i = gtid; i < n4; i += nthreads) {
            f4 vv = ((const f4 *)v)[i];
            count(key_of(vv.x)); count(key_of(vv.y)); count(key_of(vv.z)); count(key_of(vv.w));
        }
        for (uint32_t i = (n4 << 2) + gtid; i < a.n; i += nthreads) count(key_of(v[i]));
    } else {
        for (uint32_t i = gtid; i < a.n; i += nthreads) count(key_of(v[i]));
    }
    __syncthreads();
    for (int i = tid; i < NB; i += kBlock) { uint32_t h = hist[i]; if (h) atomicAdd(&gh[i], h); }
    __threadfence();
    __syncthreads();
    if (tid == 0) is_last = (atomicAdd(&s->done[1 + PASS], 1u) == gridDim.x - 1);
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    for (int i = tid; i < NB; i += kBlock) hist[i] = ld_agent32(&gh[i]);
    __syncthreads();
    find_rank_bin<NB>(hist, rank, wave_tmp, res);
    if (tid == 0) {
        const uint32_t digit = res[0] == 0xffffffffu ? 0u : res[0];
        const uint32_t left = rank - res[1];
        if (PASS == 0) { s->prefix = digit; s->need = left; }
        else if (PASS == 1) { s->prefix = (prefix << 10) | digit; s->need = left; }
        else { s->thr = (prefix << 10) | digit; s->quota = left; }
    }
}

void launch_radix_pass(const SelArgs &a, int batch, int pass, bool vec, hipStream_t st) {
    uint32_t blocks = (a.n + kChunk - 1) / kChunk;
    if (blocks > 2048) blocks = 2048;
    dim3 grid(blocks, batch);
#define LGC_RP(P)                                                                             \
    if (vec) hipLaunchKernelGGL((k_radix_pass<P, true>), grid, dim3(kBlock), 0, st, a);       \
    else hipLaunchKernelGGL((k_radix_pass<P, false>), grid, dim3(kBlock), 0, st, a)
    if (pass == 0) { LGC_RP(0); } else if (pass == 1) { LGC_RP(1); } else { LGC_RP(2); }
#undef LGC_RP
}

}  // namespace lgc
