// The streaming kernels of liblgc for gfx950 (wave64): the passes that touch every element of g, u, v.
//
// What is computed (paper: Alg. 1 / Alg. 2, first line of the layer loop, with the momentum correction of
// Sec. V-A):   u <- m*u + g ; v <- v + u   -- three separately rounded fp32 operations per element --
// and, in the candidate pass, the flags "key(v) >= t_est" (key = bits(v) & 0x7fffffff) that the selection
// kernels (topk.hip, segmented.hip) work from: one bit per element in a dense bitmap, one count per row of
// 1024 elements.  One wavefront per row, twelve 16-byte loads in flight before anything depends on them,
// non-temporal loads and stores, no LDS, no barrier, no atomics, nothing shared between wavefronts.

#include <hip/hip_ext.h>

#include "device_helpers.h"

namespace lgc {

// ------------------------------------------------------------------ one row of a wavefront

// One full row of a wavefront: 4 x 256 consecutive elements, lane l holds elements 4l..4l+3 of
// each 256.  All twelve 16-byte loads are issued before anything depends on them.  Every stream
// is touched once per call, so all loads and stores are non-temporal: on this part that alone
// lifts the fused kernel from about 60 % to 72-77 % of the HBM peak (and the plain read of v in
// the selection-only form likewise; the few candidates' values are read again by the gather).
template <bool FUSED>
__device__ __forceinline__ void full_row(const float *__restrict__ g, float *__restrict__ u, float *__restrict__ v,
                                         const float m, uint32_t (&bits)[4][4]) {
    f4 gg[4], uu[4], vv[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        if (FUSED) {
            gg[s] = __builtin_nontemporal_load((const f4 *)(g + s * 256));
            uu[s] = __builtin_nontemporal_load((const f4 *)(u + s * 256));
        }
        vv[s] = __builtin_nontemporal_load((const f4 *)(v + s * 256));
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        if (FUSED) {
#pragma unroll
            for (int j = 0; j < 4; ++j) { float x = uu[s][j], y = vv[s][j]; accum1(gg[s][j], x, y, m); uu[s][j] = x; vv[s][j] = y; }
            __builtin_nontemporal_store(uu[s], (f4 *)(u + s * 256));
            __builtin_nontemporal_store(vv[s], (f4 *)(v + s * 256));
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) bits[s][j] = __float_as_uint(vv[s][j]);
    }
}

// ------------------------------------------------------------------ plain accumulation

// Same traversal as the candidate pass below: one wavefront per row of 1024 elements,
// all twelve 16-byte loads of a row in flight before anything depends on them, non-temporal.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_accumulate(const float *__restrict__ g, float *__restrict__ u,
                                                       float *__restrict__ v, uint32_t n, uint64_t stride,
                                                       float m) {
    const size_t off = (size_t)blockIdx.y * stride;
    g += off; u += off; v += off;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t nrows = (n + kRow - 1) / kRow;
    for (uint32_t r = blockIdx.x * kWaves + wave; r < nrows; r += gridDim.x * kWaves) {
        const uint32_t row = r * (uint32_t)kRow;
        const uint32_t end = (n - row > (uint32_t)kRow) ? row + kRow : n;
        if (VEC && row + 1024 <= end) {
            uint32_t bits[4][4];
            full_row<true>(g + row + lane * 4, u + row + lane * 4, v + row + lane * 4, m, bits);
        } else {
            for (uint32_t e = row + lane; e < end; e += 64) {
                float uu = u[e], vv = v[e];
                accum1(g[e], uu, vv, m);
                u[e] = uu; v[e] = vv;
            }
        }
    }
}

// Calls launch(node0, nodes, row_begin, row_end, events) for equal shares of at most kRowsPerLaunch rows:
// several whole nodes per launch while they fit, else one node in row ranges.  `events` carries the bracket's
// start event for the first share and its stop event for the last one.
template <typename F>
static void for_each_share(uint32_t nrows, int batch, Bracket br, F launch) {
    if ((uint64_t)nrows * batch <= kRowsPerLaunch) { launch(0u, batch, 0u, nrows, br); return; }
    if (nrows <= kRowsPerLaunch) {
        const int fit = (int)(kRowsPerLaunch / nrows);              // nodes that fit one launch
        const int launches = (batch + fit - 1) / fit;
        const int per = (batch + launches - 1) / launches;          // evened out
        for (int b = 0; b < batch; b += per) {
            Bracket e;
            if (b == 0) e.start = br.start;
            if (b + per >= batch) e.stop = br.stop;
            launch((uint32_t)b, batch - b < per ? batch - b : per, 0u, nrows, e);
        }
        return;
    }
    const uint32_t ranges = (nrows + kRowsPerLaunch - 1) / kRowsPerLaunch;
    const uint32_t per = ((nrows + ranges - 1) / ranges + (uint32_t)kWaves - 1) / kWaves * kWaves;   // whole blocks
    for (int b = 0; b < batch; ++b)
        for (uint32_t r = 0; r < nrows; r += per) {
            Bracket e;
            if (b == 0 && r == 0) e.start = br.start;
            if (b == batch - 1 && nrows - r <= per) e.stop = br.stop;
            launch((uint32_t)b, 1, r, nrows - r < per ? nrows : r + per, e);
        }
}

// An ordinary launch, or, with timing events, the launch form that stamps them itself.
template <typename K, typename... Args>
static void launch_timed(K kernel, dim3 grid, dim3 block, hipStream_t st, Bracket e, Args... args) {
    if (e.start || e.stop) hipExtLaunchKernelGGL(kernel, grid, block, 0, st, e.start, e.stop, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
}

void launch_accumulate(const float *g, float *u, float *v, uint32_t n, int batch, uint64_t stride,
                       float momentum, bool vec, hipStream_t st, Bracket br) {
    const uint32_t nrows = (n + kRow - 1) / kRow;
    for_each_share(nrows, batch, br, [&](uint32_t node0, int nodes, uint32_t r0, uint32_t r1, Bracket e) {
        // a share is passed as shifted pointers and its own length (row ranges keep 16-byte alignment)
        const size_t off = (size_t)node0 * stride + (size_t)r0 * kRow;
        const uint32_t len = (r1 == nrows ? n : r1 * (uint32_t)kRow) - r0 * (uint32_t)kRow;
        dim3 grid((r1 - r0 + kWaves - 1) / kWaves, nodes);
        if (vec) launch_timed(k_accumulate<true>, grid, dim3(kBlock), st, e, g + off, u + off, v + off, len, stride, momentum);
        else launch_timed(k_accumulate<false>, grid, dim3(kBlock), st, e, g + off, u + off, v + off, len, stride, momentum);
    });
}

// ------------------------------------------------------------------ candidate pass (the streaming kernel)

// FUSED: reads g,u,v, writes u,v (the accumulation) and classifies the new v; otherwise reads v.
// One wavefront per row of 1024 elements.  The flags "key >= t_est" of the row go out as one
// full 128-byte line of the candidate bitmap (dense, coalesced: no partial-line writes), the
// row's candidate count as one word.  No barrier, no LDS, no atomics, nothing shared.
// SEG: per-layer selection; the threshold of an element is that of its segment (a.seg_t, one per
// node and segment; 0xffffffff flags nothing).  a.row_seg names the segment of a row's first
// element, with bit 31 set when the row runs into further segments.
template <bool FUSED, bool VEC, bool SEG>
__global__ __launch_bounds__(kBlock) void k_candidates(SelArgs a) {
    const int node = a.node0 + blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t off = (size_t)node * a.stride;
    const float *__restrict__ g = a.g + off;
    float *__restrict__ u = a.u + off;
    float *__restrict__ v = a.v + off;
    const uint32_t t_est = SEG ? 0u : a.sel[node].t_est;
    const uint32_t *seg_t = SEG ? a.seg_t + (size_t)node * a.n_seg : nullptr;
    const float m = a.momentum;
    unsigned long long *bitmap = a.bitmap + (size_t)node * a.rows * kRowWords;
    uint32_t *row_count = a.row_count + (size_t)node * a.rows;
    for (uint32_t r = a.row_begin + blockIdx.x * kWaves + wave; r < a.row_end; r += gridDim.x * kWaves) {
        const uint32_t row = r * (uint32_t)kRow;
        const uint32_t end = (a.n - row > (uint32_t)kRow) ? row + kRow : a.n;
        uint32_t bits[4][4];
        uint32_t thr[4][4];
        if (SEG) {
            const uint32_t rs = a.row_seg[r];
            uint32_t l = rs & 0x7fffffffu;
            const uint32_t t0 = seg_t[l];
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int j = 0; j < 4; ++j) thr[s][j] = t0;
            if (rs >> 31) {   // wave-uniform: the row crosses into the next segment(s)
                for (++l; l < a.n_seg && a.seg_off[l] < end; ++l) {
                    const uint32_t ol = a.seg_off[l], tl = seg_t[l];
#pragma unroll
                    for (int s = 0; s < 4; ++s)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (row + s * 256 + lane * 4 + j >= ol) thr[s][j] = tl;
                }
            }
        }
        if (VEC && row + 1024 <= end) {
            full_row<FUSED>(g + row + lane * 4, u + row + lane * 4, v + row + lane * 4, m, bits);
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const uint32_t e0 = row + s * 256 + lane * 4;
                f4 vv = {0.f, 0.f, 0.f, 0.f};
                if (VEC && e0 + 3 < end) {
                    vv = *(const f4 *)(v + e0);
                    if (FUSED) {
                        const f4 gg = *(const f4 *)(g + e0);
                        f4 uu = *(const f4 *)(u + e0);
#pragma unroll
                        for (int j = 0; j < 4; ++j) { float x = uu[j], y = vv[j]; accum1(gg[j], x, y, m); uu[j] = x; vv[j] = y; }
                        *(f4 *)(u + e0) = uu;
                        *(f4 *)(v + e0) = vv;
                    }
                } else {
                    for (int j = 0; j < 4; ++j) if (e0 + j < end) {
                        float y = v[e0 + j];
                        if (FUSED) {
                            float x = u[e0 + j];
                            accum1(g[e0 + j], x, y, m);
                            u[e0 + j] = x; v[e0 + j] = y;
                        }
                        vv[j] = y;
                    }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) bits[s][j] = __float_as_uint(vv[j]);
            }
        }
        // 16 flag words of the row; lane i < 16 ends up holding word i
        uint32_t lo = 0, hi = 0, count = 0;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t e = row + s * 256 + lane * 4 + j;
                const unsigned long long mk = __ballot(e < end && (bits[s][j] & 0x7fffffffu) >= (SEG ? thr[s][j] : t_est));
                count += (uint32_t)__popcll(mk);
                const bool mine = lane == s * 4 + j;
                lo = mine ? (uint32_t)mk : lo;
                hi = mine ? (uint32_t)(mk >> 32) : hi;
            }
        }
        if (lane < kRowWords) bitmap[(size_t)r * kRowWords + lane] = ((unsigned long long)hi << 32) | lo;
        if (lane == 0) row_count[r] = count;
    }
}

void launch_candidates(const SelArgs &args, int batch, bool fused, bool vec, hipStream_t st, Bracket br) {
    const uint32_t nrows = (args.n + kRow - 1) / kRow;
    const bool seg = args.seg_t != nullptr;
    for_each_share(nrows, batch, br, [&](uint32_t node0, int nodes, uint32_t r0, uint32_t r1, Bracket e) {
        SelArgs a = args;
        a.node0 = node0; a.row_begin = r0; a.row_end = r1;
        dim3 grid((r1 - r0 + kWaves - 1) / kWaves, nodes);
#define LGC_CAND(F, V, S) launch_timed(k_candidates<F, V, S>, grid, dim3(kBlock), st, e, a)
        if (seg) {
            if (fused) { if (vec) LGC_CAND(true, true, true); else LGC_CAND(true, false, true); }
            else       { if (vec) LGC_CAND(false, true, true); else LGC_CAND(false, false, true); }
        } else {
            if (fused) { if (vec) LGC_CAND(true, true, false); else LGC_CAND(true, false, false); }
            else       { if (vec) LGC_CAND(false, true, false); else LGC_CAND(false, false, false); }
        }
#undef LGC_CAND
    });
}

}  // namespace lgc
