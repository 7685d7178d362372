// Per-layer top-k selection for gfx950 (wave64).
//
// What is computed (paper: Sec. V-A and the layer loop of Alg. 1 / Alg. 2): the flat vector is a
// concatenation of layers (segments); every segment l keeps exactly its own k_l largest
// magnitudes (same key and tie rule as the flat selection), and the kept values of all segments
// are concatenated in segment order.
//
// How: segments of at least 8 K elements with a small k_l / n_l are "sampled": one block per
// (segment, node) reads about n_l / 64 keys (whole 128-byte lines at jittered places, at most 16 K
// keys), finds an order statistic of them in LDS and publishes it as the segment's candidate
// threshold; the streaming candidate pass and
// the gather kernel of the flat selection then list every element at or above its segment's
// threshold in index order (so each segment's candidates are one contiguous run of that list).
// All other segments are "direct": nothing is flagged for them.  Finally one block per
// (segment, node) selects exactly: from the segment's run of candidates when it holds at least
// k_l of them, else (and for direct segments) from the segment's elements of v themselves.  A block
// finds the exact k_l-th key by a 3-digit radix select (8 + 11 + 12 bits) in LDS and writes the
// kept values in index order.  No communication
// between blocks, no waiting.

#include "carry.h"
#include "device_helpers.h"

namespace lgc {


__device__ __forceinline__ uint32_t seg_mix(uint32_t h) {
    h *= 0x9E3779B1u; h ^= h >> 15; h *= 0x85EBCA77u; h ^= h >> 13; h *= 0xC2B2AE3Du; h ^= h >> 16;
    return h;
}

// Exact `rank`-th largest of the keys that `each` enumerates (block of T >= 256 threads; `each(f)`
// calls f(key) for every key this thread holds).  Three digits, most significant first: the
// 8 exponent bits, then 11 and 12 mantissa bits.  The keys of one layer share a handful of
// exponents, so the first histogram is kept in 16 copies (one per lane mod 16) to keep the LDS
// atomics of a wavefront on different addresses; mantissa digits spread by themselves.
// Returns the key; `above` receives the number of keys strictly greater.  hist: 4096 words.
template <int PASS, int T, typename Each>
__device__ __forceinline__ void radix_pass(Each each, uint32_t &rank, uint32_t &prefix, uint32_t &gt,
                                           uint32_t *hist /*[4096]*/, uint32_t *wave_tmp, uint32_t *res) {
    const uint32_t tid = threadIdx.x;
    constexpr int kWords = PASS == 1 ? 2048 : 4096;
    for (int i = tid; i < kWords; i += T) hist[i] = 0;
    __syncthreads();
    const uint32_t pre = prefix, copy = tid & 15u;
    each([=](uint32_t key) {
        if (PASS == 0) atomicAdd(&hist[((key >> 23) << 4) | copy], 1u);
        else if (PASS == 1) { if ((key >> 23) == pre) atomicAdd(&hist[(key >> 12) & 2047u], 1u); }
        else { if ((key >> 12) == pre) atomicAdd(&hist[key & 4095u], 1u); }
    });
    __syncthreads();
    if (PASS == 0) {                                         // fold the 16 copies: bins 0..255, the rest empty
        uint32_t sum = 0;
        if (tid < 256) {
#pragma unroll
            for (int c = 0; c < 16; ++c) sum += hist[tid * 16 + c];
        }
        __syncthreads();
        for (int i = tid; i < 1024; i += T) hist[i] = i < 256 ? sum : 0u;   // i < 256 only in the first trip: i == tid
        __syncthreads();
        find_rank_bin<1024>(hist, rank, wave_tmp, res);
    } else if (PASS == 1) {
        find_rank_bin<2048>(hist, rank, wave_tmp, res);
    } else {
        find_rank_bin<4096>(hist, rank, wave_tmp, res);
    }
    const uint32_t digit = res[0] == 0xffffffffu ? 0u : res[0];
    const uint32_t more = res[1];
    __syncthreads();
    rank -= more; gt += more;
    prefix = PASS == 0 ? digit : PASS == 1 ? ((prefix << 11) | digit) : ((prefix << 12) | digit);
}

template <int T, typename Each>
__device__ __forceinline__ uint32_t block_radix_select(Each each, uint32_t rank, uint32_t *hist /*[4096]*/,
                                                       uint32_t *wave_tmp, uint32_t *res, uint32_t &above) {
    uint32_t prefix = 0, gt = 0;
    radix_pass<0, T>(each, rank, prefix, gt, hist, wave_tmp, res);
    radix_pass<1, T>(each, rank, prefix, gt, hist, wave_tmp, res);
    radix_pass<2, T>(each, rank, prefix, gt, hist, wave_tmp, res);
    above = gt;
    return prefix;
}

// ------------------------------------------------------------------ thresholds of the sampled segments

// One block per (segment, node).  Direct segments publish 0xffffffff ("flag nothing").
// The keys that the accumulation WILL produce are sampled when FUSED (v + (m*u + g), not stored).
// The kernel also clears the state set that the next call will use.
template <bool FUSED, bool VEC>
__global__ __launch_bounds__(1024) void k_seg_estimate(SelArgs a) {
    __shared__ uint32_t hist[4096];
    __shared__ uint32_t wave_tmp[16], res[2];
    const uint32_t l = blockIdx.x, tid = threadIdx.x;
    const int node = blockIdx.y;
    {
        const uint32_t gt = (blockIdx.y * gridDim.x + blockIdx.x) * 1024u + tid, nt = gridDim.x * gridDim.y * 1024u;
        for (uint32_t i = gt; i < a.next_words; i += nt) a.next_state[i] = 0;
    }
    uint32_t *out = a.seg_t + (size_t)node * a.n_seg + l;
    const uint32_t packed = a.seg_rank[l];
    if (packed == 0) { if (tid == 0) *out = 0xffffffffu; return; }
    const uint32_t rank = packed & 0xffffu, threads = packed >> 16;   // 16 keys per sampling thread
    const uint32_t lo = a.seg_off[l], hi = a.seg_off[l + 1];
    if (a.seg_carry) {   // the layer's threshold offered by its previous selection (carry.h), if there is one
        Carry *c = a.seg_carry + (size_t)node * a.n_seg + l;
        const uint32_t t = a.carry_fresh ? 0u : c->next_t_est;
        const bool take = t != 0 && c->n == hi - lo && c->k == a.seg_k[l];   // the same for the whole block
        if (tid == 0) {
            c->carried_now = take;
            if (take) { *out = t; atomicAdd(&a.stats->carried, 1u); }
        }
        if (take) return;
    }
    // clusters of 32 elements (one 128-byte line per array) on 32-element boundaries of the vector,
    // inside the segment, one at a jittered place in each of threads/2 equal strata; two
    // neighbouring threads read the two halves of a cluster
    const uint32_t c0 = (lo + 31u) >> 5, c1 = hi >> 5;
    const uint32_t clusters = threads >> 1;
    const uint32_t stratum = (c1 - c0) / clusters;           // >= 3: a sampled segment has >= 8 K elements, i.e. 255 whole clusters for at most 64
    const bool active = tid < threads;
    const uint32_t ci = tid >> 1;
    const uint32_t cl = c0 + ci * stratum + seg_mix(ci * 0x9E3779B9u + l * 0x85EBCA6Bu + (uint32_t)node) % stratum;
    const size_t off = (size_t)node * a.stride + ((size_t)cl << 5) + ((tid & 1u) << 4);
    uint32_t keys[16];
    if (!active) {
#pragma unroll
        for (int j = 0; j < 16; ++j) keys[j] = 0;
    } else if (VEC) {
        f4 vv[4], uu[4], gg[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            vv[q] = *(const f4 *)(a.v + off + q * 4);
            if (FUSED) { uu[q] = *(const f4 *)(a.u + off + q * 4); gg[q] = *(const f4 *)(a.g + off + q * 4); }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float x = FUSED ? uu[q][j] : 0.f, y = vv[q][j];
                if (FUSED) accum1(gg[q][j], x, y, a.momentum);
                keys[q * 4 + j] = key_of(y);
            }
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            float y = a.v[off + j];
            if (FUSED) { float x = a.u[off + j]; accum1(a.g[off + j], x, y, a.momentum); }
            keys[j] = key_of(y);
        }
    }
    // the order statistic to 2^-11 relative resolution (exponent and 11 mantissa bits), rounded down: a threshold
    // needs no more, and a lower one only flags a few more candidates (3 % where the counts are steepest)
    auto each = [&](auto f) {
        if (active) {
#pragma unroll
            for (int j = 0; j < 16; ++j) f(keys[j]);
        }
    };
    uint32_t r = rank, prefix = 0, gt = 0;
    radix_pass<0, 1024>(each, r, prefix, gt, hist, wave_tmp, res);
    radix_pass<1, 1024>(each, r, prefix, gt, hist, wave_tmp, res);
    if (tid == 0) *out = prefix << 12;
}

void launch_seg_estimate(const SelArgs &a, int batch, bool fused, bool vec, hipStream_t st) {
    dim3 grid(a.n_seg, batch);
    if (fused) {
        if (vec) hipLaunchKernelGGL((k_seg_estimate<true, true>), grid, dim3(1024), 0, st, a);
        else hipLaunchKernelGGL((k_seg_estimate<true, false>), grid, dim3(1024), 0, st, a);
    } else {
        if (vec) hipLaunchKernelGGL((k_seg_estimate<false, true>), grid, dim3(1024), 0, st, a);
        else hipLaunchKernelGGL((k_seg_estimate<false, false>), grid, dim3(1024), 0, st, a);
    }
}

// ------------------------------------------------------------------ exact selection inside one segment

// The block's source: `bits` holds raw fp32 patterns at positions [begin, end); the position of
// entry p in the node's vector is pos[p] (candidate list) or p itself (pos == nullptr: the
// source is v).  ALIGNED: bits + (begin & ~3) is 16-byte aligned (vector loads).
// A long source is read four times (three digit passes and the output pass; it stays in the L2
// after the first) in rolled loops: unrolling those for 64 K entries was an order of magnitude
// slower (instruction fetch).
constexpr int kSelKeep = 8;                // 16-byte groups per thread that the register-cached path holds
constexpr int kSelThreads = 512;          // most segments and candidate runs are a few thousand entries

// DENSE: instead of the compact (position, value) output and the clearing of v and u, every entry p
// of the source gets dense[p] = its value if kept, +0 otherwise (the innovation component).
// SMALL: the source spans at most kSelKeep rounds (16 K entries from begin & ~3 on): it is read once
// and kept in registers for all four sweeps (the layers' candidate runs and the small layers).
template <bool ALIGNED, bool DENSE, bool SMALL>
__device__ __forceinline__ uint32_t select_in_block(const uint32_t *__restrict__ bits, const uint32_t *__restrict__ pos,
                                                const uint32_t begin, const uint32_t end, const uint32_t k,
                                                float *__restrict__ v, float *__restrict__ u,
                                                uint32_t *__restrict__ oidx, float *__restrict__ oval,
                                                float *__restrict__ dense, Stats *stats,
                                                uint32_t *hist, uint32_t *wave_tmp, uint32_t *res,
                                                uint32_t *sh_g, uint32_t *sh_e) {
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t a0 = begin & ~3u;
    const uint32_t groups = (end - a0 + 3u) >> 2;           // 16-byte groups from a0 on
    constexpr uint32_t T = kSelThreads;
    const uint32_t rounds = __builtin_amdgcn_readfirstlane((groups + T - 1u) / T);   // block-uniform loop bound

    auto load_group = [&](uint32_t g) -> u4 {                // raw patterns of entries a0 + 4g .. + 3 (0 outside)
        u4 x = {0u, 0u, 0u, 0u};
        if (g < groups) {
            const uint32_t p = a0 + (g << 2);
            if (ALIGNED && p + 4 <= end) {
                x = *(const u4 *)(bits + p);                 // entries below `begin` are masked by position later
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (p + c >= begin && p + c < end) x[c] = bits[p + c];
            }
        }
        return x;
    };
    auto inside = [&](uint32_t g, int c) { const uint32_t p = a0 + (g << 2) + c; return p >= begin && p < end; };

    u4 keep[SMALL ? kSelKeep : 1];
    if (SMALL) {
#pragma unroll
        for (int r = 0; r < kSelKeep; ++r) keep[r] = load_group(r * T + tid);
    }
    auto each_key = [&](auto f) {
        if (SMALL) {
#pragma unroll
            for (int r = 0; r < kSelKeep; ++r) {
                if ((uint32_t)r < rounds) {
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (inside(r * T + tid, c)) f(keep[r][c] & 0x7fffffffu);
                }
            }
            return;
        }
        for (uint32_t r0 = 0; r0 < rounds; r0 += 4) {        // four loads in flight
            u4 x[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) x[q] = load_group((r0 + q) * T + tid);
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (inside((r0 + q) * T + tid, c)) f(x[q][c] & 0x7fffffffu);
        }
    };

    uint32_t above;
    const uint32_t thr = block_radix_select<kSelThreads>(each_key, k, hist, wave_tmp, res, above);
    const uint32_t quota = k - above;                        // ties taken, lowest positions first

    // ordered output: entries are enumerated round by round, thread by thread, c = 0..3
    uint32_t run_g = 0, run_e = 0;                           // kept-or-tied entries of the earlier rounds
    auto emit_round = [&](const u4 x, const uint32_t g) {
        bool fg[4], fe[4];
        uint32_t lg = 0, le = 0, tg = 0, te = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t key = x[c] & 0x7fffffffu;
            const bool in = inside(g, c);
            fg[c] = in && key > thr;
            fe[c] = in && key == thr;
            const unsigned long long mg = __ballot(fg[c]), me = __ballot(fe[c]);
            lg += lanes_below(mg); tg += (uint32_t)__popcll(mg);
            le += lanes_below(me); te += (uint32_t)__popcll(me);
        }
        __syncthreads();                                     // the previous round's readers are done
        if (lane == 0) { sh_g[wave] = tg; sh_e[wave] = te; }
        __syncthreads();
        uint32_t cg = run_g + lg, ce = run_e + le, all_g = 0, all_e = 0;
#pragma unroll
        for (int w = 0; w < kSelThreads / 64; ++w) {
            const uint32_t wg = sh_g[w], we = sh_e[w];
            all_g += wg; all_e += we;
            if ((uint32_t)w < wave) { cg += wg; ce += we; }
        }
        run_g += all_g; run_e += all_e;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool kept = fg[c] || (fe[c] && ce < quota);
            const uint32_t p = a0 + (g << 2) + c;
            if (DENSE) {
                if (inside(g, c)) dense[p] = kept ? __uint_as_float(x[c]) : 0.0f;
            } else if (kept) {
                const uint32_t o = cg + (ce < quota ? ce : quota);
                const uint32_t ix = pos ? pos[p] : p;
                if (o < k) { oidx[o] = ix; oval[o] = __uint_as_float(x[c]); }
                else atomicAdd(&stats->errors, 1u);
                v[ix] = 0.0f;
                if (u) u[ix] = 0.0f;
            }
            cg += fg[c]; ce += fe[c];
        }
    };
    if (SMALL) {
#pragma unroll
        for (int r = 0; r < kSelKeep; ++r)
            if ((uint32_t)r < rounds) emit_round(keep[r], r * T + tid);   // block-uniform condition
    } else {
        u4 x = load_group(tid);
        for (uint32_t r = 0; r < rounds; ++r) {
            const u4 nx = load_group((r + 1) * T + tid);     // next round's group, in flight during this one
            emit_round(x, r * T + tid);
            x = nx;
        }
    }
    // every thread holds the block's totals: the selection must add up to k
    if (tid == 0 && run_g + (run_e < quota ? run_e : quota) != k) atomicAdd(&stats->errors, 1u);
    return thr;   // the exact k-th largest key
}

// One block per (segment, node).
template <bool VEC>
__global__ __launch_bounds__(kSelThreads) void k_seg_select(SelArgs a) {
    __shared__ uint32_t hist[4096];
    __shared__ uint32_t wave_tmp[16], res[2], sh_g[16], sh_e[16];
    const uint32_t l = blockIdx.x;
    const int node = blockIdx.y;
    // a selection of another kind on this context: the flat selection's carried thresholds lapse
    if (a.carry && l == 0 && threadIdx.x == 0) { a.carry[node].len = 0; a.carry[node].next_t_est = 0; }
    const uint32_t k = a.seg_k[l];
    if (k == 0) return;
    const uint32_t lo = a.seg_off[l], hi = a.seg_off[l + 1];
    float *v = a.v + (size_t)node * a.stride;
    float *u = a.u ? a.u + (size_t)node * a.stride : nullptr;
    uint32_t *oidx = a.out_idx + (size_t)node * a.k + a.seg_out[l];
    float *oval = a.out_vals + (size_t)node * a.k + a.seg_out[l];

    bool from_list = false;
    uint32_t p0 = 0, p1 = 0;
    const uint32_t *cidx = a.cand_idx + (size_t)node * a.cap;
    const uint32_t *cval = a.cand_val + (size_t)node * a.cap;
    if (a.seg_rank[l] != 0) {                                // sampled segment: its run of the candidate list
        const uint32_t total = a.sel[node].cand_total;
        if (total <= a.cap) {                                // nothing was lost
            // candidates listed before position x: those of the rows before x's row (written by the
            // gather kernel) plus the flags of x's row below x; wavefront 0 finds both ends
            if (threadIdx.x < 64) {
                const uint32_t lane = threadIdx.x & 31u, x = threadIdx.x < 32 ? lo : hi;
                uint32_t c = 0;
                const uint32_t row = x >> 10, e = x & 1023u;
                if (x < a.n) {
                    if (lane < (uint32_t)kRowWords) {
                        // word 4s+j, bit i  <->  element 256 s + 4 i + j of the row: those with 256 s + 4 i + j < e
                        const uint32_t sidx = lane >> 2, j = lane & 3u;
                        const int below = (int)e - (int)(256u * sidx + j);          // 4 i < below
                        const uint32_t cnt = below <= 0 ? 0u : (((uint32_t)below + 3u) >> 2 > 64u ? 64u : ((uint32_t)below + 3u) >> 2);
                        const unsigned long long w = a.bitmap[((size_t)node * a.rows + row) * kRowWords + lane];
                        const unsigned long long m = cnt >= 64u ? ~0ull : ((1ull << cnt) - 1ull);
                        c = (uint32_t)__popcll(w & m);
                    }
                    if (lane == 16) c = a.row_prefix[(size_t)node * a.rows + row];
                } else if (lane == 16) {
                    c = total;                               // the vector's end: everything is before it
                }
#pragma unroll
                for (int d = 16; d >= 1; d >>= 1) c += __shfl_xor(c, d, 64);   // sums inside each half of the wavefront
                if (lane == 0) res[threadIdx.x >> 5] = c;
            }
            __syncthreads();
            p0 = res[0]; p1 = res[1];
            __syncthreads();
            from_list = p1 - p0 >= k;
        }
        if (threadIdx.x == 0) atomicAdd(from_list ? &a.stats->fast : &a.stats->fallback, 1u);
    }
    constexpr uint32_t kSmall = (uint32_t)kSelKeep * kSelThreads * 4u;
    uint32_t thr;
    if (from_list) {
        if (p1 - (p0 & ~3u) <= kSmall)
            thr = select_in_block<true, false, true>(cval, cidx, p0, p1, k, v, u, oidx, oval, nullptr, a.stats, hist, wave_tmp, res, sh_g, sh_e);
        else
            thr = select_in_block<true, false, false>(cval, cidx, p0, p1, k, v, u, oidx, oval, nullptr, a.stats, hist, wave_tmp, res, sh_g, sh_e);
    } else {
        if (hi - (lo & ~3u) <= kSmall)
            thr = select_in_block<VEC, false, true>((const uint32_t *)v, nullptr, lo, hi, k, v, u, oidx, oval, nullptr, a.stats, hist, wave_tmp, res, sh_g, sh_e);
        else
            thr = select_in_block<VEC, false, false>((const uint32_t *)v, nullptr, lo, hi, k, v, u, oidx, oval, nullptr, a.stats, hist, wave_tmp, res, sh_g, sh_e);
    }
    // sampled layers: the record of this layer's exact thresholds, and its offer to the next selection
    if (a.seg_carry && a.seg_rank[l] != 0 && threadIdx.x == 0) {
        Carry *c = a.seg_carry + (size_t)node * a.n_seg + l;
        // a layer that keeps few values may flag k + 256: what its k-th magnitude does is noisy, and the candidates cost nothing
        const float most = fmaxf(a.carry_most, log2f((float)(k + 256u) / (float)k));
        carry_update(c, hi - lo, k, a.carry_fresh != 0, from_list, c->carried_now != 0, thr,
                     a.seg_t[(size_t)node * a.n_seg + l], p1 - p0, a.carry_target, most);
    }
}

// Innovation component (Alg. 1: threshold_inv, mask_inv; Sec. IV-C): per segment of the vector of
// selected values the k_l largest magnitudes stay, everything else becomes +0.  The input is not
// modified.  One block per (segment, node).
template <bool VEC>
__global__ __launch_bounds__(kSelThreads) void k_innovation(const float *__restrict__ vals, float *__restrict__ out,
                                                            uint32_t n, const uint32_t *__restrict__ seg_off,
                                                            const uint32_t *__restrict__ seg_k, Stats *stats) {
    __shared__ uint32_t hist[4096];
    __shared__ uint32_t wave_tmp[16], res[2], sh_g[16], sh_e[16];
    const uint32_t l = blockIdx.x;
    const uint32_t lo = seg_off[l], hi = seg_off[l + 1], k = seg_k[l];
    const float *src = vals + (size_t)blockIdx.y * n;
    float *dst = out + (size_t)blockIdx.y * n;
    if (k == 0) {
        for (uint32_t p = lo + threadIdx.x; p < hi; p += kSelThreads) dst[p] = 0.0f;
        return;
    }
    if (hi - (lo & ~3u) <= (uint32_t)kSelKeep * kSelThreads * 4u)
        select_in_block<VEC, true, true>((const uint32_t *)src, nullptr, lo, hi, k, nullptr, nullptr, nullptr, nullptr, dst, stats,
                                         hist, wave_tmp, res, sh_g, sh_e);
    else
        select_in_block<VEC, true, false>((const uint32_t *)src, nullptr, lo, hi, k, nullptr, nullptr, nullptr, nullptr, dst, stats,
                                          hist, wave_tmp, res, sh_g, sh_e);
}

void launch_innovation(const float *vals, float *out, uint32_t n, int batch, uint32_t n_seg, const uint32_t *seg_off,
                       const uint32_t *seg_k, bool vec, Stats *stats, hipStream_t st) {
    dim3 grid(n_seg, batch);
    if (vec) hipLaunchKernelGGL(k_innovation<true>, grid, dim3(kSelThreads), 0, st, vals, out, n, seg_off, seg_k, stats);
    else hipLaunchKernelGGL(k_innovation<false>, grid, dim3(kSelThreads), 0, st, vals, out, n, seg_off, seg_k, stats);
}

void launch_seg_select(const SelArgs &a, int batch, bool vec, hipStream_t st) {
    dim3 grid(a.n_seg, batch);
    if (vec) hipLaunchKernelGGL(k_seg_select<true>, grid, dim3(kSelThreads), 0, st, a);
    else hipLaunchKernelGGL(k_seg_select<false>, grid, dim3(kSelThreads), 0, st, a);
}

}  // namespace lgc
