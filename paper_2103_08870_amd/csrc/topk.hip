// Exact top-k selection kernels for gfx950 (wave64); the passes over all of g, u, v are in streaming.hip.
//
// What is computed (paper: Alg. 1 / Alg. 2, layer loop; Sec. V-A):
//   u <- m*u + g ; v <- v + u                     accumulation with momentum correction (streaming.hip)
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
//  The candidate pass writes one flag bit per element (a dense bitmap, full cache lines) and a
//  count per row of 1024, so the streaming kernel has no communication between wavefronts at
//  all and no scattered stores; a small gather kernel lists the flagged elements in index order.
//  The output over the candidates needs no communication between blocks either: short lists are
//  read whole by every block, long lists are counted per 4096-candidate chunk by one kernel and
//  written by the next.  The exact path is three radix passes, a count of every block's run of v, and the
//  ordered output of the runs: all in one block per node when the input is short, one launch whose blocks share
//  the phases out through tickets when it is the fast path's fall-back, five launches of many blocks when it
//  is chosen outright for a long input.

#include "carry.h"
#include "device_helpers.h"

namespace lgc {

// A store to a word in pinned host memory that the host reads without synchronising with the stream.
__device__ __forceinline__ void st_system32(uint32_t *p, uint32_t x) {
    __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// A selection that does not go through the fast path's report leaves "nothing on record" for the next one.
__device__ __forceinline__ void carry_lapse(const SelArgs &a, const int node) {
    if (a.carry) { a.carry[node].len = 0; a.carry[node].next_t_est = 0; }
}

// ------------------------------------------------------------------ clearing of a state set

__global__ __launch_bounds__(kBlock) void k_clear(uint32_t *words, uint32_t count) {
    for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < count; i += gridDim.x * kBlock) words[i] = 0;
}

void launch_clear(uint32_t *words, uint32_t count, hipStream_t st) {
    uint32_t blocks = (count + kBlock - 1) / kBlock;
    if (blocks > 256) blocks = 256;
    if (blocks == 0) return;
    hipLaunchKernelGGL(k_clear, dim3(blocks), dim3(kBlock), 0, st, words, count);
}

// ------------------------------------------------------------------ sampled threshold estimate

__device__ __forceinline__ uint32_t mix32(uint32_t h) {
    h *= 0x9E3779B1u; h ^= h >> 15; h *= 0x85EBCA77u; h ^= h >> 13; h *= 0xC2B2AE3Du; h ^= h >> 16;
    return h;
}

// Four neighbouring elements per thread.  The keys that the accumulation WILL produce are sampled (the fused
// source recomputes v + (m*u + g) without storing it); their first-level histogram (key >> 20)
// is accumulated per block in LDS and flushed with a few atomics.  The block of a node that finishes last then
// works out the estimate: t_est = (roughly) the rank-th largest sampled key, to 2^-13 relative resolution (first
// level from the histogram, second level from the keys).  Nobody waits for anybody.
// A node whose record of carried thresholds offers a candidate threshold for this very selection (same shape, the
// selection right after the one that wrote it) takes that one and samples nothing.
// The kernel also clears the state set that the next call will use.
template <bool FUSED, bool VEC>
__global__ __launch_bounds__(1024) void k_sample(SelArgs a) {
    __shared__ uint32_t hist[kSampleBins];
    __shared__ uint32_t wave_tmp[16], res[2];
    __shared__ uint32_t sh_last;
    const int node = blockIdx.y, tid = threadIdx.x;
    {
        const uint32_t gt = (blockIdx.y * gridDim.x + blockIdx.x) * 1024u + tid, nt = gridDim.x * gridDim.y * 1024u;
        for (uint32_t i = gt; i < a.next_words; i += nt) a.next_state[i] = 0;
    }
    if (a.carry) {   // uniform over the node's blocks
        const Carry *c = a.carry + node;
        const uint32_t t = c->next_t_est;
        if (t != 0 && c->n == a.n && c->k == a.k) {
            if (blockIdx.x == 0 && tid == 0) { a.sel[node].t_est = t; a.sel[node].carried = 1; atomicAdd(&a.stats->carried, 1u); }
            return;
        }
    }
    const size_t off = (size_t)node * a.stride;
    // four neighbouring threads read one 64-byte cluster of 16 elements; the clusters sit at
    // jittered positions, one in each of kSampleGroups/4 strata of the vector
    const uint32_t j = blockIdx.x * 1024u + tid;  // < kSampleGroups
    const uint32_t cl = j >> 2;
    // stratum cl = clusters [cl * C / 4096, (cl + 1) * C / 4096) of the vector's C = n / 16 whole clusters: the
    // strata cover the vector evenly whatever n is (n >= kMinFastN makes none of them empty)
    static_assert(kSampleGroups / 4 == 4096 && kMinFastN >= 16 * 4096, "4096 strata of at least one cluster");
    const uint32_t clusters = a.n >> 4;
    const uint32_t s_lo = (uint32_t)(((unsigned long long)cl * clusters) >> 12);
    const uint32_t s_hi = (uint32_t)(((unsigned long long)(cl + 1) * clusters) >> 12);
    const uint32_t e = ((s_lo + mix32(cl + 0x5bd1e995u * (uint32_t)node) % (s_hi - s_lo)) << 4) + ((j & 3u) << 2);
    uint32_t *smp = a.samples + (size_t)node * kSample;
    uint32_t *sh = a.sample_hist + node * kSampleBins;
    for (int i = tid; i < kSampleBins; i += 1024) hist[i] = 0;
    __syncthreads();
    u4 keys;
    f4 vv, uu = {0.f, 0.f, 0.f, 0.f}, gg = {0.f, 0.f, 0.f, 0.f};
    if (VEC) {
        vv = *(const f4 *)(a.v + off + e);
        if (FUSED) { uu = *(const f4 *)(a.u + off + e); gg = *(const f4 *)(a.g + off + e); }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            vv[i] = a.v[off + e + i];
            if (FUSED) { uu[i] = a.u[off + e + i]; gg[i] = a.g[off + e + i]; }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float x = uu[i], y = vv[i];
        if (FUSED) accum1(gg[i], x, y, a.momentum);
        keys[i] = key_of(y);
        atomicAdd(&hist[keys[i] >> 20], 1u);
    }
    *(u4 *)(smp + j * 4) = keys;
    __syncthreads();
    for (int i = tid; i < kSampleBins; i += 1024) { uint32_t h = hist[i]; if (h) atomicAdd(&sh[i], h); }

    // Which block is the last of the node to get here?  Every wavefront first waits until its stores and atomics
    // have been acknowledged, one thread releases them to the device and counts the block.
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
    if (tid == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        sh_last = atomicAdd(&a.ctr[node].sampled, 1u) == gridDim.x - 1 ? 1u : 0u;
    }
    __syncthreads();
    if (!sh_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // the other blocks' keys, through this XCD's caches

    u4 x[kSample / 4 / 1024];
#pragma unroll
    for (int r = 0; r < (int)(kSample / 4 / 1024); ++r) x[r] = *(const u4 *)(smp + (r * 1024 + tid) * 4);
    for (int i = tid; i < kSampleBins; i += 1024) hist[i] = ld_agent32(&sh[i]);
    __syncthreads();
    find_rank_bin<kSampleBins>(hist, a.rank, wave_tmp, res);
    const uint32_t b1 = res[0], need = a.rank - res[1];
    __syncthreads();
    if (b1 == 0xffffffffu) return;  // cannot happen (rank <= kSample); t_est stays 0: everything is a candidate
    hist[tid] = 0;
    __syncthreads();
#pragma unroll
    for (int r = 0; r < (int)(kSample / 4 / 1024); ++r) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if ((x[r][i] >> 20) == b1) atomicAdd(&hist[(x[r][i] >> 10) & 1023u], 1u);
    }
    __syncthreads();
    find_rank_bin<1024>(hist, need, wave_tmp, res);
    if (tid == 0) a.sel[node].t_est = (b1 << 20) | ((res[0] == 0xffffffffu ? 0u : res[0]) << 10);
}

void launch_sample(const SelArgs &a, int batch, bool fused, bool vec, hipStream_t st) {
    dim3 grid(kSampleGroups / 1024, batch);
    if (fused) {
        if (vec) hipLaunchKernelGGL((k_sample<true, true>), grid, dim3(1024), 0, st, a);
        else hipLaunchKernelGGL((k_sample<true, false>), grid, dim3(1024), 0, st, a);
    } else {
        if (vec) hipLaunchKernelGGL((k_sample<false, true>), grid, dim3(1024), 0, st, a);
        else hipLaunchKernelGGL((k_sample<false, false>), grid, dim3(1024), 0, st, a);
    }
}

// ------------------------------------------------------------------ gather of the candidates

template <int THREADS>
__device__ __forceinline__ uint32_t block_sum(uint32_t x, uint32_t *tmp /*[16]*/) {
    x = wave_sum(x);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) tmp[threadIdx.x >> 6] = x;
    __syncthreads();
    uint32_t t = 0;
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) t += tmp[w];
    return t;
}

// ROWS bitmap rows per block of THREADS threads.  Lists the candidates of its rows, in index
// order, behind those of all earlier rows of the node: position, and value re-read from v.
// Counts them in the fine histogram of d = key - t_est (bins of 2^12, last bin open-ended) and
// adds the block's count to the node's total.  The block's part of the bitmap is staged in LDS;
// the work is balanced over the threads by output position (binary search of the owning row,
// then of the bit inside the row), whatever the spread of the candidates.
// Long vectors (a.supers != 0): the candidates of every kSuperRows rows are summed by a kernel of their own, so
// that a gather block adds up at most kSuperRows row counts (and a few sums) to find its place
// instead of all the counts before it, which at 2^28 elements was most of the gather's time.

__global__ __launch_bounds__(1024) void k_row_sums(SelArgs a) {
    __shared__ uint32_t tmp[16];
    const uint32_t nrows = (a.n + kRow - 1) / kRow;
    const uint32_t *cnt = a.row_count + (size_t)blockIdx.y * a.rows;
    const uint32_t lo = blockIdx.x * kSuperRows;
    uint32_t part = 0;
#pragma unroll
    for (int r = 0; r < 2; ++r) {   // rows per node are a multiple of 4 in the scratch; rows past nrows are not read
        const uint32_t i0 = lo + (r * 1024 + threadIdx.x) * 4;
        if (i0 + 3 < nrows) { const u4 x = *(const u4 *)(cnt + i0); part += x[0] + x[1] + x[2] + x[3]; }
        else for (uint32_t i = i0; i < nrows; ++i) part += cnt[i];
    }
    const uint32_t total = block_sum<1024>(part, tmp);
    if (threadIdx.x == 0) a.row_super[(size_t)blockIdx.y * a.supers + blockIdx.x] = total;
}

template <bool HIST, int ROWS, int THREADS>
__global__ __launch_bounds__(THREADS) void k_gather(SelArgs a) {
    constexpr int kGatherRows = ROWS;
    constexpr int kPairs = (ROWS * kRowWords / 2 + THREADS - 1) / THREADS;   // pairs of bitmap words per thread
    static_assert(ROWS % 64 == 0 && ROWS <= THREADS && (ROWS & (ROWS - 1)) == 0, "rows per block");
    __shared__ uint32_t hist[HIST ? kFineBins : 1];
    __shared__ unsigned long long rows_lds[kGatherRows * kRowWords];
    __shared__ uint32_t offs[kGatherRows];
    __shared__ uint32_t tmp[16];
    const int node = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    Sel *s = a.sel + node;
    const uint32_t nrows = (a.n + kRow - 1) / kRow;
    const uint32_t first = blockIdx.x * (uint32_t)kGatherRows;
    const uint32_t mine = nrows - first < (uint32_t)kGatherRows ? nrows - first : (uint32_t)kGatherRows;
    const uint32_t *cnt = a.row_count + (size_t)node * a.rows;
    const unsigned long long *bitmap = a.bitmap + ((size_t)node * a.rows + first) * kRowWords;
    const float *v = a.v + (size_t)node * a.stride;
    uint32_t *cidx = a.cand_idx + (size_t)node * a.cap, *cval = a.cand_val + (size_t)node * a.cap;

    // all independent loads first: my row's count, my slice of the bitmap, the counts before the block
    const uint32_t c = (uint32_t)tid < mine ? cnt[first + tid] : 0u;
    ulonglong2 bm[kPairs];
#pragma unroll
    for (int q = 0; q < kPairs; ++q) {
        const uint32_t w2 = q * THREADS + tid;   // pair of words
        bm[q] = (w2 * 2 < mine * kRowWords) ? *(const ulonglong2 *)(bitmap + (size_t)w2 * 2) : ulonglong2{0ull, 0ull};
    }
    const uint32_t t_est = HIST ? s->t_est : 0u;
    // candidates before the block: whole groups of kSuperRows rows (summed beforehand when the
    // vector has more than one group), then the rows of the block's own group
    const uint32_t group = a.supers ? first / kSuperRows : 0u;
    uint32_t part = (uint32_t)tid < group ? a.row_super[(size_t)node * a.supers + tid] : 0u;
    for (uint32_t i0 = group * kSuperRows + tid * 4; i0 < first; i0 += 4 * THREADS * 4) {   // first and the row stride are multiples of 4
        u4 x[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = (i0 + r * 4 * THREADS < first) ? *(const u4 *)(cnt + i0 + r * 4 * THREADS) : (u4){0u, 0u, 0u, 0u};
#pragma unroll
        for (int r = 0; r < 4; ++r) part += x[r][0] + x[r][1] + x[r][2] + x[r][3];
    }
#pragma unroll
    for (int q = 0; q < kPairs; ++q) {
        if ((q * THREADS + tid) * 2 < kGatherRows * kRowWords) {
            rows_lds[(q * THREADS + tid) * 2] = bm[q].x;
            rows_lds[(q * THREADS + tid) * 2 + 1] = bm[q].y;
        }
    }
    if (HIST) for (int i = tid; i < kFineBins; i += THREADS) hist[i] = 0;
    const uint32_t before = block_sum<THREADS>(part, tmp);   // contains barriers: LDS is filled for all
    // exclusive scan of c over the first kGatherRows threads
    uint32_t incl = c;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(incl, d, 64);
        if (lane >= d) incl += y;
    }
    __syncthreads();
    if (lane == 63) tmp[wave] = incl;
    __syncthreads();
    uint32_t excl = incl - c, block_total = 0;
#pragma unroll
    for (int w = 0; w < kGatherRows / 64; ++w) { if (w < wave) excl += tmp[w]; block_total += tmp[w]; }
    if (tid < kGatherRows) offs[tid] = excl;
    // per-layer selection: where each row's candidates start in the list
    if (!HIST && (uint32_t)tid < mine) a.row_prefix[(size_t)node * a.rows + first + tid] = before + excl;
    if (tid == 0 && block_total) atomicAdd(&s->cand_total, block_total);
    __syncthreads();

    for (uint32_t p = tid; p < block_total; p += THREADS) {
        // last row r with offs[r] <= p: it is the one that holds output position p
        uint32_t r = 0;
#pragma unroll
        for (int step = kGatherRows / 2; step >= 1; step >>= 1)
            if (offs[r + step] <= p) r += step;
        uint32_t i = p - offs[r];   // the i-th candidate of row r, in element order (s, lane, j)
        const unsigned long long *w = rows_lds + r * kRowWords;
        unsigned long long w0 = 0, w1 = 0, w2 = 0, w3 = 0;
        uint32_t sub = 0;
        bool found = false;
#pragma unroll
        for (int sr = 0; sr < 4; ++sr) {
            const unsigned long long x0 = w[4 * sr], x1 = w[4 * sr + 1], x2 = w[4 * sr + 2], x3 = w[4 * sr + 3];
            const uint32_t cs = (uint32_t)(__popcll(x0) + __popcll(x1) + __popcll(x2) + __popcll(x3));
            if (!found) {
                if (i < cs) { found = true; sub = sr; w0 = x0; w1 = x1; w2 = x2; w3 = x3; }
                else i -= cs;
            }
        }
        // largest l such that the lanes below l hold at most i flags: lane l holds candidate i
        uint32_t l = 0;
#pragma unroll
        for (int step = 32; step >= 1; step >>= 1) {
            const unsigned long long below = (1ull << (l + step)) - 1ull;   // lanes 0 .. l+step-1
            const uint32_t cb = (uint32_t)(__popcll(w0 & below) + __popcll(w1 & below) + __popcll(w2 & below) + __popcll(w3 & below));
            if (cb <= i) l += step;
        }
        const unsigned long long below = (1ull << l) - 1ull;
        uint32_t rem = i - (uint32_t)(__popcll(w0 & below) + __popcll(w1 & below) + __popcll(w2 & below) + __popcll(w3 & below));
        const uint32_t b0 = (uint32_t)(w0 >> l) & 1u, b1 = (uint32_t)(w1 >> l) & 1u, b2 = (uint32_t)(w2 >> l) & 1u;
        uint32_t j;
        if (b0 && rem == 0) j = 0;
        else { rem -= b0; if (b1 && rem == 0) j = 1; else { rem -= b1; j = (b2 && rem == 0) ? 2 : 3; } }
        const uint32_t ix = (first + r) * (uint32_t)kRow + sub * 256 + l * 4 + j;
        const uint32_t vb = ix < a.n ? __float_as_uint(v[ix]) : 0u;
        const uint32_t q = before + p;
        if (q < a.cap) { cidx[q] = ix; cval[q] = vb; }
        if (HIST) {
            const uint32_t d = ((vb & 0x7fffffffu) - t_est) >> kFineShift;
            atomicAdd(&hist[d < (uint32_t)kFineBins - 1 ? d : (uint32_t)kFineBins - 1], 1u);
        }
    }
    if (HIST) {
        __syncthreads();
        uint32_t *fine = a.fine_hist + node * kFineBins;
        for (int i = tid; i < kFineBins; i += THREADS) { const uint32_t h = hist[i]; if (h) atomicAdd(&fine[i], h); }
    }
}

template <int ROWS, int THREADS>
static void launch_gather_shape(const SelArgs &g, uint32_t nrows, int batch, hipStream_t st) {
    const dim3 grid((nrows + ROWS - 1) / ROWS, batch);
    // the per-layer selection has one threshold per segment, so no histogram above "the" estimate
    if (g.seg_t) hipLaunchKernelGGL((k_gather<false, ROWS, THREADS>), grid, dim3(THREADS), 0, st, g);
    else hipLaunchKernelGGL((k_gather<true, ROWS, THREADS>), grid, dim3(THREADS), 0, st, g);
}

void launch_gather(const SelArgs &a, int batch, hipStream_t st) {
    const uint32_t nrows = (a.n + kRow - 1) / kRow;
    // the sums per group pay for their launch from about 32 K rows on (measured: at 25 K rows the gather
    // gains 0.5 us from them, at 256 K rows 17 us)
    SelArgs g = a;
    if (nrows > 4 * kSuperRows)
        hipLaunchKernelGGL(k_row_sums, dim3((nrows + kSuperRows - 1) / kSuperRows, batch), dim3(1024), 0, st, g);
    else
        g.supers = 0;
    // 128 rows per block of 1024 threads; measured on the ResNet50-sized workload (4 nodes): 64 rows x 512
    // threads 18.0 us, 64 x 1024 20.2, 128 x 512 19.8, 64 x 256 21.5, this shape 18.2 (the same within noise:
    // what the kernel costs is its chain of dependent memory round trips, not the search work of its busiest block)
    launch_gather_shape<128, 1024>(g, nrows, batch, st);
}

// Adds, for every candidate i < total that passes `member`, one count to hist[digit(d)], where
// d = key - t_est.  Four independent 16-byte loads are issued before their LDS atomics.
template <typename Member, typename Digit>
__device__ __forceinline__ void count_candidates(const uint32_t *cval, uint32_t total, uint32_t t_est,
                                                 uint32_t *hist, Member member, Digit digit) {
    const uint32_t tid = threadIdx.x, nt = blockDim.x, n4 = total >> 2;
    for (uint32_t i = tid; i < n4; i += 4 * nt) {
        u4 x[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t ii = i + r * nt;
            x[r] = ii < n4 ? *(const u4 *)(cval + ii * 4) : (u4){0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (i + r * nt < n4) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t d = (x[r][c] & 0x7fffffffu) - t_est;
                    if (member(d)) atomicAdd(&hist[digit(d)], 1u);
                }
            }
        }
    }
    for (uint32_t i = (n4 << 2) + tid; i < total; i += nt) {
        const uint32_t d = (cval[i] & 0x7fffffffu) - t_est;
        if (member(d)) atomicAdd(&hist[digit(d)], 1u);
    }
}

// ------------------------------------------------------------------ exact k-th key among the candidates

// What the one thread that knows a selection's outcome on the fast path leaves behind: the node's state for the
// kernels after it, the statistics, the word the host polls, and the record of carried thresholds (carry.h).
__device__ __forceinline__ void report_outcome(const SelArgs &a, const int node, Sel *s, const bool ok, const uint32_t thr,
                                               const uint32_t quota, const uint32_t total, const uint32_t t_est) {
    s->fast_ok = ok;
    if (ok) { s->thr = thr; s->quota = quota; }
    atomicAdd(ok ? &a.stats->fast : &a.stats->fallback, 1u);
    // the host sees the outcome without synchronising; a carried threshold that failed says nothing about the data
    if (a.notify && (ok || !s->carried)) st_system32(a.notify + (ok ? 1 : 0), a.notify_value);
    if (a.carry) carry_update(a.carry + node, a.n, a.k, false, ok, s->carried != 0, thr, t_est, total, a.carry_target, a.carry_most);
}



// Block-wide: the exact k-th largest key T* and the number of ties to take, from the fine
// histogram (first level, bins of 2^12 above t_est) and a second-level histogram of the low 12
// bits inside the bin that holds the k-th key.  LOCAL = true: the second level is counted here
// from all gathered candidates; false: it was counted by k_select_level2 into a.level2_hist.
// Returns false (for all threads alike) if count(candidates) < k, candidates were lost, or T*
// lies in the open-ended last bin: then the node is left to the exact path.
template <bool LOCAL>
__device__ bool find_threshold(const SelArgs &a, int node, uint32_t total, uint32_t *hist /*[kFineBins]*/,
                               uint32_t *wave_tmp, uint32_t *res, uint32_t &thr, uint32_t &quota) {
    const Sel *s = a.sel + node;
    const int tid = threadIdx.x, nt = blockDim.x;
    if (total < a.k || total > a.cap) return false;
    const uint32_t t_est = s->t_est;
    for (int i = tid; i < kFineBins; i += nt) hist[i] = a.fine_hist[node * kFineBins + i];
    __syncthreads();
    find_rank_bin<kFineBins>(hist, a.k, wave_tmp, res);
    const uint32_t bin = res[0], need = a.k - res[1];
    __syncthreads();
    if (bin >= (uint32_t)kFineBins - 1) return false;
    if (LOCAL) {
        for (int i = tid; i < kFineBins; i += nt) hist[i] = 0;
        __syncthreads();
        count_candidates(a.cand_val + (size_t)node * a.cap, total, t_est, hist,
                         [=](uint32_t d) { return (d >> kFineShift) == bin; },
                         [=](uint32_t d) { return d & ((1u << kFineShift) - 1); });
    } else {
        for (int i = tid; i < kFineBins; i += nt) hist[i] = a.level2_hist[node * kFineBins + i];
    }
    __syncthreads();
    find_rank_bin<kFineBins>(hist, need, wave_tmp, res);
    thr = t_est + (bin << kFineShift) + res[0];
    quota = need - res[1];
    __syncthreads();
    return true;
}

// Second-level histogram for long candidate lists: many blocks, each counts a slice.
__global__ __launch_bounds__(1024) void k_select_level2(SelArgs a) {
    __shared__ uint32_t hist[kFineBins];
    __shared__ uint32_t wave_tmp[16], res[2];
    const int node = blockIdx.y, tid = threadIdx.x;
    const Sel *s = a.sel + node;
    const uint32_t total = s->cand_total;
    if (total < a.k || total > a.cap) return;
    const uint32_t t_est = s->t_est;
    for (int i = tid; i < kFineBins; i += 1024) hist[i] = a.fine_hist[node * kFineBins + i];
    __syncthreads();
    find_rank_bin<kFineBins>(hist, a.k, wave_tmp, res);
    const uint32_t bin = res[0];
    __syncthreads();
    if (bin >= (uint32_t)kFineBins - 1) return;
    for (int i = tid; i < kFineBins; i += 1024) hist[i] = 0;
    __syncthreads();
    const uint32_t per = (((total + gridDim.x - 1) / gridDim.x) + 3) & ~3u;   // slice, multiple of 4
    const uint32_t lo = blockIdx.x * per;
    if (lo < total) {
        const uint32_t len = total - lo < per ? total - lo : per;
        count_candidates(a.cand_val + (size_t)node * a.cap + lo, len, t_est, hist,
                         [=](uint32_t d) { return (d >> kFineShift) == bin; },
                         [=](uint32_t d) { return d & ((1u << kFineShift) - 1); });
    }
    __syncthreads();
    uint32_t *l2 = a.level2_hist + node * kFineBins;
    for (int i = tid; i < kFineBins; i += 1024) { const uint32_t h = hist[i]; if (h) atomicAdd(&l2[i], h); }
}

// Output for short candidate lists: block b (1024 threads) owns candidates [4096 b, 4096 b + 4096).
// Every block reads ALL candidate keys once (the first 64 K stay in registers), finds T* from
// them itself and counts the selected candidates before its own: no communication between
// blocks.  Writes the selected elements in index order and zeroes them in v (and u).
constexpr int kKeep = 16;   // 16-byte key groups per thread held in registers

__device__ __forceinline__ void output_direct(const SelArgs &a, const int node, const uint32_t block, uint32_t *hist /*[kFineBins]*/,
                                              uint32_t *wave_tmp /*[16]*/, uint32_t *res /*[2]*/) {
    __shared__ uint32_t sh_pg[16], sh_pe[16], sh_tg[16], sh_te[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    Sel *s = a.sel + node;
    const uint32_t total = s->cand_total;
    const uint32_t *cidx = a.cand_idx + (size_t)node * a.cap;
    const uint32_t *cval = a.cand_val + (size_t)node * a.cap;
    const uint32_t base = block * 4096u, e0 = base + tid * 4;
    bool ok = total >= a.k && total <= a.cap;
    const uint32_t n4 = ok ? (total + 3) / 4 : 0u;   // 16-byte groups (the list's capacity is a multiple of 4)

    // independent loads first: the keys, my four positions and values, the fine histogram.
    // The registers hold keys (sign cleared); entries past the end of the list hold 0xffffffff,
    // which no key equals and which lies in no histogram bin.
    auto as_keys = [&](u4 x, uint32_t g4) -> u4 {
#pragma unroll
        for (int c = 0; c < 4; ++c) x[c] = g4 * 4 + c < total ? (x[c] & 0x7fffffffu) : 0xffffffffu;
        return x;
    };
    u4 keys[kKeep];
#pragma unroll
    for (int r = 0; r < kKeep; ++r) {
        const uint32_t g4 = r * 1024 + tid;
        keys[r] = g4 < n4 ? *(const u4 *)(cval + (size_t)g4 * 4) : (u4){0u, 0u, 0u, 0u};
    }
    u4 ci = {0, 0, 0, 0}, cv = {0u, 0u, 0u, 0u};
    if (ok && e0 < total) { ci = *(const u4 *)(cidx + e0); cv = *(const u4 *)(cval + e0); }
#pragma unroll
    for (int r = 0; r < kKeep; ++r) keys[r] = as_keys(keys[r], r * 1024 + tid);
    for (int i = tid; i < kFineBins; i += 1024) hist[i] = a.fine_hist[node * kFineBins + i];
    const uint32_t t_est = s->t_est;
    __syncthreads();

    uint32_t thr = 0, quota = 0;
    if (ok) {   // uniform
        find_rank_bin<kFineBins>(hist, a.k, wave_tmp, res);
        const uint32_t bin = res[0], need = a.k - res[1];
        __syncthreads();
        ok = bin < (uint32_t)kFineBins - 1;   // T* beyond the histogram's range: leave it to the exact path
        if (ok) {
            for (int i = tid; i < kFineBins; i += 1024) hist[i] = 0;
            __syncthreads();
            const uint32_t bin_base = t_est + (bin << kFineShift);   // keys of the bin: bin_base .. bin_base + 4095
            auto tally = [&](uint32_t key) {
                const uint32_t d = key - bin_base;
                if (d < (1u << kFineShift)) atomicAdd(&hist[d], 1u);
            };
#pragma unroll
            for (int r = 0; r < kKeep; ++r) {
#pragma unroll
                for (int c = 0; c < 4; ++c) tally(keys[r][c]);
            }
            for (uint32_t g4 = kKeep * 1024 + tid; g4 < n4; g4 += 1024) {
                const u4 x = as_keys(*(const u4 *)(cval + (size_t)g4 * 4), g4);
#pragma unroll
                for (int c = 0; c < 4; ++c) tally(x[c]);
            }
            __syncthreads();
            find_rank_bin<kFineBins>(hist, need, wave_tmp, res);
            thr = t_est + (bin << kFineShift) + res[0];
            quota = need - res[1];
        }
    }
    if (block == 0 && tid == 0) report_outcome(a, node, s, ok, thr, quota, total, t_est);
    if (!ok || base >= total) return;

    // selected-or-tied counts among the candidates before mine: groups r*1024 + tid, r < block
    // (all of those lie before the end of the list, so none is the 0xffffffff filler)
    uint32_t pg = 0, pe = 0;
#pragma unroll
    for (int r = 0; r < kKeep; ++r) {
        if (r < (int)block) {
#pragma unroll
            for (int c = 0; c < 4; ++c) { pg += keys[r][c] > thr; pe += keys[r][c] == thr; }
        }
    }
    for (uint32_t r = kKeep; r < block; ++r) {
        const u4 x = *(const u4 *)(cval + (size_t)(r * 1024 + tid) * 4);
#pragma unroll
        for (int c = 0; c < 4; ++c) { const uint32_t key = x[c] & 0x7fffffffu; pg += key > thr; pe += key == thr; }
    }
    pg = wave_sum(pg); pe = wave_sum(pe);
    uint32_t lg = 0, le = 0, tg = 0, te = 0;
    bool fg[4], fe[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t key = cv[j] & 0x7fffffffu;
        fg[j] = e0 + j < total && key > thr;
        fe[j] = e0 + j < total && key == thr;
        const unsigned long long mg = __ballot(fg[j]), me = __ballot(fe[j]);
        lg += lanes_below(mg); tg += (uint32_t)__popcll(mg);
        le += lanes_below(me); te += (uint32_t)__popcll(me);
    }
    if (lane == 0) { sh_pg[wave] = pg; sh_pe[wave] = pe; sh_tg[wave] = tg; sh_te[wave] = te; }
    __syncthreads();
    // flagged elements before my first one: all of the earlier blocks' candidates, the lower
    // wavefronts of this block, the lower lanes of this wavefront
    uint32_t cg = lg, ce = le;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        cg += sh_pg[w]; ce += sh_pe[w];
        if (w < wave) { cg += sh_tg[w]; ce += sh_te[w]; }
    }

    if (block == (total - 1) / 4096 && tid == 1023) {
        // the last thread of the last block sees everything: the selection must add up to k
        uint32_t g_all = cg, e_all = ce;
        for (int j = 0; j < 4; ++j) { g_all += fg[j]; e_all += fe[j]; }
        if (g_all + (e_all < quota ? e_all : quota) != a.k) atomicAdd(&a.stats->errors, 1u);
    }
    float *v = a.v + (size_t)node * a.stride;
    float *u = a.u ? a.u + (size_t)node * a.stride : nullptr;
    uint32_t *oidx = a.out_idx + (size_t)node * a.k;
    float *oval = a.out_vals + (size_t)node * a.k;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (fg[j] || (fe[j] && ce < quota)) {
            const uint32_t o = cg + (ce < quota ? ce : quota);
            if (o < a.k) { oidx[o] = ci[j]; oval[o] = __uint_as_float(cv[j]); }
            else atomicAdd(&a.stats->errors, 1u);
            v[ci[j]] = 0.0f;
            if (u) u[ci[j]] = 0.0f;
        }
        cg += fg[j]; ce += fe[j];
    }
}

// ------------------------------------------------------------------ ordered output of the exact path

// The threshold T* and the tie quota are known.  The selected elements (key > T*, and the first
// `quota` elements with key == T*) are written to the output in index order and zeroed in v
// (and u), reading v itself.  Every block of the node (THREADS threads) owns a run of consecutive chunks of
// 16 * THREADS elements: kRows rows of 4 * THREADS, four consecutive elements per thread and row.
// load_chunk: the value bits of this thread's 16 elements of a chunk and their flags (bit r*4+j).
template <bool VEC, int THREADS>
__device__ __forceinline__ void load_chunk(const float *__restrict__ v, const uint32_t base, const uint32_t n,
                                           const uint32_t thr, uint32_t (&bits)[kRows][4], uint32_t &gtm, uint32_t &eqm) {
    const int tid = threadIdx.x;
    gtm = 0; eqm = 0;
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const uint32_t e0 = base + r * (THREADS * 4) + tid * 4;
        f4 vv = {0.f, 0.f, 0.f, 0.f};
        if (VEC && e0 + 3 < n) vv = *(const f4 *)(v + e0);
        else { for (int j = 0; j < 4; ++j) if (e0 + j < n) vv[j] = v[e0 + j]; }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bits[r][j] = __float_as_uint(vv[j]);
            const bool valid = e0 + j < n;
            const uint32_t key = bits[r][j] & 0x7fffffffu;
            gtm |= (uint32_t)(valid && key > thr) << (r * 4 + j);
            eqm |= (uint32_t)(valid && key == thr) << (r * 4 + j);
        }
    }
}

// count_run: the counts of "greater" and "equal" over run number `run` of the node, stored as
// totals[run] = greater << 32 | equal.  emit_run (once all runs are counted): the counts of the runs before
// this one place the run in the output; the run is then written chunk by chunk with a running offset.
template <bool VEC, int THREADS>
__device__ __forceinline__ void count_run(const SelArgs &a, const int node, const uint32_t thr,
                                          const uint32_t c_lo, const uint32_t c_hi, const uint32_t run) {
    constexpr int W = THREADS / 64;
    __shared__ uint32_t sh_cnt[2][W];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *v = a.v + (size_t)node * a.stride;
    uint32_t g = 0, e = 0;
    for (uint32_t chunk = c_lo; chunk < c_hi; ++chunk) {
        uint32_t bits[kRows][4], gtm, eqm;
        load_chunk<VEC, THREADS>(v, chunk * (uint32_t)(16 * THREADS), a.n, thr, bits, gtm, eqm);
        g += (uint32_t)__popc(gtm); e += (uint32_t)__popc(eqm);
    }
    g = wave_sum(g); e = wave_sum(e);
    if (lane == 0) { sh_cnt[0][wave] = g; sh_cnt[1][wave] = e; }
    __syncthreads();
    if (tid == 0) {
        uint32_t bg = 0, be = 0;
        for (int w = 0; w < W; ++w) { bg += sh_cnt[0][w]; be += sh_cnt[1][w]; }
        st_agent(&a.status_exact[(size_t)node * a.status_exact_stride + run], ((unsigned long long)bg << 32) | be);
    }
}

template <bool VEC, int THREADS>
__device__ __forceinline__ void emit_run(const SelArgs &a, const int node, const uint32_t thr, const uint32_t quota,
                                         const uint32_t c_lo, const uint32_t c_hi, const uint32_t nchunks,
                                         const uint32_t run) {
    constexpr int W = THREADS / 64;
    __shared__ uint32_t sh_gt[kRows][W], sh_eq[kRows][W];
    __shared__ uint32_t sh_pre[2][W];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t off = (size_t)node * a.stride;
    float *u = a.u ? a.u + off : nullptr;
    float *v = a.v + off;
    uint32_t *oidx = a.out_idx + (size_t)node * a.k;
    float *oval = a.out_vals + (size_t)node * a.k;
    // selected-or-tied elements of the runs before this one (their totals are complete)
    const unsigned long long *totals = a.status_exact + (size_t)node * a.status_exact_stride;
    uint32_t pg = 0, pe = 0;
    __syncthreads();   // a block that emits several runs: the previous run's readers of sh_pre are done
    for (uint32_t b = tid; b < run; b += THREADS) {
        const unsigned long long t = ld_agent(&totals[b]);
        pg += (uint32_t)(t >> 32); pe += (uint32_t)t;
    }
    pg = wave_sum(pg); pe = wave_sum(pe);
    if (lane == 0) { sh_pre[0][wave] = pg; sh_pre[1][wave] = pe; }
    __syncthreads();
    uint32_t pre_gt = 0, pre_eq = 0;
#pragma unroll
    for (int w = 0; w < W; ++w) { pre_gt += sh_pre[0][w]; pre_eq += sh_pre[1][w]; }

    for (uint32_t chunk = c_lo; chunk < c_hi; ++chunk) {   // c_lo, c_hi: the same for the whole block
        const uint32_t base = chunk * (uint32_t)(16 * THREADS);
        uint32_t bits[kRows][4], gtm, eqm;
        load_chunk<VEC, THREADS>(v, base, a.n, thr, bits, gtm, eqm);
        // position of my flagged elements inside the chunk, in index order (row, wave, lane, j)
        uint32_t lane_gt[kRows], lane_eq[kRows];
        __syncthreads();   // the previous chunk's readers of sh_gt / sh_eq are done
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            uint32_t lg = 0, le = 0, tg = 0, te = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const unsigned long long mg = __ballot((gtm >> (r * 4 + j)) & 1u);
                const unsigned long long me = __ballot((eqm >> (r * 4 + j)) & 1u);
                lg += lanes_below(mg); tg += (uint32_t)__popcll(mg);
                le += lanes_below(me); te += (uint32_t)__popcll(me);
            }
            lane_gt[r] = lg; lane_eq[r] = le;
            if (lane == 0) { sh_gt[r][wave] = tg; sh_eq[r][wave] = te; }
        }
        __syncthreads();
        uint32_t off_gt[kRows], off_eq[kRows], blk_gt = 0, blk_eq = 0;
        if constexpr (W <= 4) {
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
#pragma unroll
                for (int w = 0; w < W; ++w) {
                    if (w == wave) { off_gt[r] = blk_gt; off_eq[r] = blk_eq; }
                    blk_gt += sh_gt[r][w]; blk_eq += sh_eq[r][w];
                }
            }
        } else {
            // many wavefronts: lane w takes wavefront w's totals and the sums go over the lanes (reading all
            // kRows x W totals into registers at once is what a block of 16 wavefronts has no room for)
#pragma unroll 1
            for (int r = 0; r < kRows; ++r) {
                const uint32_t tg = lane < W ? sh_gt[r][lane] : 0u, te = lane < W ? sh_eq[r][lane] : 0u;
                off_gt[r] = blk_gt + wave_sum(lane < wave ? tg : 0u);
                off_eq[r] = blk_eq + wave_sum(lane < wave ? te : 0u);
                blk_gt += wave_sum(tg); blk_eq += wave_sum(te);
            }
        }
        if (tid == 0 && chunk == nchunks - 1) {   // the last chunk of the node sees everything: the selection must add up to k
            const uint32_t te = pre_eq + blk_eq;
            if (pre_gt + blk_gt + (te < quota ? te : quota) != a.k) atomicAdd(&a.stats->errors, 1u);
        }
        if ((gtm | eqm) != 0) {
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
                uint32_t cg = pre_gt + off_gt[r] + lane_gt[r];
                uint32_t ce = pre_eq + off_eq[r] + lane_eq[r];
                const uint32_t e0 = base + r * (THREADS * 4) + tid * 4;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool fg = (gtm >> (r * 4 + j)) & 1u, fe = (eqm >> (r * 4 + j)) & 1u;
                    if (fg || (fe && ce < quota)) {
                        const uint32_t o = cg + (ce < quota ? ce : quota);
                        if (o < a.k) { oidx[o] = e0 + j; oval[o] = __uint_as_float(bits[r][j]); }
                        else atomicAdd(&a.stats->errors, 1u);
                        v[e0 + j] = 0.0f;
                        if (u) u[e0 + j] = 0.0f;
                    }
                    cg += fg; ce += fe;
                }
            }
        }
        pre_gt += blk_gt; pre_eq += blk_eq;   // block-uniform
    }
}

// Long candidate lists, after k_select_level2.  Two kernels with nothing exchanged between the
// blocks of either: k_count_chunks derives T* and the tie quota from the two histograms (every
// block, same result in all) and counts, for each 4096-candidate chunk, the keys above T* and
// the keys equal to it; k_emit_scanned adds up the counts of the chunks before its own, which
// places its chunk's selected elements in the output, in index order.
constexpr int kCountChunks = 4;   // chunks per block of k_count_chunks

__global__ __launch_bounds__(1024) void k_count_chunks(SelArgs a) {
    __shared__ uint32_t hist[kFineBins];
    __shared__ uint32_t wave_tmp[16], res[2];
    __shared__ uint32_t sh_gt[kCountChunks][16], sh_eq[kCountChunks][16];
    const int node = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    Sel *s = a.sel + node;
    const uint32_t total = s->cand_total;
    const uint32_t *cval = a.cand_val + (size_t)node * a.cap;
    const uint32_t base = blockIdx.x * (uint32_t)(kCountChunks * kChunk);
    const bool in_range = total <= a.cap;
    // the keys first, so that the loads are under way while the threshold is worked out
    u4 x[kCountChunks];
#pragma unroll
    for (int c = 0; c < kCountChunks; ++c) {
        const uint32_t e0 = base + c * kChunk + tid * 4;   // the list's capacity is a multiple of 4
        x[c] = (in_range && e0 < total) ? *(const u4 *)(cval + e0) : (u4){0u, 0u, 0u, 0u};
    }
    uint32_t thr = 0, quota = 0;
    const bool ok = find_threshold<false>(a, node, total, hist, wave_tmp, res, thr, quota);
    if (blockIdx.x == 0 && tid == 0) report_outcome(a, node, s, ok, thr, quota, total, s->t_est);
    if (!ok || base >= total) return;
#pragma unroll
    for (int c = 0; c < kCountChunks; ++c) {
        const uint32_t e0 = base + c * kChunk + tid * 4;
        uint32_t gt = 0, eq = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t key = x[c][j] & 0x7fffffffu;
            gt += e0 + j < total && key > thr;
            eq += e0 + j < total && key == thr;
        }
        gt = wave_sum(gt); eq = wave_sum(eq);
        if (lane == 0) { sh_gt[c][wave] = gt; sh_eq[c][wave] = eq; }
    }
    __syncthreads();
    if (tid < kCountChunks) {
        const uint32_t chunk = blockIdx.x * kCountChunks + tid;
        if (chunk * (uint32_t)kChunk < total) {
            uint32_t gt = 0, eq = 0;
            for (int w = 0; w < 16; ++w) { gt += sh_gt[tid][w]; eq += sh_eq[tid][w]; }
            a.status_cand[(size_t)node * a.status_cand_stride + chunk] = ((unsigned long long)gt << 32) | eq;
        }
    }
}

__global__ __launch_bounds__(1024) void k_emit_scanned(SelArgs a) {
    __shared__ uint32_t sh_pg[16], sh_pe[16], sh_tg[16], sh_te[16];
    const int node = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const Sel *s = a.sel + node;
    const uint32_t total = s->cand_total;
    const uint32_t chunk = blockIdx.x, base = chunk * (uint32_t)kChunk, e0 = base + tid * 4;
    if (!s->fast_ok || base >= total) return;   // uniform; fast_ok implies k <= total <= cap
    const uint32_t thr = s->thr, quota = s->quota;
    const uint32_t *cidx = a.cand_idx + (size_t)node * a.cap;
    const uint32_t *cval = a.cand_val + (size_t)node * a.cap;
    const unsigned long long *counts = a.status_cand + (size_t)node * a.status_cand_stride;
    u4 ci = {0, 0, 0, 0}, cv = {0u, 0u, 0u, 0u};
    if (e0 < total) { ci = *(const u4 *)(cidx + e0); cv = *(const u4 *)(cval + e0); }
    uint32_t pg = 0, pe = 0;
    for (uint32_t c = tid; c < chunk; c += 1024) {
        const unsigned long long w = counts[c];
        pg += (uint32_t)(w >> 32); pe += (uint32_t)w;
    }
    pg = wave_sum(pg); pe = wave_sum(pe);
    uint32_t lg = 0, le = 0, tg = 0, te = 0;
    bool fg[4], fe[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t key = cv[j] & 0x7fffffffu;
        fg[j] = e0 + j < total && key > thr;
        fe[j] = e0 + j < total && key == thr;
        const unsigned long long mg = __ballot(fg[j]), me = __ballot(fe[j]);
        lg += lanes_below(mg); tg += (uint32_t)__popcll(mg);
        le += lanes_below(me); te += (uint32_t)__popcll(me);
    }
    if (lane == 0) { sh_pg[wave] = pg; sh_pe[wave] = pe; sh_tg[wave] = tg; sh_te[wave] = te; }
    __syncthreads();
    // flagged elements before my first one: the earlier chunks, the lower wavefronts of this
    // block, the lower lanes of this wavefront
    uint32_t cg = lg, ce = le;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        cg += sh_pg[w]; ce += sh_pe[w];
        if (w < wave) { cg += sh_tg[w]; ce += sh_te[w]; }
    }
    if (chunk == (total - 1) / (uint32_t)kChunk && tid == 1023) {
        // the last thread of the last chunk sees everything: the selection must add up to k
        uint32_t g_all = cg, e_all = ce;
        for (int j = 0; j < 4; ++j) { g_all += fg[j]; e_all += fe[j]; }
        if (g_all + (e_all < quota ? e_all : quota) != a.k) atomicAdd(&a.stats->errors, 1u);
    }
    float *v = a.v + (size_t)node * a.stride;
    float *u = a.u ? a.u + (size_t)node * a.stride : nullptr;
    uint32_t *oidx = a.out_idx + (size_t)node * a.k;
    float *oval = a.out_vals + (size_t)node * a.k;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (fg[j] || (fe[j] && ce < quota)) {
            const uint32_t o = cg + (ce < quota ? ce : quota);
            if (o < a.k) { oidx[o] = ci[j]; oval[o] = __uint_as_float(cv[j]); }
            else atomicAdd(&a.stats->errors, 1u);
            v[ci[j]] = 0.0f;
            if (u) u[ci[j]] = 0.0f;
        }
        cg += fg[j]; ce += fe[j];
    }
}

// ------------------------------------------------------------------ exact path

// Radix select of the exact k-th largest key over all of v (digits of 11, 10 and 10 bits: each
// pass histograms one digit of the keys that match the digits fixed so far, the next digit is then
// fixed from the histogram), followed by the ordered output compaction of v with that key.
// Three forms:
//  * k_exact_block: ONE block per node does all of it (three passes over the node's v with an LDS
//    histogram, then the ordered output): short vectors.
//  * k_exact: one launch of several blocks per node that share the phases out through tickets: the
//    fall-back of the fast path (it exits at once for the nodes the fast path served, which is nearly
//    always: the launch then costs little more than an empty one).
//  * k_exact_step: the same phases as five launches of many blocks, for exact selection chosen
//    outright on long vectors; the kernel boundaries are the only exchange between blocks.

// counts digit `pass` of the keys whose higher digits equal `prefix` into hist (LDS), this block's share of v
template <bool VEC, int THREADS>
__device__ __forceinline__ void radix_tally(const float *__restrict__ v, const uint32_t n, const uint32_t first,
                                            const uint32_t nthreads, const int pass, const uint32_t prefix,
                                            uint32_t *hist) {
    auto count = [&](uint32_t key) {
        if (pass == 0) atomicAdd(&hist[key >> 20], 1u);
        else if (pass == 1) { if ((key >> 20) == prefix) atomicAdd(&hist[(key >> 10) & 1023u], 1u); }
        else { if ((key >> 10) == prefix) atomicAdd(&hist[key & 1023u], 1u); }
    };
    if (VEC) {
        const uint32_t n4 = n >> 2;
        for (uint32_t i = first; i < n4; i += 4 * nthreads) {   // four 16-byte loads in flight per thread
            f4 vv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t ii = i + r * nthreads;   // < 2^29 + 2^22: no wrap
                vv[r] = ii < n4 ? ((const f4 *)v)[ii] : (f4){0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (i + r * nthreads < n4) {
                    count(key_of(vv[r].x)); count(key_of(vv[r].y)); count(key_of(vv[r].z)); count(key_of(vv[r].w));
                }
            }
        }
        for (uint32_t i = (n4 << 2) + first; i < n; i += nthreads) count(key_of(v[i]));
    } else {
        for (uint32_t i = first; i < n; i += nthreads) count(key_of(v[i]));
    }
}

// One pass over share `run` of `nruns` of the node's v: the histogram of digit `pass` among the keys whose
// higher digits equal `prefix`, counted in LDS and added to the node's histogram of that pass.
template <bool VEC, int THREADS>
__device__ __forceinline__ void radix_count(const SelArgs &a, const int node, const int pass, const uint32_t prefix,
                                            uint32_t *hist /*[kRadixBins]*/, const uint32_t run, const uint32_t nruns) {
    const int tid = threadIdx.x;
    const int nb = pass == 0 ? kRadixBins : 1024;
    uint32_t *gh = a.radix_hist + (node * 3 + pass) * kRadixBins;
    for (int i = tid; i < nb; i += THREADS) hist[i] = 0;
    __syncthreads();
    radix_tally<VEC, THREADS>(a.v + (size_t)node * a.stride, a.n, run * THREADS + tid, nruns * THREADS, pass, prefix, hist);
    __syncthreads();
    for (int i = tid; i < nb; i += THREADS) { const uint32_t h = hist[i]; if (h) atomicAdd(&gh[i], h); }
}

// From a finished histogram of `pass` in LDS: the digit that holds the rank-th largest key, appended to prefix;
// rank becomes the rank inside that digit's keys.  Block-wide.
__device__ __forceinline__ void radix_digit(const int pass, const uint32_t *hist, uint32_t *wave_tmp, uint32_t *res,
                                            uint32_t &prefix, uint32_t &rank) {
    if (pass == 0) find_rank_bin<kRadixBins>(hist, rank, wave_tmp, res);
    else find_rank_bin<1024>(hist, rank, wave_tmp, res);
    const uint32_t digit = res[0] == 0xffffffffu ? 0u : res[0];
    rank -= res[1];
    prefix = pass == 0 ? digit : ((prefix << 10) | digit);
    __syncthreads();
}

// Once every block's counts of `pass` are in the node's histogram (the launch before): fix the next digit.
template <int THREADS>
__device__ __forceinline__ void radix_fix(const SelArgs &a, const int node, const int pass, uint32_t *hist,
                                          uint32_t *wave_tmp, uint32_t *res, uint32_t &prefix, uint32_t &rank) {
    const int tid = threadIdx.x;
    const int nb = pass == 0 ? kRadixBins : 1024;
    const uint32_t *gh = a.radix_hist + (node * 3 + pass) * kRadixBins;
    for (int i = tid; i < kRadixBins; i += THREADS) hist[i] = i < nb ? ld_agent32(&gh[i]) : 0u;
    __syncthreads();
    radix_digit(pass, hist, wave_tmp, res, prefix, rank);
}

// run number `run` of `nruns` in the ordered output: the chunks [run * per, (run + 1) * per) of the node
template <int THREADS>
__device__ __forceinline__ void block_run(const SelArgs &a, const uint32_t run, const uint32_t nruns, uint32_t &c_lo,
                                          uint32_t &c_hi, uint32_t &nchunks) {
    nchunks = (a.n + 16u * THREADS - 1) / (16u * THREADS);   // a chunk: 16 elements per thread
    const uint32_t per = (nchunks + nruns - 1) / nruns;
    c_lo = run * per < nchunks ? run * per : nchunks;
    c_hi = c_lo + per < nchunks ? c_lo + per : nchunks;
}

// One block of 1024 threads per node (grid (1, nodes)), everything in that block.
template <bool VEC>
__global__ __launch_bounds__(1024) void k_exact_block(SelArgs a) {
    __shared__ uint32_t hist[kRadixBins];
    __shared__ uint32_t wave_tmp[16], res[2];
    const int node = blockIdx.y, tid = threadIdx.x;
    Sel *s = a.sel + node;
    if (!a.force && s->fast_ok) return;   // the same for the whole block
    if (a.force) {   // no sampling kernel ran in this call: the next call's state set is cleared here
        for (uint32_t i = blockIdx.y * 1024u + tid; i < a.next_words; i += gridDim.y * 1024u) a.next_state[i] = 0;
    }
    const float *v = a.v + (size_t)node * a.stride;
    uint32_t prefix = 0, rank = a.k;
    for (int pass = 0; pass < 3; ++pass) {
        for (int i = tid; i < kRadixBins; i += 1024) hist[i] = 0;
        __syncthreads();
        radix_tally<VEC, 1024>(v, a.n, tid, 1024u, pass, prefix, hist);
        __syncthreads();
        radix_digit(pass, hist, wave_tmp, res, prefix, rank);
    }
    // prefix is now the full key T*; rank the number of ties to take
    if (tid == 0) { s->thr = prefix; s->quota = rank; carry_lapse(a, node); }
    const uint32_t nchunks = (a.n + 16383u) / 16384u;
    emit_run<VEC, 1024>(a, node, prefix, rank, 0u, nchunks, nchunks, 0u);
}

// The same phases in one launch of several blocks per node, for the fast path's fall-back on long vectors (it
// exits at once for the nodes the fast path served).  The shares of the five phases (three radix passes,
// count, output; R shares each) are handed out through a ticket counter, phase by phase, to whichever blocks
// are running; a block that draws a share of phase p first waits until the R shares of phase p - 1 are
// complete.  Every share it waits for was drawn before its own, hence by a block that is running and that
// waits, in turn, only for shares drawn still earlier: the waits end whatever number of the kernel's blocks
// the device holds at a time, and whatever else runs beside them (there is no condition on residency; one
// block alone would work through all the shares).  The waits are bounded all the same: an expired wait is
// counted as a device error (lgc_stats) and ends every other wait within a few polls.
__device__ __forceinline__ bool phase_wait(const SelArgs &a, const Ctr *c, const int phase, const uint32_t shares) {
    __shared__ uint32_t sh_ok;
    if (threadIdx.x == 0) {
        uint32_t spins = 0, ok = 1;
        while (ld_agent32(&c->done[phase]) < shares) {
            if (++spins > a.spin_limit) { atomicAdd(&a.stats->errors, 1u); ok = 0; break; }
            if ((spins & 255u) == 0 && ld_agent32(&a.stats->errors) != 0) { ok = 0; break; }
            __builtin_amdgcn_s_sleep(8);
        }
        sh_ok = ok;
    }
    __syncthreads();
    return __builtin_amdgcn_readfirstlane(sh_ok) != 0;   // wave-uniform for the compiler: callers branch on it
}

// Completion of a share.  Every wavefront waits until its own stores and atomics have been acknowledged (a
// wait, no cache operation), the block barrier collects them, and ONE thread issues the device-scope release
// (the write-back of this XCD's L2) before it counts the share.  No acquire on the other side: everything that
// crosses blocks (the summed histograms, the runs' counts) is read with device-scope atomic loads, which do
// not go through the non-coherent caches.
__device__ __forceinline__ void phase_done(Ctr *c, const int phase) {
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
    if (threadIdx.x == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        atomicAdd(&c->done[phase], 1u);
    }
}

// The ticket loop of one block; `shares` = shares per phase = blocks of the node that run this loop.
template <bool VEC, int THREADS>
__device__ __forceinline__ void exact_tickets(const SelArgs &a, const int node, const uint32_t shares, uint32_t *hist /*[kRadixBins]*/,
                                              uint32_t *wave_tmp /*[THREADS / 64]*/, uint32_t *res /*[2]*/) {
    __shared__ uint32_t sh_ticket;
    const int tid = threadIdx.x;
    Sel *s = a.sel + node;
    Ctr *c = a.ctr + node;
    uint32_t prefix = 0, rank = a.k;
    int fixed = 0;                       // digits of T* this block has worked out so far
    for (;;) {
        __syncthreads();                 // the previous round's readers of sh_ticket are done
        if (tid == 0) sh_ticket = atomicAdd(&c->ticket, 1u);
        __syncthreads();
        const uint32_t t = __builtin_amdgcn_readfirstlane(sh_ticket);
        if (t >= 5u * shares) break;
        const int phase = (int)(t / shares);
        const uint32_t run = t % shares;
        if (phase > 0 && !phase_wait(a, c, phase - 1, shares)) return;   // a wait expired somewhere: give up, lgc_stats reports it
        for (; fixed < (phase < 3 ? phase : 3); ++fixed) radix_fix<THREADS>(a, node, fixed, hist, wave_tmp, res, prefix, rank);
        if (phase < 3) {
            radix_count<VEC, THREADS>(a, node, phase, prefix, hist, run, shares);
        } else {
            uint32_t c_lo, c_hi, nchunks;
            block_run<THREADS>(a, run, shares, c_lo, c_hi, nchunks);
            if (phase == 3) {
                if (run == 0 && tid == 0) { s->thr = prefix; s->quota = rank; carry_lapse(a, node); }   // prefix is the full key T*, rank the ties to take
                count_run<VEC, THREADS>(a, node, prefix, c_lo, c_hi, run);
            } else {
                emit_run<VEC, THREADS>(a, node, prefix, rank, c_lo, c_hi, nchunks, run);
            }
        }
        phase_done(c, phase);
    }
}

// Exact selection as one launch of its own: about one block of 1024 threads per compute unit, shared by the nodes.
template <bool VEC>
__global__ __launch_bounds__(1024) void k_exact(SelArgs a) {
    __shared__ uint32_t hist[kRadixBins];
    __shared__ uint32_t wave_tmp[16], res[2];
    const int node = blockIdx.y, tid = threadIdx.x;
    if (!a.force && a.sel[node].fast_ok) return;
    if (a.force) {   // no sampling kernel ran in this call: the next call's state set is cleared here
        const uint32_t gtid = blockIdx.x * 1024u + tid, nthreads = gridDim.x * 1024u, all = gridDim.y * nthreads;
        for (uint32_t i = blockIdx.y * nthreads + gtid; i < a.next_words; i += all) a.next_state[i] = 0;
    }
    exact_tickets<VEC, 1024>(a, node, gridDim.x, hist, wave_tmp, res);
}

// Output for short candidate lists and the fall-back in ONE launch: blocks 0 .. out_blocks - 1 of a node (grid y)
// are the output blocks (output_direct), the blocks after them stand by for the exact path.  Each of those decides
// for itself, from the candidate count and the fine histogram, whether the output blocks can serve the node
// (the same test they make: enough candidates, none lost, T* inside the histogram's range) and leaves if so,
// which is nearly always and costs them one block-wide search; otherwise they run the ticket loop.  A launch
// of its own for the fall-back costs 4.5 us per call even when it has nothing to do.
template <bool VEC>
__global__ __launch_bounds__(1024) void k_output_or_exact(SelArgs a, uint32_t out_blocks) {
    __shared__ uint32_t hist[kFineBins];
    __shared__ uint32_t wave_tmp[16], res[2];
    // grid (nodes, blocks per node): blocks are handed out with x fastest, so every node's output blocks are on the
    // device before the first stand-by block (a compute unit holds one block of this kernel at a time)
    // (measured: 367.1 against 368.0 us per call with the nodes in y and the blocks in x)
    const int node = blockIdx.x, tid = threadIdx.x;
    if (blockIdx.y < out_blocks) { output_direct(a, node, blockIdx.y, hist, wave_tmp, res); return; }
    const uint32_t total = a.sel[node].cand_total;
    bool ok = total >= a.k && total <= a.cap;
    if (ok) {   // the same for the whole block
        for (int i = tid; i < kFineBins; i += 1024) hist[i] = a.fine_hist[node * kFineBins + i];
        __syncthreads();
        find_rank_bin<kFineBins>(hist, a.k, wave_tmp, res);
        ok = res[0] < (uint32_t)kFineBins - 1;
        __syncthreads();
    }
    if (ok) return;
    exact_tickets<VEC, 1024>(a, node, gridDim.y - out_blocks, hist, wave_tmp, res);
}

// Five launches: step 0..2: the radix pass of that digit (the digits before it are fixed again from their
// finished histograms: a few microseconds, no exchange); step 3: T*, the tie quota and the counts of every
// block's run; step 4: the ordered output.  The blocks need not be resident together, and their number is
// chosen for the passes over v alone.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_exact_step(SelArgs a, int step) {
    __shared__ uint32_t hist[kRadixBins];
    __shared__ uint32_t wave_tmp[kWaves], res[2];
    const int node = blockIdx.y, tid = threadIdx.x;
    Sel *s = a.sel + node;
    if (step == 0) {   // forced path only: the next call's state set is cleared here
        const uint32_t gtid = blockIdx.x * kBlock + tid, nthreads = gridDim.x * kBlock, all = gridDim.y * nthreads;
        for (uint32_t i = blockIdx.y * nthreads + gtid; i < a.next_words; i += all) a.next_state[i] = 0;
    }
    uint32_t c_lo, c_hi, nchunks;
    block_run<kBlock>(a, blockIdx.x, gridDim.x, c_lo, c_hi, nchunks);
    if (step == 4) {
        emit_run<VEC, kBlock>(a, node, s->thr, s->quota, c_lo, c_hi, nchunks, blockIdx.x);
        return;
    }
    uint32_t prefix = 0, rank = a.k;
    for (int pass = 0; pass < (step < 3 ? step : 3); ++pass) radix_fix<kBlock>(a, node, pass, hist, wave_tmp, res, prefix, rank);
    if (step < 3) {
        radix_count<VEC, kBlock>(a, node, step, prefix, hist, blockIdx.x, gridDim.x);
        return;
    }
    if (blockIdx.x == 0 && tid == 0) { s->thr = prefix; s->quota = rank; carry_lapse(a, node); }
    count_run<VEC, kBlock>(a, node, prefix, c_lo, c_hi, blockIdx.x);
}

constexpr uint64_t kStepMinElems = 1ull << 20;   // forced exact selection of this many elements (all nodes) and more: five launches
constexpr uint32_t kBlockMaxElems = 1u << 15;    // vectors up to this length: one block per node does everything

void launch_exact(const SelArgs &a, int batch, bool vec, int cus, hipStream_t st) {
    const uint32_t chunks = (a.n + kChunk - 1) / kChunk;
    if (a.force && (uint64_t)a.n * batch >= kStepMinElems) {
        // five launches: about four blocks per compute unit in all (fewer make a block's share of a pass long,
        // more make the histogram flushes dear)
        uint32_t per_node = (uint32_t)(4 * cus / batch);
        if (per_node > chunks) per_node = chunks;
        if (per_node < 1) per_node = 1;
        dim3 grid2(per_node, batch);
        for (int step = 0; step < 5; ++step) {
            if (vec) hipLaunchKernelGGL(k_exact_step<true>, grid2, dim3(kBlock), 0, st, a, step);
            else hipLaunchKernelGGL(k_exact_step<false>, grid2, dim3(kBlock), 0, st, a, step);
        }
        return;
    }
    if (a.n <= kBlockMaxElems) {
        if (vec) hipLaunchKernelGGL(k_exact_block<true>, dim3(1, batch), dim3(1024), 0, st, a);
        else hipLaunchKernelGGL(k_exact_block<false>, dim3(1, batch), dim3(1024), 0, st, a);
        return;
    }
    // one launch, about one block of 1024 threads per compute unit shared by the nodes: each block more makes the
    // phase changes dearer (a device-scope release per share), each block less the five passes over v slower
    uint32_t per_node = (uint32_t)(cus / batch);
    const uint32_t shares_max = (a.n + 16383u) / 16384u;
    if (per_node > shares_max) per_node = shares_max;
    if (per_node < 1) per_node = 1;
    dim3 grid(per_node, batch);
    if (vec) hipLaunchKernelGGL(k_exact<true>, grid, dim3(1024), 0, st, a);
    else hipLaunchKernelGGL(k_exact<false>, grid, dim3(1024), 0, st, a);
}

// direct = true: short candidate lists (each block reads the whole list; the fall-back rides in the same
// launch); false: long lists (second-level histogram by many blocks, counts per chunk, output).  Returns
// whether the fall-back to the exact path is part of what was launched.
bool launch_output_from_candidates(const SelArgs &a, int batch, bool direct, bool vec, int cus, hipStream_t st) {
    if (direct) {
        const uint32_t out_blocks = (a.cap + 4095) / 4096;
        // stand-by blocks of 1024 threads, about one per compute unit shared by the nodes, as in the stand-alone
        // launch.  Measured on tie-heavy input, where every call falls back (4 nodes x 25.6 M elements / 8 nodes x
        // 67 M; the exact path chosen outright: 0.96 / 4.9 ms): a quarter as many blocks 3.04 / 15.6 ms, half as
        // many 1.85 / 9.4 ms, this many 1.31 / 6.4 ms, twice as many 1.37 / 6.5 ms; a call that does not fall back
        // takes 368.3, 368.9, 369.0 and 372.0 us with them (the blocks decide and leave while the output blocks work).
        const uint32_t chunks = (a.n + 16383u) / 16384u;
        uint32_t standby = (uint32_t)(cus / batch);
        if (standby > chunks) standby = chunks;
        if (standby < 1) standby = 1;
        const dim3 grid(batch, out_blocks + standby);
        if (vec) hipLaunchKernelGGL(k_output_or_exact<true>, grid, dim3(1024), 0, st, a, out_blocks);
        else hipLaunchKernelGGL(k_output_or_exact<false>, grid, dim3(1024), 0, st, a, out_blocks);
        return true;
    }
    uint32_t blocks = (a.cap + 16383) / 16384;
    if (blocks > 256) blocks = 256;
    hipLaunchKernelGGL(k_select_level2, dim3(blocks, batch), dim3(1024), 0, st, a);
    const uint32_t chunks = (a.cap + kChunk - 1) / kChunk;
    hipLaunchKernelGGL(k_count_chunks, dim3((chunks + kCountChunks - 1) / kCountChunks, batch), dim3(1024), 0, st, a);
    hipLaunchKernelGGL(k_emit_scanned, dim3(chunks, batch), dim3(1024), 0, st, a);
    return false;
}

}  // namespace lgc
