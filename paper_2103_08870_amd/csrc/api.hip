// Host side of liblgc: the C ABI declared in include/lgc.h.  Validates arguments, owns the
// scratch memory, chooses the selection path and enqueues the kernels.  Nothing here
// synchronises or copies to the host on the hot path.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "lgc_internal.h"

using namespace lgc;

struct lgc_ctx {
    int device = 0;
    uint64_t max_n = 0, max_k = 0;
    int max_batch = 0;
    uint32_t cap = 0;
    void *scratch = nullptr;  // one device allocation, carved by scratch_layout (not owned when the context is a view of the static scratch)
    bool single_state = false;  // one state set, cleared by a launch of its own at the start of every call
    Stats *stats = nullptr;
    // two state sets (Sel records, histograms, chunk and block counts), used by alternate calls
    uint32_t *state[2] = {nullptr, nullptr};
    uint32_t state_words = 0;
    int cur = 0;                      // set the next call will use (it is clean)
    int cus = 1;                      // compute units of the device
    uint32_t rows = 0, status_cand_stride = 0, status_exact_stride = 0;
    uint32_t *samples = nullptr, *row_count = nullptr, *row_super = nullptr;
    uint32_t supers = 0;
    unsigned long long *bitmap = nullptr;
    uint32_t *cand_idx = nullptr, *cand_val = nullptr;
    float *act[2] = {nullptr, nullptr};  // autoencoder activations (ping-pong), grown on demand
    size_t act_floats = 0;
    // per-layer selection: thresholds [max_batch][n_seg] and a candidate list of its own, grown on demand
    uint32_t *seg_t = nullptr, *seg_cand = nullptr, *seg_row_prefix = nullptr;
    size_t seg_t_words = 0, seg_cand_words = 0;
    int opt_path = 0, opt_profile = 0, opt_carry = 1;
    // Thresholds carried from one selection to the next (one record per node, device memory, see Carry); for the
    // per-layer selection one record per layer and node, sized with the rest of its scratch by lgc_reserve
    Carry *carry = nullptr;
    Carry *seg_carry = nullptr;
    size_t seg_carry_records = 0;
    const lgc_segments *last_seg = nullptr;   // the plan of the previous selection, if that was a per-layer one
    uint64_t last_seg_k = 0;
    // Automatic path choice: a selection stores its call number to one of two pinned host words (fell back /
    // served by the fast path); the host looks at them (an ordinary read, no synchronisation) when it queues the
    // next selection, and after fall-backs takes the exact path outright for a while before it tries the fast path again.
    uint32_t *fell_back_host = nullptr, *fell_back_dev = nullptr;
    uint32_t call_number = 0, fell_back_seen = 0;
    int exact_calls_left = 0, penalty = 0;
    std::vector<hipEvent_t> ev;  // pairs: start, stop
    size_t ev_used = 0;
    char err[256] = {0};
};

struct lgc_segments {
    int device = 0;
    uint64_t n = 0, total_k = 0;
    uint32_t n_seg = 0, n_sampled = 0, rows = 0, cap = 0;
    uint32_t *dev = nullptr;  // one device allocation holding the five arrays below
    uint32_t *off = nullptr, *k = nullptr, *out = nullptr, *rank = nullptr, *row_seg = nullptr;
};

struct lgc_ae {
    int device = 0;
    float slope = 0.f;
    bool innovation = false;  // the last decoder layer takes the innovation component as one more channel
    std::vector<lgc_layer> enc, dec;
    std::vector<LayerDev> enc_dev, dec_dev;
    float *weights = nullptr;  // device copy of all weights and biases
    float *weights_t = nullptr;  // contraction-major copies for the layers that run on the matrix cores
};

static thread_local char g_err[256] = "";

static lgc_status fail(lgc_ctx *ctx, lgc_status s, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    if (ctx) memcpy(ctx->err, g_err, sizeof g_err);
    return s;
}

#define HIP_TRY(ctx, call)                                                                     \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return fail(ctx, e_ == hipErrorOutOfMemory ? LGC_ENOMEM : LGC_EHIP, "%s: %s", #call, \
                        hipGetErrorString(e_));                                                \
    } while (0)

namespace {

// No C++ exception leaves the library: the entry points that use containers run their bodies here.
template <typename F>
lgc_status no_throw(lgc_ctx *ctx, F &&body) noexcept {
    try {
        return body();
    } catch (const std::bad_alloc &) {
        return fail(ctx, LGC_ENOMEM, "out of host memory");
    } catch (...) {
        return fail(ctx, LGC_EHIP, "unexpected C++ exception");
    }
}

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
        if (prev == dev) prev = -1;
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// expected number of candidates above the sampled estimate, see choose_rank
double expected_candidates(double n, double k) {
    const double per = n / (double)kSample;
    return k + 6.0 * sqrt(k * per) + 8.0 * per;
}

uint32_t candidate_capacity(uint64_t max_n, uint64_t max_k) {
    double e = 1.5 * expected_candidates((double)max_n, (double)max_k) + 8192.0;
    if (e > 2.0e9) e = 2.0e9;
    return (uint32_t)align_up((size_t)e, kChunk);
}

// The estimate is the rank-th largest of kSample sampled keys.  With rk = k*kSample/n sampled
// keys expected among the true top k, rank = rk + 6*sqrt(rk) + 8 leaves about six standard
// deviations of head-room for count(candidates) >= k.
uint32_t choose_rank(uint32_t n, uint32_t k) {
    const double rk = (double)k * (double)kSample / (double)n;
    return (uint32_t)ceil(rk + 6.0 * sqrt(rk) + 8.0);
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

// The pair of events that times the next streaming call (LGC_OPT_PROFILE), or none.  The launches stamp the events
// themselves (start time of the first launch, end time of the last): nothing else enters the queue.
Bracket profile_bracket(lgc_ctx *c) {
    Bracket br;
    if (!c->opt_profile) return br;
    if (c->ev_used + 2 > c->ev.size()) {
        if (c->ev.size() >= 2 * 8192) return br;  // pool exhausted: stop timing until the next read
        hipEvent_t a, b;
        if (hipEventCreateWithFlags(&a, hipEventDisableSystemFence) != hipSuccess) return br;
        if (hipEventCreateWithFlags(&b, hipEventDisableSystemFence) != hipSuccess) { (void)hipEventDestroy(a); return br; }
        try {
            c->ev.reserve(c->ev.size() + 2);
        } catch (...) {
            (void)hipEventDestroy(a); (void)hipEventDestroy(b);
            return br;
        }
        c->ev.push_back(a);
        c->ev.push_back(b);
    }
    br.start = c->ev[c->ev_used];
    br.stop = c->ev[c->ev_used + 1];
    c->ev_used += 2;
    return br;
}

lgc_status check_common(lgc_ctx *ctx, uint64_t n, int batch, uint64_t stride) {
    if (!ctx) return fail(nullptr, LGC_EINVAL, "ctx is NULL");
    if (n == 0) return fail(ctx, LGC_EINVAL, "n == 0");
    if (n >= (1ull << 31)) return fail(ctx, LGC_EINVAL, "n = %llu is not below 2^31", (unsigned long long)n);
    if (n > ctx->max_n) return fail(ctx, LGC_EINVAL, "n = %llu exceeds the context's max_n = %llu",
                                    (unsigned long long)n, (unsigned long long)ctx->max_n);
    if (batch < 1 || batch > ctx->max_batch)
        return fail(ctx, LGC_EINVAL, "batch = %d outside [1, %d]", batch, ctx->max_batch);
    if (batch > 1 && stride < n) return fail(ctx, LGC_EINVAL, "stride < n");
    return LGC_OK;
}

// word offsets of the parts of one state set
struct StateLayout {
    size_t ctr, sel, sample_hist, fine_hist, level2_hist, radix_hist, status_cand, status_exact, words;
};
StateLayout state_layout(int max_batch, uint32_t status_cand_stride, uint32_t status_exact_stride) {
    StateLayout L;
    const size_t B = (size_t)max_batch;
    size_t o = 0;
    L.ctr = o; o += B * sizeof(Ctr) / 4;   // first: the set starts on a 256-byte boundary
    L.sel = o; o += B * sizeof(Sel) / 4;
    L.sample_hist = o; o += B * kSampleBins;
    L.fine_hist = o; o += B * kFineBins;
    L.level2_hist = o; o += B * kFineBins;
    L.radix_hist = o; o += B * 3 * kRadixBins;
    L.status_cand = o; o += B * status_cand_stride * 2;
    L.status_exact = o; o += B * status_exact_stride * 2;
    L.words = o;
    return L;
}

// The selection scratch of a context for (max_n, max_k, max_batch): byte offsets of its parts in one block of
// device memory.  Everything before `samples` (statistics, carried thresholds, state sets) must start at zero.
struct ScratchLayout {
    bool ok = false;
    uint32_t cap = 0, rows = 0, supers = 0, status_cand_stride = 0, status_exact_stride = 0, state_words = 0;
    size_t stats = 0, carry = 0, state[2] = {0, 0}, samples = 0, row_count = 0, row_super = 0, bitmap = 0, cand_idx = 0, cand_val = 0;
    size_t bytes = 0;
};

ScratchLayout scratch_layout(uint64_t max_n, uint64_t max_k, int max_batch, bool two_state_sets) {
    ScratchLayout s;
    s.cap = candidate_capacity(max_n, max_k);
    s.rows = (uint32_t)align_up((max_n + kRow - 1) / kRow, 4);
    s.status_exact_stride = (uint32_t)((max_n + kChunk - 1) / kChunk);
    s.status_cand_stride = (s.cap + kChunk - 1) / kChunk;
    const StateLayout L = state_layout(max_batch, s.status_cand_stride, s.status_exact_stride);
    if (L.words >= (1ull << 31)) return s;
    s.state_words = (uint32_t)L.words;
    s.supers = (s.rows + kSuperRows - 1) / kSuperRows;
    const size_t B = (size_t)max_batch, A = 256;
    size_t off = 0;
    auto carve = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, A); return o; };
    s.stats = carve(sizeof(Stats));
    s.carry = carve(B * sizeof(Carry));
    s.state[0] = carve(L.words * 4);
    s.state[1] = two_state_sets ? carve(L.words * 4) : s.state[0];
    s.samples = carve(B * kSample * 4);
    s.row_count = carve(B * s.rows * 4);
    s.row_super = carve(B * s.supers * 4);
    s.bitmap = carve(B * (size_t)s.rows * kRowWords * 8);
    s.cand_idx = carve(B * (size_t)s.cap * 4);
    s.cand_val = carve(B * (size_t)s.cap * 4);
    s.bytes = off;
    s.ok = true;
    return s;
}

void bind_scratch(lgc_ctx *c, void *base_ptr, const ScratchLayout &s) {
    char *base = (char *)base_ptr;
    c->scratch = base_ptr;
    c->cap = s.cap; c->rows = s.rows; c->supers = s.supers;
    c->status_cand_stride = s.status_cand_stride; c->status_exact_stride = s.status_exact_stride;
    c->state_words = s.state_words;
    c->stats = (Stats *)(base + s.stats);
    c->carry = (Carry *)(base + s.carry);
    c->state[0] = (uint32_t *)(base + s.state[0]);
    c->state[1] = (uint32_t *)(base + s.state[1]);
    c->samples = (uint32_t *)(base + s.samples);
    c->row_count = (uint32_t *)(base + s.row_count);
    c->row_super = (uint32_t *)(base + s.row_super);
    c->bitmap = (unsigned long long *)(base + s.bitmap);
    c->cand_idx = (uint32_t *)(base + s.cand_idx);
    c->cand_val = (uint32_t *)(base + s.cand_val);
}

SelArgs make_args(lgc_ctx *c, const float *g, float *u, float *v, uint64_t n, uint64_t stride, float m,
                  uint64_t k, float *out_vals, uint32_t *out_idx) {
    SelArgs a;
    memset(&a, 0, sizeof a);
    a.g = g; a.u = u; a.v = v;
    a.stride = stride; a.n = (uint32_t)n; a.k = (uint32_t)k; a.momentum = m;
    a.rank = 0; a.cap = c->cap; a.rows = c->rows;
    a.status_cand_stride = c->status_cand_stride; a.status_exact_stride = c->status_exact_stride;
    a.spin_limit = 1u << 22;
    a.force = 0;
    a.stats = c->stats;
    a.notify = c->fell_back_dev;
    a.notify_value = 0;
    a.carry = c->opt_carry && !c->single_state ? c->carry : nullptr;
    const StateLayout L = state_layout(c->max_batch, c->status_cand_stride, c->status_exact_stride);
    uint32_t *cur = c->state[c->cur];
    a.sel = (Sel *)(cur + L.sel);
    a.ctr = (Ctr *)(cur + L.ctr);
    a.sample_hist = cur + L.sample_hist; a.fine_hist = cur + L.fine_hist; a.level2_hist = cur + L.level2_hist; a.radix_hist = cur + L.radix_hist;
    a.status_cand = (unsigned long long *)(cur + L.status_cand);
    a.status_exact = (unsigned long long *)(cur + L.status_exact);
    a.next_state = c->state[c->cur ^ 1]; a.next_words = c->single_state ? 0u : c->state_words;
    a.samples = c->samples; a.row_count = c->row_count; a.bitmap = c->bitmap;
    a.row_super = c->row_super; a.supers = c->supers;
    a.cand_idx = c->cand_idx; a.cand_val = c->cand_val;
    a.out_vals = out_vals; a.out_idx = out_idx;
    return a;
}

constexpr int kMaxExactCalls = 64;   // most selections in a row that take the exact path outright after fall-backs were seen

// accumulate (optional) + select; g == nullptr means selection only
lgc_status run_select(lgc_ctx *ctx, const float *g, float *u, float *v, uint64_t n, int batch, uint64_t stride,
                      float m, uint64_t k, float *out_vals, uint32_t *out_idx, hipStream_t st) {
    const bool fused = g != nullptr;
    const bool vec = aligned(v, 16) && (!u || aligned(u, 16)) && (!g || aligned(g, 16)) &&
                     (batch == 1 || stride % 4 == 0);
    if (k == 0) {
        if (fused) {
            launch_accumulate(g, u, v, (uint32_t)n, batch, stride, m, vec, st, profile_bracket(ctx));
        }
        return LGC_OK;
    }
    SelArgs a = make_args(ctx, g, u, v, n, stride, m, k, out_vals, out_idx);
    {   // a carried threshold aims at 1.5 k candidates, or at what a sample would give where that is fewer (large k)
        const double sampled = expected_candidates((double)n, (double)k) / (double)k;
        a.carry_target = (float)log2(sampled < 1.5 ? sampled : 1.5);
        // and is offered only if it is expected to flag no more than 2.2 k, and no more than the list holds with
        // a third of the margin to spare (log scale)
        const double room = 0.75 * log2((double)ctx->cap / (double)k);
        a.carry_most = (float)(room < log2(2.2) ? room : log2(2.2));
    }
    ctx->last_seg = nullptr;
    bool fast = ctx->opt_path != 1 && n >= kMinFastN;
    if (fast) {
        a.rank = choose_rank((uint32_t)n, (uint32_t)k);
        fast = a.rank <= kSample / 4 &&
               1.5 * expected_candidates((double)n, (double)k) + 4096.0 <= (double)ctx->cap;
    }
    if (fast && ctx->opt_path == 0 && ctx->fell_back_host) {
        // data on which the fast path keeps failing (very many equal magnitudes around the k-th largest): reaching
        // the exact path through the failed fast path costs nearly twice what taking it outright does.  Each newly
        // seen fall-back doubles the number of selections that take the exact path outright before the fast path is
        // tried again (1, 2, 4, ... 64); a fast-path success seen after the last fall-back resets it.
        const uint32_t fell_back = ((volatile uint32_t *)ctx->fell_back_host)[0];
        const uint32_t served = ((volatile uint32_t *)ctx->fell_back_host)[1];
        if (fell_back != ctx->fell_back_seen) {
            ctx->fell_back_seen = fell_back;
            ctx->penalty = ctx->penalty ? (ctx->penalty * 2 > kMaxExactCalls ? kMaxExactCalls : ctx->penalty * 2) : 1;
            ctx->exact_calls_left = ctx->penalty;
        } else if ((int32_t)(served - fell_back) > 0) {
            ctx->penalty = 0;
        }
        if (ctx->exact_calls_left > 0) { --ctx->exact_calls_left; fast = false; }
    }
    if (fast) {
        if (++ctx->call_number == 0) ctx->call_number = 1;
        a.notify_value = ctx->call_number;
    }
    ctx->cur ^= 1;  // this call uses the clean set and cleans the other one for the next call
    if (fast) {
        launch_sample(a, batch, fused, vec, st);   // also clears the next call's state set
        launch_candidates(a, batch, fused, vec, st, profile_bracket(ctx));
        launch_gather(a, batch, st);
        a.force = 0;
        // the exact path as fall-back, for nodes the fast path hands back: with short candidate lists it rides in
        // the output launch, otherwise one launch of its own that nearly always has nothing to do
        if (!launch_output_from_candidates(a, batch, expected_candidates((double)n, (double)k) <= 131072.0, vec, ctx->cus, st))
            launch_exact(a, batch, vec, ctx->cus, st);
    } else {
        if (fused) {
            launch_accumulate(g, u, v, (uint32_t)n, batch, stride, m, vec, st, profile_bracket(ctx));
        }
        a.force = 1;   // exact path chosen outright (as five launches when the input is long); it also clears the next call's state set
        launch_exact(a, batch, vec, ctx->cus, st);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, LGC_EHIP, "kernel launch: %s", hipGetErrorString(e));
    return LGC_OK;
}

}  // namespace

// ------------------------------------------------------------------ context

extern "C" lgc_status lgc_create(lgc_ctx **out, int device, uint64_t max_n, uint64_t max_k, int max_batch) {
    if (!out) return fail(nullptr, LGC_EINVAL, "out is NULL");
    *out = nullptr;
    if (max_n == 0 || max_n >= (1ull << 31)) return fail(nullptr, LGC_EINVAL, "max_n must be in [1, 2^31)");
    if (max_k > max_n) return fail(nullptr, LGC_EINVAL, "max_k > max_n");
    if (max_batch < 1 || max_batch > 4096) return fail(nullptr, LGC_EINVAL, "max_batch must be in [1, 4096]");
    int ndev = 0;
    HIP_TRY(nullptr, hipGetDeviceCount(&ndev));
    if (device < 0 || device >= ndev) return fail(nullptr, LGC_EINVAL, "no HIP device %d", device);
    DeviceGuard guard(device);
    if (!guard.ok) return fail(nullptr, LGC_EHIP, "cannot select device %d", device);

    lgc_ctx *c = new (std::nothrow) lgc_ctx;
    if (!c) return fail(nullptr, LGC_ENOMEM, "out of host memory");
    c->device = device; c->max_n = max_n; c->max_k = max_k; c->max_batch = max_batch;
    {
        hipDeviceProp_t prop;
        hipError_t pe = hipGetDeviceProperties(&prop, device);
        if (pe != hipSuccess) { delete c; return fail(nullptr, LGC_EHIP, "hipGetDeviceProperties: %s", hipGetErrorString(pe)); }
        c->cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
    }
    const ScratchLayout L = scratch_layout(max_n, max_k, max_batch, true);
    if (!L.ok) { delete c; return fail(nullptr, LGC_EINVAL, "max_n * max_batch too large"); }
    void *block = nullptr;
    hipError_t e = hipMalloc(&block, L.bytes);
    if (e != hipSuccess) {
        delete c;
        return fail(nullptr, LGC_ENOMEM, "hipMalloc of %zu bytes of scratch: %s", L.bytes, hipGetErrorString(e));
    }
    // only the statistics, the carried thresholds and the two state sets must start at zero
    e = hipMemset(block, 0, L.samples);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipFree(block);
        delete c;
        return fail(nullptr, LGC_EHIP, "hipMemset: %s", hipGetErrorString(e));
    }
    bind_scratch(c, block, L);
    // the pinned words of the automatic path choice; without them (allocation refused) the choice is simply not adaptive
    void *pinned = nullptr, *pinned_dev = nullptr;
    if (hipHostMalloc(&pinned, 64, hipHostMallocMapped) == hipSuccess) {
        memset(pinned, 0, 64);
        if (hipHostGetDevicePointer(&pinned_dev, pinned, 0) == hipSuccess) {
            c->fell_back_host = (uint32_t *)pinned;
            c->fell_back_dev = (uint32_t *)pinned_dev;
        } else {
            (void)hipHostFree(pinned);
        }
    }
    (void)hipGetLastError();
    *out = c;
    return LGC_OK;
}

extern "C" void lgc_destroy(lgc_ctx *ctx) {
    if (!ctx) return;
    DeviceGuard guard(ctx->device);
    (void)hipDeviceSynchronize();
    for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
    if (ctx->act[0]) (void)hipFree(ctx->act[0]);
    if (ctx->seg_t) (void)hipFree(ctx->seg_t);
    if (ctx->seg_carry) (void)hipFree(ctx->seg_carry);
    if (ctx->seg_cand) (void)hipFree(ctx->seg_cand);
    if (ctx->seg_row_prefix) (void)hipFree(ctx->seg_row_prefix);
    if (ctx->scratch) (void)hipFree(ctx->scratch);
    if (ctx->fell_back_host) (void)hipHostFree(ctx->fell_back_host);
    delete ctx;
}

extern "C" const char *lgc_last_error(const lgc_ctx *ctx) { return ctx ? ctx->err : g_err; }

extern "C" const char *lgc_status_string(lgc_status s) {
    switch (s) {
        case LGC_OK: return "ok";
        case LGC_EINVAL: return "invalid argument";
        case LGC_ENOMEM: return "out of memory";
        case LGC_EHIP: return "HIP runtime error";
        case LGC_EDEVICE: return "device-side failure";
    }
    return "unknown status";
}

// ------------------------------------------------------------------ a1, a2

extern "C" lgc_status lgc_accumulate(lgc_ctx *ctx, const float *g, float *u, float *v, uint64_t n, int batch,
                                     uint64_t stride, float momentum, void *stream) {
    lgc_status s = check_common(ctx, n, batch, stride);
    if (s != LGC_OK) return s;
    if (!g || !u || !v) return fail(ctx, LGC_EINVAL, "g, u and v must not be NULL");
    if (!aligned(g, 4) || !aligned(u, 4) || !aligned(v, 4)) return fail(ctx, LGC_EINVAL, "pointer not 4-byte aligned");
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    return run_select(ctx, g, u, v, n, batch, stride, momentum, 0, nullptr, nullptr, (hipStream_t)stream);
}

static lgc_status check_select(lgc_ctx *ctx, uint64_t n, uint64_t k, const float *out_vals, const uint32_t *out_idx) {
    if (k > n) return fail(ctx, LGC_EINVAL, "k = %llu > n = %llu", (unsigned long long)k, (unsigned long long)n);
    if (k > ctx->max_k) return fail(ctx, LGC_EINVAL, "k = %llu exceeds the context's max_k = %llu",
                                    (unsigned long long)k, (unsigned long long)ctx->max_k);
    if (k > 0 && (!out_vals || !out_idx)) return fail(ctx, LGC_EINVAL, "out_vals and out_idx must not be NULL");
    if (!aligned(out_vals, 4) || !aligned(out_idx, 4)) return fail(ctx, LGC_EINVAL, "pointer not 4-byte aligned");
    return LGC_OK;
}

extern "C" lgc_status lgc_topk(lgc_ctx *ctx, float *v, float *u, uint64_t n, int batch, uint64_t stride,
                               uint64_t k, float *out_vals, uint32_t *out_idx, void *stream) {
    lgc_status s = check_common(ctx, n, batch, stride);
    if (s != LGC_OK) return s;
    if (!v) return fail(ctx, LGC_EINVAL, "v must not be NULL");
    if (!aligned(v, 4) || !aligned(u, 4)) return fail(ctx, LGC_EINVAL, "pointer not 4-byte aligned");
    if ((s = check_select(ctx, n, k, out_vals, out_idx)) != LGC_OK) return s;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    return run_select(ctx, nullptr, u, v, n, batch, stride, 0.f, k, out_vals, out_idx, (hipStream_t)stream);
}

extern "C" lgc_status lgc_accumulate_topk(lgc_ctx *ctx, const float *g, float *u, float *v, uint64_t n,
                                          int batch, uint64_t stride, float momentum, uint64_t k,
                                          float *out_vals, uint32_t *out_idx, void *stream) {
    lgc_status s = check_common(ctx, n, batch, stride);
    if (s != LGC_OK) return s;
    if (!g || !u || !v) return fail(ctx, LGC_EINVAL, "g, u and v must not be NULL");
    if (!aligned(g, 4) || !aligned(u, 4) || !aligned(v, 4)) return fail(ctx, LGC_EINVAL, "pointer not 4-byte aligned");
    if ((s = check_select(ctx, n, k, out_vals, out_idx)) != LGC_OK) return s;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    return run_select(ctx, g, u, v, n, batch, stride, momentum, k, out_vals, out_idx, (hipStream_t)stream);
}

// ------------------------------------------------------------------ a1 + a2 without any allocation

// Selection scratch for callers that cannot allocate (see lgc_accumulate_topk_static in lgc.h): a fixed array in
// device memory, one copy on every GPU that loads the library, held until the process ends.  In host code this
// NAME is only a handle for hipGetSymbolAddress; the array's memory on a given GPU is reached through the
// address that call returns for that GPU (static_dev[].ptr), never through the name.
constexpr size_t kStaticScratchBytes = (size_t)LGC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char lgc_static_scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxStaticDevices = 64;
struct StaticDev {
    unsigned char *ptr = nullptr;   // this GPU's copy of lgc_static_scratch
    int cus = 1;
    bool ready = false;
};
StaticDev static_dev[kMaxStaticDevices];
std::mutex static_dev_mutex;

// once per device, with that device current
lgc_status static_dev_setup(int device, StaticDev **out) {
    std::lock_guard<std::mutex> lock(static_dev_mutex);
    StaticDev &d = static_dev[device];
    if (!d.ready) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(lgc_static_scratch));
        if (e != hipSuccess || !p)
            return fail(nullptr, LGC_EHIP, "hipGetSymbolAddress(lgc_static_scratch) on device %d: %s", device, hipGetErrorString(e));
        int cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
        if (e != hipSuccess) return fail(nullptr, LGC_EHIP, "hipDeviceGetAttribute: %s", hipGetErrorString(e));
        d.ptr = (unsigned char *)p;
        d.cus = cus > 0 ? cus : 1;
        d.ready = true;
    }
    *out = &d;
    return LGC_OK;
}
}  // namespace

extern "C" lgc_status lgc_accumulate_topk_static(int device, const float *g, float *u, float *v, uint64_t n, int batch,
                                                 uint64_t stride, float momentum, uint64_t k, float *out_vals,
                                                 uint32_t *out_idx, void *stream) {
    if (n == 0 || n >= (1ull << 31)) return fail(nullptr, LGC_EINVAL, "n must be in [1, 2^31)");
    if (batch < 1 || batch > 4096) return fail(nullptr, LGC_EINVAL, "batch must be in [1, 4096]");
    if (batch > 1 && stride < n) return fail(nullptr, LGC_EINVAL, "stride < n");
    if (k > n) return fail(nullptr, LGC_EINVAL, "k = %llu > n = %llu", (unsigned long long)k, (unsigned long long)n);
    if (!g || !u || !v) return fail(nullptr, LGC_EINVAL, "g, u and v must not be NULL");
    if (k > 0 && (!out_vals || !out_idx)) return fail(nullptr, LGC_EINVAL, "out_vals and out_idx must not be NULL");
    if (!aligned(g, 4) || !aligned(u, 4) || !aligned(v, 4) || !aligned(out_vals, 4) || !aligned(out_idx, 4))
        return fail(nullptr, LGC_EINVAL, "pointer not 4-byte aligned");
    // the same scratch a context for exactly (n, k, batch) would own, with one state set instead of two
    const ScratchLayout L = scratch_layout(n, k, batch, false);
    if (!L.ok || L.bytes > kStaticScratchBytes)
        return fail(nullptr, LGC_EINVAL,
                    "lgc_accumulate_topk_static: n = %llu, k = %llu, batch = %d need %zu bytes of scratch, the static "
                    "scratch holds %zu (about batch * (n / 8 + 1 MB)); use a context (lgc_create) for larger inputs",
                    (unsigned long long)n, (unsigned long long)k, batch, L.ok ? L.bytes : (size_t)0, kStaticScratchBytes);
    int ndev = 0;
    HIP_TRY(nullptr, hipGetDeviceCount(&ndev));
    if (device < 0 || device >= ndev || device >= kMaxStaticDevices) return fail(nullptr, LGC_EINVAL, "no HIP device %d", device);
    DeviceGuard guard(device);
    if (!guard.ok) return fail(nullptr, LGC_EHIP, "cannot select device %d", device);
    StaticDev *sd = nullptr;
    lgc_status s = static_dev_setup(device, &sd);
    if (s != LGC_OK) return s;

    lgc_ctx view;   // a view of the static scratch for this call; lives on the stack, owns nothing
    view.device = device; view.max_n = n; view.max_k = k; view.max_batch = batch;
    view.cus = sd->cus;
    view.single_state = true;
    bind_scratch(&view, sd->ptr, L);
    hipStream_t st = (hipStream_t)stream;
    // the array keeps the last call's contents: statistics and the state set start every call at zero
    // (a fill kernel, not a memset, so that the call can be recorded into a HIP graph)
    if (k > 0) launch_clear((uint32_t *)sd->ptr, (uint32_t)(L.samples / 4), st);
    return run_select(&view, g, u, v, n, batch, stride, momentum, k, out_vals, out_idx, st);
}

// ------------------------------------------------------------------ autoencoder

static bool layer_ok(const lgc_layer &l) {
    return l.c_in >= 1 && l.c_out >= 1 && l.c_in <= 4096 && l.c_out <= 4096 && (l.ksize == 1 || l.ksize == 3) &&
           (l.stride == 1 || l.stride == 2);
}

extern "C" lgc_status lgc_ae_create(lgc_ae **out, int device, int n_enc, const lgc_layer *enc, int n_dec,
                                    const lgc_layer *dec, float slope, const float *const *enc_w,
                                    const float *const *enc_b, const float *const *dec_w,
                                    const float *const *dec_b) {
    if (!out) return fail(nullptr, LGC_EINVAL, "out is NULL");
    *out = nullptr;
    if (n_enc < 1 || n_dec < 1 || n_enc > 64 || n_dec > 64 || !enc || !dec || !enc_w || !enc_b || !dec_w || !dec_b)
        return fail(nullptr, LGC_EINVAL, "bad autoencoder description");
    int strided_enc = 0, strided_dec = 0;
    bool with_innovation = false;
    for (int l = 0; l < n_enc; ++l) {
        if (!layer_ok(enc[l]) || !enc_w[l] || !enc_b[l]) return fail(nullptr, LGC_EINVAL, "bad encoder layer %d", l);
        if (l > 0 && enc[l].c_in != enc[l - 1].c_out) return fail(nullptr, LGC_EINVAL, "encoder layer %d: channel mismatch", l);
        strided_enc += enc[l].stride == 2;
    }
    for (int l = 0; l < n_dec; ++l) {
        if (!layer_ok(dec[l]) || !dec_w[l] || !dec_b[l]) return fail(nullptr, LGC_EINVAL, "bad decoder layer %d", l);
        if (l > 0 && dec[l].c_in != dec[l - 1].c_out) {
            // decoder with the innovation component (Sec. IV-C): one more channel into the last, stride-1 layer
            const bool concat = l == n_dec - 1 && dec[l].c_in == dec[l - 1].c_out + 1 && dec[l].stride == 1;
            if (!concat) return fail(nullptr, LGC_EINVAL, "decoder layer %d: channel mismatch", l);
            with_innovation = true;
        }
        strided_dec += dec[l].stride == 2;
    }
    if (enc[0].c_in != 1 || dec[n_dec - 1].c_out != 1) return fail(nullptr, LGC_EINVAL, "input and output must have one channel");
    if (dec[0].c_in != enc[n_enc - 1].c_out) return fail(nullptr, LGC_EINVAL, "decoder input channels != latent channels");
    if (strided_enc != strided_dec) return fail(nullptr, LGC_EINVAL, "encoder and decoder differ in stride-2 layers");
    int ndev = 0;
    HIP_TRY(nullptr, hipGetDeviceCount(&ndev));
    if (device < 0 || device >= ndev) return fail(nullptr, LGC_EINVAL, "no HIP device %d", device);
    DeviceGuard guard(device);
    if (!guard.ok) return fail(nullptr, LGC_EHIP, "cannot select device %d", device);

    lgc_ae *ae = new (std::nothrow) lgc_ae;
    if (!ae) return fail(nullptr, LGC_ENOMEM, "out of host memory");
    ae->device = device; ae->slope = slope; ae->innovation = with_innovation;
    try {
        ae->enc.assign(enc, enc + n_enc);
        ae->dec.assign(dec, dec + n_dec);
        ae->enc_dev.reserve(n_enc);   // so that the push_back calls below cannot throw
        ae->dec_dev.reserve(n_dec);
    } catch (...) {
        delete ae;
        return fail(nullptr, LGC_ENOMEM, "out of host memory");
    }
    size_t total = 0;
    auto wsize = [](const lgc_layer &l) { return align_up((size_t)l.c_in * l.c_out * l.ksize, 64); };
    auto bsize = [](const lgc_layer &l) { return align_up((size_t)l.c_out, 64); };
    for (auto &l : ae->enc) total += wsize(l) + bsize(l);
    for (auto &l : ae->dec) total += wsize(l) + bsize(l);
    hipError_t e = hipMalloc((void **)&ae->weights, total * 4);
    if (e != hipSuccess) { delete ae; return fail(nullptr, LGC_ENOMEM, "hipMalloc of autoencoder weights: %s", hipGetErrorString(e)); }
    size_t off = 0;
    auto take = [&](const lgc_layer &l, const float *w, const float *b, std::vector<LayerDev> &dst) -> hipError_t {
        LayerDev d{l.c_in, l.c_out, l.ksize, l.stride, ae->weights + off, nullptr};
        hipError_t r = hipMemcpy(ae->weights + off, w, (size_t)l.c_in * l.c_out * l.ksize * 4, hipMemcpyDeviceToDevice);
        if (r != hipSuccess) return r;
        off += wsize(l);
        d.b = ae->weights + off;
        r = hipMemcpy(ae->weights + off, b, (size_t)l.c_out * 4, hipMemcpyDeviceToDevice);
        off += bsize(l);
        dst.push_back(d);
        return r;
    };
    for (int l = 0; l < n_enc && e == hipSuccess; ++l) e = take(enc[l], enc_w[l], enc_b[l], ae->enc_dev);
    for (int l = 0; l < n_dec && e == hipSuccess; ++l) e = take(dec[l], dec_w[l], dec_b[l], ae->dec_dev);
    if (e == hipSuccess) {
        // deep kernel-3 / stride-2 layers run on the matrix cores from a contraction-major copy of their weights
        auto deep = [](const lgc_layer &l, int co_multiple) {
            return l.ksize == 3 && l.stride == 2 && l.c_in % 16 == 0 && l.c_out % co_multiple == 0;
        };
        size_t t_total = 0;
        for (auto &l : ae->enc) if (deep(l, 64)) t_total += wsize(l);
        for (auto &l : ae->dec) if (deep(l, 32)) t_total += wsize(l);
        if (t_total) {
            e = hipMalloc((void **)&ae->weights_t, t_total * 4);
            size_t t_off = 0;
            for (size_t l = 0; l < ae->enc.size() && e == hipSuccess; ++l)
                if (deep(ae->enc[l], 64)) {
                    launch_weights_contraction_major(ae->enc_dev[l].w, ae->weights_t + t_off, ae->enc[l].c_in, ae->enc[l].c_out, false, nullptr);
                    ae->enc_dev[l].wt = ae->weights_t + t_off;
                    t_off += wsize(ae->enc[l]);
                }
            for (size_t l = 0; l < ae->dec.size() && e == hipSuccess; ++l)
                if (deep(ae->dec[l], 32) && !(with_innovation && l + 1 == ae->dec.size())) {
                    launch_weights_contraction_major(ae->dec_dev[l].w, ae->weights_t + t_off, ae->dec[l].c_in, ae->dec[l].c_out, true, nullptr);
                    ae->dec_dev[l].wt = ae->weights_t + t_off;
                    t_off += wsize(ae->dec[l]);
                }
            if (e == hipSuccess) e = hipGetLastError();
        }
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        if (ae->weights_t) (void)hipFree(ae->weights_t);
        (void)hipFree(ae->weights);
        delete ae;
        return fail(nullptr, LGC_EHIP, "copying autoencoder weights: %s", hipGetErrorString(e));
    }
    *out = ae;
    return LGC_OK;
}

extern "C" void lgc_ae_destroy(lgc_ae *ae) {
    if (!ae) return;
    DeviceGuard guard(ae->device);
    (void)hipDeviceSynchronize();
    if (ae->weights) (void)hipFree(ae->weights);
    if (ae->weights_t) (void)hipFree(ae->weights_t);
    delete ae;
}

static uint64_t conv_len(uint64_t l_in, const lgc_layer &l) {
    if (l_in == 0) return 0;
    const uint64_t pad = (l.ksize - 1) / 2;
    return (l_in + 2 * pad - l.ksize) / l.stride + 1;
}

// lengths after each encoder layer: [k, L1, ..., L_latent]
static std::vector<uint64_t> enc_lengths(const lgc_ae *ae, uint64_t k) {
    std::vector<uint64_t> v{k};
    for (auto &l : ae->enc) v.push_back(conv_len(v.back(), l));
    return v;
}

// output length of each decoder layer: a stride-1 layer keeps the length, the strided layers
// restore, last consumed first, the lengths the strided encoder layers consumed
static std::vector<uint64_t> dec_lengths(const lgc_ae *ae, uint64_t k) {
    std::vector<uint64_t> el = enc_lengths(ae, k), consumed, out;
    for (size_t i = 0; i < ae->enc.size(); ++i)
        if (ae->enc[i].stride == 2) consumed.push_back(el[i]);
    uint64_t cur = el.back();
    for (auto &l : ae->dec) {
        if (l.stride == 2) { cur = consumed.back(); consumed.pop_back(); }
        out.push_back(cur);
    }
    return out;
}

extern "C" uint64_t lgc_latent_len(const lgc_ae *ae, uint64_t k) {
    if (!ae) return 0;
    uint64_t len = k;   // no container here: nothing can throw
    for (auto &l : ae->enc) len = conv_len(len, l);
    return len * (uint64_t)ae->enc.back().c_out;
}

// floats per activation buffer that encoder and decoder need for inputs of k values and `batch` nodes (the
// largest intermediate tensor of either stack)
static size_t act_need(const lgc_ae *ae, uint64_t k, int batch) {
    size_t need = 0;
    uint64_t len = k;
    for (size_t l = 0; l < ae->enc.size(); ++l) {
        len = conv_len(len, ae->enc[l]);
        if (l + 1 < ae->enc.size()) need = std::max(need, (size_t)batch * ae->enc[l].c_out * (size_t)len);
        // a deep layer with few output tiles runs with its contraction split: room for the partial sums, which
        // never exceed 512 tiles of 64 x 64 (smaller calls split further, up to that many blocks)
        if (l > 0 && ae->enc_dev[l].wt && ae->enc[l].c_in >= 128 && ae->enc[l].c_out % 64 == 0)
            need = std::max(need, (size_t)512 * 64 * 64);
    }
    const std::vector<uint64_t> out_len = dec_lengths(ae, k);
    for (size_t l = 0; l + 1 < ae->dec.size(); ++l)
        need = std::max(need, (size_t)batch * ae->dec[l].c_out * (size_t)out_len[l]);
    return need;
}

// only from lgc_reserve: the hot-path calls never allocate
static lgc_status ensure_act(lgc_ctx *ctx, size_t floats) {
    if (floats <= ctx->act_floats) return LGC_OK;
    if (ctx->act[0]) {
        HIP_TRY(ctx, hipDeviceSynchronize());
        HIP_TRY(ctx, hipFree(ctx->act[0]));
        ctx->act[0] = ctx->act[1] = nullptr; ctx->act_floats = 0;
    }
    floats = align_up(floats, 64);
    HIP_TRY(ctx, hipMalloc((void **)&ctx->act[0], 2 * floats * 4));
    ctx->act[1] = ctx->act[0] + floats;
    ctx->act_floats = floats;
    return LGC_OK;
}

static lgc_status check_ae_call(lgc_ctx *ctx, const lgc_ae *ae, const void *a, const void *b, uint64_t k, int batch) {
    if (!ctx) return fail(nullptr, LGC_EINVAL, "ctx is NULL");
    if (!ae) return fail(ctx, LGC_EINVAL, "ae is NULL");
    if (ae->device != ctx->device) return fail(ctx, LGC_EINVAL, "autoencoder and context live on different devices");
    if (batch < 1 || batch > ctx->max_batch) return fail(ctx, LGC_EINVAL, "batch = %d outside [1, %d]", batch, ctx->max_batch);
    if (k > ctx->max_k) return fail(ctx, LGC_EINVAL, "k exceeds the context's max_k");
    if (k > 0 && (!a || !b)) return fail(ctx, LGC_EINVAL, "NULL data pointer");
    if (!aligned(a, 4) || !aligned(b, 4)) return fail(ctx, LGC_EINVAL, "pointer not 4-byte aligned");
    return LGC_OK;
}

static lgc_status run_encode(lgc_ctx *ctx, const lgc_ae *ae, const float *vals, uint64_t k, int batch,
                             float *latent, void *stream) {
    lgc_status s = check_ae_call(ctx, ae, vals, latent, k, batch);
    if (s != LGC_OK) return s;
    if (k == 0) return LGC_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    hipStream_t st = (hipStream_t)stream;
    std::vector<uint64_t> len = enc_lengths(ae, k);
    const size_t nl = ae->enc.size();
    if (nl == 2 && launch_encoder2(vals, latent, ae->enc_dev[0], ae->enc_dev[1], (uint32_t)len[0], (uint32_t)len[1],
                                   (uint32_t)len[2], batch, ae->slope, st)) {
        hipError_t e2 = hipGetLastError();
        if (e2 != hipSuccess) return fail(ctx, LGC_EHIP, "kernel launch: %s", hipGetErrorString(e2));
        return LGC_OK;
    }
    size_t need = 0;
    for (size_t l = 0; l < nl; ++l) {
        size_t f = l + 1 < nl ? (size_t)batch * ae->enc[l].c_out * len[l + 1] : 0;
        const int splits = l > 0 ? conv3s2_mfma_splits(ae->enc_dev[l], (uint32_t)len[l + 1], batch) : 1;
        if (splits > 1) f = std::max(f, (size_t)splits * batch * ae->enc[l].c_out * len[l + 1]);
        if (f > need) need = f;
    }
    if (need > ctx->act_floats)
        return fail(ctx, LGC_EINVAL, "lgc_encode: activation scratch for k = %llu, batch = %d not reserved: call "
                                     "lgc_reserve(ctx, ae, k, batch, NULL) once beforehand", (unsigned long long)k, batch);
    const float *cur = vals;
    // a layer never writes the buffer it reads: the activation buffer that is not `cur`
    auto other = [&](const float *c) { return c == ctx->act[0] ? ctx->act[1] : ctx->act[0]; };
    for (size_t l = 0; l < nl; ++l) {
        const bool last = l + 1 == nl;
        if (l == 0 && nl > 2) {   // the one-channel first layer inside the staging of the deep layer after it
            if (launch_conv3s2_mfma_head(vals, ctx->act[1], ae->enc_dev[0], ae->enc_dev[1], (uint32_t)len[0], (uint32_t)len[1],
                                         (uint32_t)len[2], batch, true, ae->slope, st)) {
                cur = ctx->act[1];
                ++l;
                continue;
            }
        }
        // a deep layer with too few output tiles to fill the device: contraction split over several blocks, partial
        // sums to the free activation buffer, then a finish kernel (which also applies a kernel-1 layer that follows)
        const int splits = (cur == ctx->act[0] || cur == ctx->act[1])
                               ? conv3s2_mfma_splits(ae->enc_dev[l], (uint32_t)len[l + 1], batch) : 1;
        if (splits > 1) {
            const LayerDev *tail = nullptr;
            if (!last && ae->enc[l + 1].ksize == 1 && ae->enc[l + 1].stride == 1 && ae->enc[l + 1].c_out <= 4) tail = &ae->enc_dev[l + 1];
            const bool out_is_last = tail ? l + 2 == nl : last;
            float *part = other(cur);
            float *dst = out_is_last ? latent : const_cast<float *>(cur);   // the layer's input is free once the partial sums exist
            if (launch_conv3s2_mfma_splitk(cur, part, dst, ae->enc_dev[l], (uint32_t)len[l], (uint32_t)len[l + 1], batch, splits,
                                           !last, ae->slope, st, tail, tail && !out_is_last)) {
                cur = dst;
                if (tail) ++l;
                continue;
            }
        }
        if (l + 1 < nl) {   // a deep layer and the kernel-1 layer after it in one launch, where the shapes allow
            const bool next_last = l + 2 == nl;
            float *dst2 = next_last ? latent : other(cur);
            if (launch_conv3s2_mfma(cur, dst2, ae->enc_dev[l], (uint32_t)len[l], (uint32_t)len[l + 1], batch, true, ae->slope,
                                    st, &ae->enc_dev[l + 1], !next_last)) {
                cur = dst2;
                ++l;
                continue;
            }
        }
        float *dst = last ? latent : other(cur);
        if (!launch_conv3s2_mfma(cur, dst, ae->enc_dev[l], (uint32_t)len[l], (uint32_t)len[l + 1], batch, !last, ae->slope, st))
            launch_conv1d(cur, dst, ae->enc_dev[l], (uint32_t)len[l], (uint32_t)len[l + 1], batch, !last, ae->slope, st);
        cur = dst;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, LGC_EHIP, "kernel launch: %s", hipGetErrorString(e));
    return LGC_OK;
}

extern "C" lgc_status lgc_encode(lgc_ctx *ctx, const lgc_ae *ae, const float *vals, uint64_t k, int batch,
                                 float *latent, void *stream) {
    return no_throw(ctx, [&] { return run_encode(ctx, ae, vals, k, batch, latent, stream); });
}

static lgc_status run_decode(lgc_ctx *ctx, const lgc_ae *ae, const float *latent, const float *innov, uint64_t k,
                             int batch, float *rec, void *stream) {
    lgc_status s = check_ae_call(ctx, ae, latent, rec, k, batch);
    if (s != LGC_OK) return s;
    if (ae->innovation != (innov != nullptr))
        return fail(ctx, LGC_EINVAL, ae->innovation ? "this autoencoder's decoder needs the innovation component: use lgc_decode_innovation"
                                                     : "this autoencoder's decoder takes no innovation component: use lgc_decode");
    if (!aligned(innov, 4)) return fail(ctx, LGC_EINVAL, "pointer not 4-byte aligned");
    if (k == 0) return LGC_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    hipStream_t st = (hipStream_t)stream;
    std::vector<uint64_t> out_len = dec_lengths(ae, k);
    uint64_t in_len = enc_lengths(ae, k).back();
    const size_t nl = ae->dec.size();
    if (!innov && nl == 2 &&
        launch_decoder2(latent, rec, ae->dec_dev[0], ae->dec_dev[1], (uint32_t)in_len, (uint32_t)out_len[0],
                        (uint32_t)out_len[1], batch, ae->slope, st)) {
        hipError_t e2 = hipGetLastError();
        if (e2 != hipSuccess) return fail(ctx, LGC_EHIP, "kernel launch: %s", hipGetErrorString(e2));
        return LGC_OK;
    }
    if (innov && nl == 3 &&
        launch_decoder3i(latent, innov, rec, ae->dec_dev[0], ae->dec_dev[1], ae->dec_dev[2], (uint32_t)in_len,
                         (uint32_t)out_len[0], (uint32_t)out_len[1], batch, ae->slope, st)) {
        hipError_t e3 = hipGetLastError();
        if (e3 != hipSuccess) return fail(ctx, LGC_EHIP, "kernel launch: %s", hipGetErrorString(e3));
        return LGC_OK;
    }
    size_t need = 0;
    for (size_t l = 0; l + 1 < nl; ++l) {
        size_t f = (size_t)batch * ae->dec[l].c_out * out_len[l];
        if (f > need) need = f;
    }
    if (need > ctx->act_floats)
        return fail(ctx, LGC_EINVAL, "lgc_decode: activation scratch for k = %llu, batch = %d not reserved: call "
                                     "lgc_reserve(ctx, ae, k, batch, NULL) once beforehand", (unsigned long long)k, batch);
    const float *cur = latent;
    // a layer never writes the buffer it reads: the activation buffer that is not `cur`
    auto other = [&](const float *c) { return c == ctx->act[0] ? ctx->act[1] : ctx->act[0]; };
    for (size_t l = 0; l < nl; ++l) {
        const bool last = l + 1 == nl;
        if (l == 0 && nl > 3) {   // the two narrow first layers inside the staging of the deep layer after them
            if (launch_convt3s2_mfma_head(latent, ctx->act[0], ae->dec_dev[0], ae->dec_dev[1], ae->dec_dev[2], (uint32_t)in_len,
                                          (uint32_t)out_len[1], (uint32_t)out_len[2], batch, true, ae->slope, st)) {
                cur = ctx->act[0];
                in_len = out_len[2];
                l = 2;
                continue;
            }
        }
        if (l + 1 < nl && !innov) {   // a deep layer and the kernel-1 layer after it in one launch, where the shapes allow
            const bool next_last = l + 2 == nl;
            float *dst2 = next_last ? rec : other(cur);
            if (launch_convt3s2_mfma(cur, dst2, ae->dec_dev[l], (uint32_t)in_len, (uint32_t)out_len[l], batch, true, ae->slope,
                                     st, &ae->dec_dev[l + 1], !next_last)) {
                cur = dst2;
                in_len = out_len[l + 1];
                ++l;
                continue;
            }
        }
        float *dst = last ? rec : other(cur);
        const float *extra = last ? innov : nullptr;
        if (extra || !launch_convt3s2_mfma(cur, dst, ae->dec_dev[l], (uint32_t)in_len, (uint32_t)out_len[l], batch, !last,
                                           ae->slope, st))
            launch_conv_transpose1d(cur, dst, ae->dec_dev[l], (uint32_t)in_len, (uint32_t)out_len[l], batch, !last,
                                    ae->slope, st, extra);
        cur = dst;
        in_len = out_len[l];
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, LGC_EHIP, "kernel launch: %s", hipGetErrorString(e));
    return LGC_OK;
}

extern "C" lgc_status lgc_decode(lgc_ctx *ctx, const lgc_ae *ae, const float *latent, uint64_t k, int batch,
                                 float *rec, void *stream) {
    return no_throw(ctx, [&] { return run_decode(ctx, ae, latent, nullptr, k, batch, rec, stream); });
}

extern "C" lgc_status lgc_decode_innovation(lgc_ctx *ctx, const lgc_ae *ae, const float *latent, const float *innov,
                                            uint64_t k, int batch, float *rec, void *stream) {
    if (ctx && k > 0 && !innov) return fail(ctx, LGC_EINVAL, "innov must not be NULL");
    if (ctx && ae && k == 0 && !innov && ae->innovation) return LGC_OK;
    return no_throw(ctx, [&] { return run_decode(ctx, ae, latent, innov, k, batch, rec, stream); });
}

extern "C" lgc_status lgc_innovation(lgc_ctx *ctx, const lgc_segments *seg, const float *vals, int batch, float *out,
                                     void *stream) {
    if (!ctx) return fail(nullptr, LGC_EINVAL, "ctx is NULL");
    if (!seg) return fail(ctx, LGC_EINVAL, "segments is NULL");
    if (seg->device != ctx->device) return fail(ctx, LGC_EINVAL, "segment plan and context live on different devices");
    if (batch < 1 || batch > ctx->max_batch) return fail(ctx, LGC_EINVAL, "batch = %d outside [1, %d]", batch, ctx->max_batch);
    if (!vals || !out) return fail(ctx, LGC_EINVAL, "NULL data pointer");
    if (vals == out) return fail(ctx, LGC_EINVAL, "out must not alias vals");
    if (!aligned(vals, 4) || !aligned(out, 4)) return fail(ctx, LGC_EINVAL, "pointer not 4-byte aligned");
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    const bool vec = aligned(vals, 16) && (batch == 1 || seg->n % 4 == 0);
    launch_innovation(vals, out, (uint32_t)seg->n, batch, seg->n_seg, seg->off, seg->k, vec, ctx->stats,
                      (hipStream_t)stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, LGC_EHIP, "kernel launch: %s", hipGetErrorString(e));
    return LGC_OK;
}

// ------------------------------------------------------------------ a5

extern "C" lgc_status lgc_scatter(lgc_ctx *ctx, const float *vals, const uint32_t *idx, uint64_t k, int batch,
                                  float scale, float *dense, uint64_t n, void *stream) {
    if (!ctx) return fail(nullptr, LGC_EINVAL, "ctx is NULL");
    if (n == 0 || n >= (1ull << 31)) return fail(ctx, LGC_EINVAL, "n must be in [1, 2^31)");
    if (batch < 1 || batch > ctx->max_batch) return fail(ctx, LGC_EINVAL, "batch = %d outside [1, %d]", batch, ctx->max_batch);
    if (k > n) return fail(ctx, LGC_EINVAL, "k > n");
    if (!dense || (k > 0 && (!vals || !idx))) return fail(ctx, LGC_EINVAL, "NULL data pointer");
    if (!aligned(vals, 4) || !aligned(idx, 4) || !aligned(dense, 4)) return fail(ctx, LGC_EINVAL, "pointer not 4-byte aligned");
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    // up to 8 nodes go through one launch; more are applied by one launch per node, in order
    if (batch == 1 ||
        !launch_scatter_nodes(vals, idx, (uint32_t)k, batch, scale, dense, (uint32_t)n, ctx->stats, (hipStream_t)stream))
        for (int b = 0; b < batch; ++b)
            launch_scatter(vals + (size_t)b * k, idx + (size_t)b * k, (uint32_t)k, scale, dense, (uint32_t)n, ctx->stats,
                           (hipStream_t)stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, LGC_EHIP, "kernel launch: %s", hipGetErrorString(e));
    return LGC_OK;
}

// ------------------------------------------------------------------ per-layer selection

constexpr uint32_t kSegSampleKeys = 16384;   // keys sampled per sampled segment (1024 threads x 16)
constexpr uint64_t kSegMinSampled = 8192;   // smaller segments are selected from v directly (measured at 161 layers x 4 nodes:
                                             // 16 K: k_seg_select 30 us, fused call 385 us; 8 K: 27 / 379; 4 K: 27 / 382, more layers whose
                                             // thresholds are too noisy to carry)

static lgc_status segments_create(lgc_segments **out, int device, uint64_t n, uint64_t n_seg,
                                  const uint64_t *offsets, const uint64_t *ks) {
    if (!out) return fail(nullptr, LGC_EINVAL, "out is NULL");
    *out = nullptr;
    if (!offsets || !ks) return fail(nullptr, LGC_EINVAL, "offsets and ks must not be NULL");
    if (n == 0 || n >= (1ull << 31)) return fail(nullptr, LGC_EINVAL, "n must be in [1, 2^31)");
    if (n_seg == 0 || n_seg > (1ull << 20) || n_seg > n) return fail(nullptr, LGC_EINVAL, "n_seg must be in [1, min(n, 2^20)]");
    if (offsets[0] != 0 || offsets[n_seg] != n) return fail(nullptr, LGC_EINVAL, "offsets must start at 0 and end at n");
    int ndev = 0;
    HIP_TRY(nullptr, hipGetDeviceCount(&ndev));
    if (device < 0 || device >= ndev) return fail(nullptr, LGC_EINVAL, "no HIP device %d", device);
    const uint32_t rows = (uint32_t)((n + kRow - 1) / kRow);
    std::vector<uint32_t> h_off(n_seg + 1), h_k(n_seg), h_out(n_seg + 1), h_rank(n_seg), h_row(rows);
    uint64_t total = 0;
    double expected = 0.0;
    uint32_t n_sampled = 0;
    for (uint64_t l = 0; l < n_seg; ++l) {
        if (offsets[l + 1] <= offsets[l]) return fail(nullptr, LGC_EINVAL, "segment %llu is empty or offsets descend", (unsigned long long)l);
        const uint64_t len = offsets[l + 1] - offsets[l];
        if (ks[l] > len) return fail(nullptr, LGC_EINVAL, "ks[%llu] exceeds the segment's length", (unsigned long long)l);
        h_off[l] = (uint32_t)offsets[l]; h_k[l] = (uint32_t)ks[l]; h_out[l] = (uint32_t)total;
        total += ks[l];
        // sampled: the candidate threshold is the rank-th largest of S sampled keys, S about n_l / 64
        // (whole 128-byte lines of 32 elements, at most 16 K keys), with six standard deviations of
        // head-room above the expected rank of the k-th key (see choose_rank)
        h_rank[l] = 0;
        if (len >= kSegMinSampled && ks[l] > 0) {
            uint64_t samples = (len / 64 + 31) / 32 * 32;
            if (samples < 2048) samples = 2048;
            if (samples > kSegSampleKeys) samples = kSegSampleKeys;
            const double rk = (double)ks[l] * (double)samples / (double)len;
            const double r = ceil(rk + 6.0 * sqrt(rk) + 8.0);
            if (r <= (double)samples / 4) {
                h_rank[l] = (uint32_t)r | ((uint32_t)(samples / 16) << 16);
                expected += (double)len * r / (double)samples;
                ++n_sampled;
            }
        }
    }
    h_off[n_seg] = (uint32_t)n; h_out[n_seg] = (uint32_t)total;
    if (total >= (1ull << 31)) return fail(nullptr, LGC_EINVAL, "sum of ks too large");
    {
        uint64_t l = 0;
        for (uint32_t r = 0; r < rows; ++r) {
            const uint64_t first = (uint64_t)r * kRow, end = first + kRow < n ? first + kRow : n;
            while (offsets[l + 1] <= first) ++l;
            h_row[r] = (uint32_t)l | (offsets[l + 1] < end ? 0x80000000u : 0u);
        }
    }
    DeviceGuard guard(device);
    if (!guard.ok) return fail(nullptr, LGC_EHIP, "cannot select device %d", device);
    lgc_segments *sg = new (std::nothrow) lgc_segments;
    if (!sg) return fail(nullptr, LGC_ENOMEM, "out of host memory");
    sg->device = device; sg->n = n; sg->total_k = total; sg->n_seg = (uint32_t)n_seg; sg->n_sampled = n_sampled;
    sg->rows = rows;
    double cap = 1.5 * expected + 16384.0;
    if (cap > 2.0e9) cap = 2.0e9;
    sg->cap = (uint32_t)align_up((size_t)cap, 4);
    const size_t words = (n_seg + 1) + n_seg + (n_seg + 1) + n_seg + rows;
    hipError_t e = hipMalloc((void **)&sg->dev, words * 4);
    if (e != hipSuccess) { delete sg; return fail(nullptr, LGC_ENOMEM, "hipMalloc of the segment plan: %s", hipGetErrorString(e)); }
    uint32_t *p = sg->dev;
    auto put = [&](uint32_t *&dst, const std::vector<uint32_t> &src) {
        dst = p;
        if (e == hipSuccess) e = hipMemcpy(p, src.data(), src.size() * 4, hipMemcpyHostToDevice);
        p += src.size();
    };
    put(sg->off, h_off); put(sg->k, h_k); put(sg->out, h_out); put(sg->rank, h_rank); put(sg->row_seg, h_row);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipFree(sg->dev);
        delete sg;
        return fail(nullptr, LGC_EHIP, "copying the segment plan: %s", hipGetErrorString(e));
    }
    *out = sg;
    return LGC_OK;
}

extern "C" lgc_status lgc_segments_create(lgc_segments **out, int device, uint64_t n, uint64_t n_seg,
                                          const uint64_t *offsets, const uint64_t *ks) {
    // the host-side tables are built before anything is allocated on the device, so nothing is
    // left behind if they cannot be
    return no_throw(nullptr, [&] { return segments_create(out, device, n, n_seg, offsets, ks); });
}

extern "C" void lgc_segments_destroy(lgc_segments *seg) {
    if (!seg) return;
    DeviceGuard guard(seg->device);
    (void)hipDeviceSynchronize();
    if (seg->dev) (void)hipFree(seg->dev);
    delete seg;
}

extern "C" uint64_t lgc_segments_total_k(const lgc_segments *seg) { return seg ? seg->total_k : 0; }

static bool seg_scratch_fits(const lgc_ctx *ctx, const lgc_segments *seg) {
    return (size_t)ctx->max_batch * seg->n_seg <= ctx->seg_t_words && ctx->seg_row_prefix &&
           (size_t)ctx->max_batch * seg->n_seg <= ctx->seg_carry_records &&
           2 * (size_t)ctx->max_batch * seg->cap <= ctx->seg_cand_words;
}

// only from lgc_reserve: the hot-path calls never allocate
static lgc_status ensure_seg_scratch(lgc_ctx *ctx, const lgc_segments *seg) {
    const size_t t_words = (size_t)ctx->max_batch * seg->n_seg;
    if (t_words > ctx->seg_t_words) {
        if (ctx->seg_t) { HIP_TRY(ctx, hipDeviceSynchronize()); HIP_TRY(ctx, hipFree(ctx->seg_t)); ctx->seg_t = nullptr; ctx->seg_t_words = 0; }
        HIP_TRY(ctx, hipMalloc((void **)&ctx->seg_t, t_words * 4));
        ctx->seg_t_words = t_words;
    }
    if (!ctx->seg_row_prefix)
        HIP_TRY(ctx, hipMalloc((void **)&ctx->seg_row_prefix, (size_t)ctx->max_batch * ctx->rows * 4));
    if (t_words > ctx->seg_carry_records) {
        if (ctx->seg_carry) { HIP_TRY(ctx, hipDeviceSynchronize()); HIP_TRY(ctx, hipFree(ctx->seg_carry)); ctx->seg_carry = nullptr; ctx->seg_carry_records = 0; }
        HIP_TRY(ctx, hipMalloc((void **)&ctx->seg_carry, t_words * sizeof(Carry)));
        ctx->seg_carry_records = t_words;
        HIP_TRY(ctx, hipMemset(ctx->seg_carry, 0, t_words * sizeof(Carry)));
        ctx->last_seg = nullptr;
    }
    const size_t c_words = 2 * (size_t)ctx->max_batch * seg->cap;
    if (c_words > ctx->seg_cand_words) {
        if (ctx->seg_cand) { HIP_TRY(ctx, hipDeviceSynchronize()); HIP_TRY(ctx, hipFree(ctx->seg_cand)); ctx->seg_cand = nullptr; ctx->seg_cand_words = 0; }
        HIP_TRY(ctx, hipMalloc((void **)&ctx->seg_cand, c_words * 4));
        ctx->seg_cand_words = c_words;
    }
    return LGC_OK;
}

static lgc_status run_segmented(lgc_ctx *ctx, const lgc_segments *seg, const float *g, float *u, float *v, int batch,
                                uint64_t stride, float m, float *out_vals, uint32_t *out_idx, void *stream) {
    if (!ctx) return fail(nullptr, LGC_EINVAL, "ctx is NULL");
    if (!seg) return fail(ctx, LGC_EINVAL, "segments is NULL");
    if (seg->device != ctx->device) return fail(ctx, LGC_EINVAL, "segment plan and context live on different devices");
    lgc_status s = check_common(ctx, seg->n, batch, stride);
    if (s != LGC_OK) return s;
    if (!v || (g && !u)) return fail(ctx, LGC_EINVAL, "v (and, with g, u) must not be NULL");
    if (!aligned(g, 4) || !aligned(u, 4) || !aligned(v, 4)) return fail(ctx, LGC_EINVAL, "pointer not 4-byte aligned");
    if ((s = check_select(ctx, seg->n, seg->total_k, out_vals, out_idx)) != LGC_OK) return s;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    hipStream_t st = (hipStream_t)stream;
    const bool fused = g != nullptr;
    const bool vec = aligned(v, 16) && (!u || aligned(u, 16)) && (!g || aligned(g, 16)) &&
                     (batch == 1 || stride % 4 == 0);
    if (seg->total_k == 0) {
        if (fused) launch_accumulate(g, u, v, (uint32_t)seg->n, batch, stride, m, vec, st);
        return LGC_OK;
    }
    if (!seg_scratch_fits(ctx, seg))
        return fail(ctx, LGC_EINVAL, "per-layer selection: scratch for this segment plan not reserved: call "
                                     "lgc_reserve(ctx, NULL, 0, 0, seg) once beforehand");
    SelArgs a = make_args(ctx, g, u, v, seg->n, stride, m, seg->total_k, out_vals, out_idx);
    a.n_seg = seg->n_seg; a.seg_off = seg->off; a.seg_k = seg->k; a.seg_out = seg->out; a.seg_rank = seg->rank;
    a.row_seg = seg->row_seg; a.seg_t = ctx->seg_t; a.row_prefix = ctx->seg_row_prefix;
    a.cap = seg->cap;
    a.cand_idx = ctx->seg_cand; a.cand_val = ctx->seg_cand + (size_t)ctx->max_batch * seg->cap;
    // per-layer thresholds carried from the previous selection, if that was one with this plan (a layer's record also
    // names its length and k); the list holds 4.5 k candidates in all (a layer's sample flags 3 k_l), a carried
    // threshold aims at 2 k_l and may be expected to flag 3.2 k_l at most, or k_l + 256 in a layer of few
    a.seg_carry = ctx->opt_carry && !ctx->single_state ? ctx->seg_carry : nullptr;
    a.carry_fresh = !(ctx->last_seg == seg && ctx->last_seg_k == seg->total_k);
    a.carry_target = (float)log2(2.0);
    a.carry_most = (float)log2(3.2);
    ctx->last_seg = seg; ctx->last_seg_k = seg->total_k;
    ctx->cur ^= 1;  // this call uses the clean set and cleans the other one for the next call
    if (seg->n_sampled) {
        launch_seg_estimate(a, batch, fused, vec, st);   // also clears the next call's state set
        launch_candidates(a, batch, fused, vec, st, profile_bracket(ctx));
        launch_gather(a, batch, st);
    } else {
        launch_clear(a.next_state, a.next_words, st);
        if (fused) {
            launch_accumulate(g, u, v, (uint32_t)seg->n, batch, stride, m, vec, st, profile_bracket(ctx));
        }
    }
    launch_seg_select(a, batch, vec, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, LGC_EHIP, "kernel launch: %s", hipGetErrorString(e));
    return LGC_OK;
}

extern "C" lgc_status lgc_topk_segmented(lgc_ctx *ctx, const lgc_segments *seg, float *v, float *u, int batch,
                                         uint64_t stride, float *out_vals, uint32_t *out_idx, void *stream) {
    return run_segmented(ctx, seg, nullptr, u, v, batch, stride, 0.f, out_vals, out_idx, stream);
}

extern "C" lgc_status lgc_accumulate_topk_segmented(lgc_ctx *ctx, const lgc_segments *seg, const float *g, float *u,
                                                    float *v, int batch, uint64_t stride, float momentum,
                                                    float *out_vals, uint32_t *out_idx, void *stream) {
    if (ctx && !g) return fail(ctx, LGC_EINVAL, "g must not be NULL");
    return run_segmented(ctx, seg, g, u, v, batch, stride, momentum, out_vals, out_idx, stream);
}

// ------------------------------------------------------------------ ring-allreduce pattern

static lgc_status gather_common(lgc_ctx *ctx, const float *g, float *u, float *v, uint64_t n, int batch,
                                uint64_t stride, float momentum, const uint32_t *idx, uint64_t k, float *out_vals,
                                void *stream) {
    lgc_status s = check_common(ctx, n, batch, stride);
    if (s != LGC_OK) return s;
    if (!v || (g && !u)) return fail(ctx, LGC_EINVAL, "v (and, with g, u) must not be NULL");
    if (k > n) return fail(ctx, LGC_EINVAL, "k > n");
    if (k > 0 && (!idx || !out_vals)) return fail(ctx, LGC_EINVAL, "idx and out_vals must not be NULL");
    if (!aligned(g, 4) || !aligned(u, 4) || !aligned(v, 4) || !aligned(idx, 4) || !aligned(out_vals, 4))
        return fail(ctx, LGC_EINVAL, "pointer not 4-byte aligned");
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    hipStream_t st = (hipStream_t)stream;
    if (g) {
        const bool vec = aligned(v, 16) && aligned(u, 16) && aligned(g, 16) && (batch == 1 || stride % 4 == 0);
        launch_accumulate(g, u, v, (uint32_t)n, batch, stride, momentum, vec, st, profile_bracket(ctx));
    }
    launch_gather_at(v, u, stride, (uint32_t)n, batch, idx, (uint32_t)k, out_vals, ctx->stats, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, LGC_EHIP, "kernel launch: %s", hipGetErrorString(e));
    return LGC_OK;
}

extern "C" lgc_status lgc_gather(lgc_ctx *ctx, float *v, float *u, uint64_t n, int batch, uint64_t stride,
                                 const uint32_t *idx, uint64_t k, float *out_vals, void *stream) {
    return gather_common(ctx, nullptr, u, v, n, batch, stride, 0.f, idx, k, out_vals, stream);
}

extern "C" lgc_status lgc_accumulate_gather(lgc_ctx *ctx, const float *g, float *u, float *v, uint64_t n, int batch,
                                            uint64_t stride, float momentum, const uint32_t *idx, uint64_t k,
                                            float *out_vals, void *stream) {
    if (ctx && !g) return fail(ctx, LGC_EINVAL, "g must not be NULL");
    return gather_common(ctx, g, u, v, n, batch, stride, momentum, idx, k, out_vals, stream);
}

extern "C" lgc_status lgc_average(lgc_ctx *ctx, const float *x, uint64_t len, int batch, float scale, float *out,
                                  void *stream) {
    if (!ctx) return fail(nullptr, LGC_EINVAL, "ctx is NULL");
    if (batch < 1 || batch > ctx->max_batch) return fail(ctx, LGC_EINVAL, "batch = %d outside [1, %d]", batch, ctx->max_batch);
    if (len >= (1ull << 32)) return fail(ctx, LGC_EINVAL, "len must be below 2^32");
    if (len > 0 && (!x || !out)) return fail(ctx, LGC_EINVAL, "NULL data pointer");
    if (!aligned(x, 4) || !aligned(out, 4)) return fail(ctx, LGC_EINVAL, "pointer not 4-byte aligned");
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    launch_average(x, (uint32_t)len, batch, scale, out, (hipStream_t)stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, LGC_EHIP, "kernel launch: %s", hipGetErrorString(e));
    return LGC_OK;
}

// ------------------------------------------------------------------ reservation

extern "C" lgc_status lgc_reserve(lgc_ctx *ctx, const lgc_ae *ae, uint64_t k, int batch, const lgc_segments *seg) {
    if (!ctx) return fail(nullptr, LGC_EINVAL, "ctx is NULL");
    if (ae) {
        if (ae->device != ctx->device) return fail(ctx, LGC_EINVAL, "autoencoder and context live on different devices");
        if (batch < 1 || batch > ctx->max_batch) return fail(ctx, LGC_EINVAL, "batch = %d outside [1, %d]", batch, ctx->max_batch);
        if (k > ctx->max_k) return fail(ctx, LGC_EINVAL, "k exceeds the context's max_k");
    }
    if (seg) {
        if (seg->device != ctx->device) return fail(ctx, LGC_EINVAL, "segment plan and context live on different devices");
        if (seg->n > ctx->max_n || seg->total_k > ctx->max_k) return fail(ctx, LGC_EINVAL, "segment plan exceeds the context's max_n / max_k");
    }
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    return no_throw(ctx, [&]() -> lgc_status {
        lgc_status s = LGC_OK;
        if (ae && k > 0 && (s = ensure_act(ctx, act_need(ae, k, batch))) != LGC_OK) return s;
        if (seg && (s = ensure_seg_scratch(ctx, seg)) != LGC_OK) return s;
        return LGC_OK;
    });
}

// ------------------------------------------------------------------ diagnostics

extern "C" lgc_status lgc_set_option(lgc_ctx *ctx, lgc_option opt, int64_t value) {
    if (!ctx) return fail(nullptr, LGC_EINVAL, "ctx is NULL");
    switch (opt) {
        case LGC_OPT_SELECT_PATH:
            if (value < 0 || value > 2) return fail(ctx, LGC_EINVAL, "LGC_OPT_SELECT_PATH takes 0, 1 or 2");
            ctx->opt_path = (int)value;
            ctx->exact_calls_left = ctx->penalty = 0;   // the automatic choice starts afresh: what fell back before the change does not count
            if (ctx->fell_back_host) ctx->fell_back_seen = *(volatile uint32_t *)ctx->fell_back_host;
            return LGC_OK;
        case LGC_OPT_PROFILE:
            ctx->opt_profile = value != 0;
            return LGC_OK;
        case LGC_OPT_CARRY_THRESHOLD:
            ctx->opt_carry = value != 0;
            {   // whatever has been recorded so far serves no later selection
                DeviceGuard guard(ctx->device);
                if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
                HIP_TRY(ctx, hipDeviceSynchronize());
                HIP_TRY(ctx, hipMemset(ctx->carry, 0, (size_t)ctx->max_batch * sizeof(Carry)));
                if (ctx->seg_carry) HIP_TRY(ctx, hipMemset(ctx->seg_carry, 0, ctx->seg_carry_records * sizeof(Carry)));
                ctx->last_seg = nullptr;
            }
            return LGC_OK;
    }
    return fail(ctx, LGC_EINVAL, "unknown option %d", (int)opt);
}

extern "C" lgc_status lgc_stats(lgc_ctx *ctx, uint64_t *fast, uint64_t *fallback, uint64_t *errors) {
    if (!ctx) return fail(nullptr, LGC_EINVAL, "ctx is NULL");
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    HIP_TRY(ctx, hipDeviceSynchronize());
    Stats h;
    HIP_TRY(ctx, hipMemcpy(&h, ctx->stats, sizeof h, hipMemcpyDeviceToHost));
    HIP_TRY(ctx, hipMemset(ctx->stats, 0, offsetof(Stats, carried)));
    if (fast) *fast = h.fast;
    if (fallback) *fallback = h.fallback;
    if (errors) *errors = h.errors;
    if (h.errors) return fail(ctx, LGC_EDEVICE, "%u device-side failures since the last lgc_stats", h.errors);
    return LGC_OK;
}

extern "C" lgc_status lgc_stats_carried(lgc_ctx *ctx, uint64_t *carried) {
    if (!ctx) return fail(nullptr, LGC_EINVAL, "ctx is NULL");
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    HIP_TRY(ctx, hipDeviceSynchronize());
    uint32_t h = 0;
    HIP_TRY(ctx, hipMemcpy(&h, &ctx->stats->carried, sizeof h, hipMemcpyDeviceToHost));
    HIP_TRY(ctx, hipMemset(&ctx->stats->carried, 0, sizeof h));
    if (carried) *carried = h;
    return LGC_OK;
}

extern "C" lgc_status lgc_profile_read(lgc_ctx *ctx, double *total_ms, uint64_t *launches) {
    if (!ctx) return fail(nullptr, LGC_EINVAL, "ctx is NULL");
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return fail(ctx, LGC_EHIP, "cannot select device %d", ctx->device);
    HIP_TRY(ctx, hipDeviceSynchronize());
    double sum = 0.0;
    for (size_t i = 0; i + 1 < ctx->ev_used; i += 2) {
        float ms = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->ev[i], ctx->ev[i + 1]));
        sum += ms;
    }
    if (total_ms) *total_ms = sum;
    if (launches) *launches = ctx->ev_used / 2;
    ctx->ev_used = 0;
    return LGC_OK;
}
