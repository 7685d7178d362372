// Internal declarations shared by the translation units of liblgc (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lgc.h"

namespace lgc {

// ---- geometry of the streaming / ordered-compaction kernels -----------------
constexpr int kBlock = 256;                     // threads per block (4 wavefronts of 64)
constexpr int kRows = 4;                        // float4 rows per thread
constexpr int kRowElems = kBlock * 4;           // 1024 elements per row
constexpr int kChunk = kRowElems * kRows;       // 4096 elements per block
constexpr int kWaves = kBlock / 64;

// ---- threshold estimate from a sample --------------------------------------
constexpr uint32_t kSample = 65536;             // sampled keys per node
constexpr uint32_t kSampleGroups = kSample / 4; // sampled in groups of 4 neighbours
constexpr int kSampleBins = 2048;               // first level: key >> 20
constexpr uint32_t kMinFastN = 1u << 18;        // below this the exact path is used directly (and is as fast)

// ---- histogram of the candidates above the estimate -------------------------
constexpr int kFineBins = 4096;
constexpr int kFineShift = 12;

// ---- exact radix select over the full vector (3 passes: 11 + 10 + 10 bits) --
constexpr int kRadixBins = 2048;

// ---- candidate bitmap: the candidate pass works in rows of 1024 consecutive elements, one
// wavefront per row; a row's candidate flags are 16 words of 64 bits (one full 128-byte line):
// word 4s+j, bit l  <->  element  row*1024 + 256 s + 4 l + j   (s, j in 0..3, l = lane)
constexpr int kRow = 1024;
constexpr int kRowWords = 16;
constexpr uint32_t kSuperRows = 8192;           // rows per group whose candidates are summed ahead of the gather

// The streaming kernels are launched over at most this many rows (a little over 2 GB of g, u, v
// traffic; the ResNet50-sized workload, 4 x 25 000 rows, is one launch): measured on MI355X,
// launches that move 3.5 GB and more sustain 70-72 % of the HBM peak instead of 75-77 %, whatever
// the split (more nodes per launch or longer vectors).
constexpr uint32_t kRowsPerLaunch = 104 * 1024;

// Per-node selection state, device memory.  It lives in a "state set" together with the
// histograms and chunk / block counts; there are two sets, used by alternate calls, and each
// call clears the set of the next one.
struct Sel {
    uint32_t t_est;       // fast path: candidates are the elements with key >= t_est
    uint32_t cand_total;  // number of candidates found (atomic adds in the gather kernel only)
    uint32_t thr;         // exact k-th largest key T*
    uint32_t quota;       // how many elements with key == T* are taken (lowest indices first)
    uint32_t fast_ok;     // 1: the fast path produced this node's output
    uint32_t carried;     // 1: t_est was carried over from earlier selections, not sampled
    uint32_t pad[10];
};
static_assert(sizeof(Sel) == 64, "Sel is one 64-byte record");

// Words that blocks of one kernel update with device-scope atomics while the kernel runs.  They
// live in a cache line of their own: a line that receives atomics from several XCDs must not
// also receive plain stores in the same kernel (each XCD has its own, non-coherent L2).
struct Ctr {
    uint32_t ticket;      // exact path in one launch: next share to hand out (phase = ticket / shares)
    uint32_t done[5];     // completed shares of each phase
    uint32_t sampled;     // sampling blocks of the node that have finished (the last one works out the estimate)
    uint32_t pad[25];
};
static_assert(sizeof(Ctr) == 128, "Ctr is one 128-byte line");

struct Stats {
    uint32_t fast, fallback, errors;
    uint32_t carried;     // selections whose candidate threshold was carried over instead of sampled
};

// Per-node record that outlives the call (it is in neither state set): the exact thresholds T* of the last
// selections of the context, as log2 of their magnitude, and, when they have moved smoothly enough, the candidate
// threshold that the next selection may use without sampling.  Written by the one thread that reports a
// selection's outcome, read by the sampling kernel of the next selection.  Every selection of the context ends by
// writing it, on the device: the fast path its outcome, the exact path and the per-layer selection "nothing on
// record" (len = 0, no offer); so the record is always the previous selection's, also in a replayed HIP graph.
struct Carry {
    uint32_t carried_now; // per-layer selection: the layer's threshold of the call under way was taken from this record
    uint32_t n, k;        // its vector length and k: the record only serves a selection of the same shape
    uint32_t len;         // fast-path selections in a row so far (counted up to 255; 0: none)
    float log2_t[3];      // log2 |T*| of the last min(len, 3) selections, latest first
    uint32_t next_t_est;  // candidate threshold (key) offered to the next selection; 0: sample
    uint32_t fails;       // carried thresholds that sent their selection to the exact path, up to 5; each doubles the
                          // selections in a row required before the next offer, 64 carried selections that held take one off
    uint32_t held;        // carried selections that held since `fails` last changed
    float miss;           // how far T* lay from the trend of the two selections before it (log2), largest of the
                          // recent selections: each selection's own miss, or 0.85 of the value before
    uint32_t pad[5];
};
static_assert(sizeof(Carry) == 64, "Carry is one 64-byte record");

// Everything the selection kernels need; passed by value.
struct SelArgs {
    const float *g;   // fresh gradient (fused source only)
    float *u;         // momentum buffer (nullable for plain selection)
    float *v;         // accumulated gradient
    uint64_t stride;  // elements between nodes
    uint32_t n;       // elements per node
    uint32_t k;       // selected per node
    float momentum;
    uint32_t node0, row_begin, row_end;   // the streaming kernel's share of this launch: nodes node0.., rows [row_begin, row_end)
    uint32_t rank;    // rank of the sample's order statistic used as estimate
    uint32_t cap;     // capacity of the gathered candidate list, per node
    uint32_t rows;    // bitmap rows per node (stride of row_count; bitmap stride is rows * kRowWords)
    uint32_t status_cand_stride, status_exact_stride;  // 64-bit words per node: chunk counts of the candidate list, block counts of the exact path
    uint32_t spin_limit;      // bound of a wait for the shares of the previous phase (exact path in one launch)
    int force;                // exact path chosen by the host (ignore fast_ok)
    Stats *stats;
    uint32_t *notify;         // two pinned host words (device address; null: none): a selection stores notify_value to word 0
                              // when it falls back, to word 1 when the fast path served it
    uint32_t notify_value;
    Carry *carry;             // [batch] thresholds carried from selection to selection (null: always sample)
    float carry_target;       // log2 of (candidates aimed at by a carried threshold) / k
    float carry_most;         // log2 of (most candidates a carried threshold may be expected to flag) / k
    Carry *seg_carry;         // per-layer selection: [batch][n_seg] records, one per layer and node (null: always sample)
    uint32_t carry_fresh;     // per-layer selection: the records are not the previous selection's
    // current state set
    Sel *sel;
    Ctr *ctr;
    uint32_t *sample_hist;    // [batch][kSampleBins]
    uint32_t *fine_hist;      // [batch][kFineBins]
    uint32_t *level2_hist;    // [batch][kFineBins]
    uint32_t *radix_hist;     // [batch][3][kRadixBins]
    unsigned long long *status_cand;   // per 4096-candidate chunk of a long list: keys above T* (high half), equal to T* (low half)
    unsigned long long *status_exact;  // exact path: per block, keys above T* (high half) and equal to it (low half) in its run of v
    // state set of the next call, cleared by this one
    uint32_t *next_state;
    uint32_t next_words;
    // bulk scratch
    uint32_t *samples;        // [batch][kSample]
    uint32_t *row_count;      // [batch][rows]  candidates per row
    uint32_t *row_super;      // [batch][supers] candidates per group of kSuperRows rows (vectors of more than one group)
    uint32_t supers;           // groups per node in row_super; 0: the gather adds up the row counts themselves
    unsigned long long *bitmap;  // [batch][rows][kRowWords]
    uint32_t *cand_idx;       // [batch][cap]  gathered, index-ordered
    uint32_t *cand_val;
    float *out_vals;          // [batch][k]
    uint32_t *out_idx;        // [batch][k]
    // per-layer selection (null / 0 otherwise): the segment plan and the per-call thresholds
    uint32_t n_seg;
    const uint32_t *seg_off;  // [n_seg + 1] first element of every segment, then n
    const uint32_t *seg_k;    // [n_seg]     values kept per segment
    const uint32_t *seg_out;  // [n_seg + 1] first output slot of every segment (prefix sums of seg_k)
    const uint32_t *seg_rank; // [n_seg]     0 = not sampled; else rank of the sample's order statistic (low 16
                              //             bits) and the number of sampling threads (high 16 bits)
    const uint32_t *row_seg;  // [rows]      segment of the row's first element | bit 31: crosses a boundary
    uint32_t *seg_t;          // [batch][n_seg] candidate thresholds of this call
    uint32_t *row_prefix;     // [batch][rows]  candidates listed before each row (written by the gather kernel)
};

// launchers (topk.hip) — all asynchronous on `st`
// Timing of a streaming call's launches (null events: none): `start` is given the start time of the first
// launch, `stop` the end time of the last one, by the launches themselves, with no packet of their own in the queue.
struct Bracket {
    hipEvent_t start = nullptr, stop = nullptr;
};
void launch_accumulate(const float *g, float *u, float *v, uint32_t n, int batch, uint64_t stride,
                       float momentum, bool vec, hipStream_t st, Bracket br = Bracket());
void launch_clear(uint32_t *words, uint32_t count, hipStream_t st);
void launch_sample(const SelArgs &a, int batch, bool fused, bool vec, hipStream_t st);
void launch_candidates(const SelArgs &a, int batch, bool fused, bool vec, hipStream_t st, Bracket br = Bracket());
void launch_gather(const SelArgs &a, int batch, hipStream_t st);
bool launch_output_from_candidates(const SelArgs &a, int batch, bool direct, bool vec, int cus, hipStream_t st);
void launch_exact(const SelArgs &a, int batch, bool vec, int cus, hipStream_t st);
// per-layer selection (segmented.hip)
void launch_seg_estimate(const SelArgs &a, int batch, bool fused, bool vec, hipStream_t st);
void launch_seg_select(const SelArgs &a, int batch, bool vec, hipStream_t st);
void launch_innovation(const float *vals, float *out, uint32_t n, int batch, uint32_t n_seg, const uint32_t *seg_off,
                       const uint32_t *seg_k, bool vec, Stats *stats, hipStream_t st);

// autoencoder.hip
struct LayerDev {
    int c_in, c_out, ksize, stride;
    const float *w, *b;         // device
    const float *wt = nullptr;  // device: weights in contraction-major order for the MFMA kernels, or null
};
void launch_conv1d(const float *in, float *out, const LayerDev &l, uint32_t l_in, uint32_t l_out,
                   int batch, bool act, float slope, hipStream_t st);
// extra (nullable): one more input channel per node, [batch][l_in], appended after the c_in - 1 channels of `in`
void launch_conv_transpose1d(const float *in, float *out, const LayerDev &l, uint32_t l_in,
                             uint32_t l_out, int batch, bool act, float slope, hipStream_t st,
                             const float *extra = nullptr);
// whole two-layer stacks in one launch; false = shape not covered (nothing launched)
bool launch_encoder2(const float *x, float *z, const LayerDev &a, const LayerDev &b, uint32_t l0, uint32_t l1,
                     uint32_t l2, int batch, float slope, hipStream_t st);
bool launch_decoder2(const float *z, float *y, const LayerDev &a, const LayerDev &b, uint32_t l2, uint32_t l1,
                     uint32_t l0, int batch, float slope, hipStream_t st);
bool launch_decoder3i(const float *z, const float *innov, float *y, const LayerDev &a, const LayerDev &b,
                      const LayerDev &c, uint32_t l2, uint32_t l1, uint32_t l0, int batch, float slope, hipStream_t st);
void launch_scatter(const float *vals, const uint32_t *idx, uint32_t k, float scale, float *dense,
                    uint32_t n, Stats *stats, hipStream_t st);

// all nodes in one launch (positions ascending within each node); false = batch too large for it
bool launch_scatter_nodes(const float *vals, const uint32_t *idx, uint32_t k, int batch, float scale, float *dense,
                          uint32_t n, Stats *stats, hipStream_t st);

// ae_mfma.hip: deep kernel-3 / stride-2 layers on the matrix cores; false = layer not covered (nothing launched)
void launch_weights_contraction_major(const float *w, float *wt, int c_in, int c_out, bool transposed, hipStream_t st);
// tail (nullable): the kernel-1 / stride-1 layer that follows, applied in the same launch when its shape allows
// (64 -> at most 4 channels after a convolution, 32 -> 1 after a transposed one); `out` is then the tail's output
bool launch_conv3s2_mfma(const float *in, float *out, const LayerDev &l, uint32_t l_in, uint32_t l_out, int batch,
                         bool act, float slope, hipStream_t st, const LayerDev *tail = nullptr, bool tail_act = false);
// split contraction: how many ways (1 = not at all), and the launch (partial sums to `part`, then a finish kernel)
int conv3s2_mfma_splits(const LayerDev &l, uint32_t l_out, int batch);
bool launch_conv3s2_mfma_splitk(const float *in, float *part, float *out, const LayerDev &l, uint32_t l_in, uint32_t l_out,
                                int batch, int splits, bool act, float slope, hipStream_t st, const LayerDev *tail = nullptr,
                                bool tail_act = false);
bool launch_conv3s2_mfma_head(const float *x, float *out, const LayerDev &head, const LayerDev &l, uint32_t l_x,
                              uint32_t l_in, uint32_t l_out, int batch, bool act, float slope, hipStream_t st);
bool launch_convt3s2_mfma(const float *in, float *out, const LayerDev &l, uint32_t l_in, uint32_t l_out, int batch,
                          bool act, float slope, hipStream_t st, const LayerDev *tail = nullptr, bool tail_act = false);
bool launch_convt3s2_mfma_head(const float *z, float *out, const LayerDev &h1, const LayerDev &h2, const LayerDev &l,
                               uint32_t l_z, uint32_t l_in, uint32_t l_out, int batch, bool act, float slope,
                               hipStream_t st);
void launch_gather_at(float *v, float *u, uint64_t stride, uint32_t n, int batch, const uint32_t *idx, uint32_t k,
                      float *out, Stats *stats, hipStream_t st);
void launch_average(const float *x, uint32_t len, int batch, float scale, float *out, hipStream_t st);

}  // namespace lgc
