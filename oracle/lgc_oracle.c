/*
 * CPU oracle for the per-node compression path of Learned Gradient Compression.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
 * definition that the GPU library is checked against.  It shares no code,
 * header, table or helper with the HIP path and must never be called from it.
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Every function states the passage of the paper it follows.  Where the paper
 * is silent the reading taken is stated next to the code.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -shared -fPIC
 * (no FMA contraction: each fp32 operation below rounds once, on its own).
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ helpers */

static uint32_t f32_bits(float x) { uint32_t b; memcpy(&b, &x, 4); return b; }

/* Magnitude key: the IEEE-754 bit pattern with the sign cleared.  For finite
 * values it orders exactly like |x|; it also gives every other fp32 value a
 * place (NaN above Inf, -0 equal to +0), so the order is total. */
static uint32_t mag_key(float x) { return f32_bits(x) & 0x7FFFFFFFu; }

/* ------------------------------------------------------------- accumulation */

/*
 * Local accumulation with momentum correction.
 *
 * Alg. 1 / Alg. 2, first line of the layer loop: the fresh gradient is added
 * to the carried residual, g_l = grad + g_acc.  Sec. V-A (last paragraph) has
 * the unsent part accumulated with a momentum correction in the manner of DGC
 * and gives no formula; the reading taken is DGC's published rule
 *     u <- m*u + g        (momentum buffer)
 *     v <- v + u          (accumulated gradient, the paper's g_acc / g_l)
 * With m = 0 this is exactly the paper's line.  Each arithmetic operation is a
 * separate fp32 rounding (product, then sum, then sum).
 */
void oracle_accumulate(const float *g, float *u, float *v, size_t n, float m)
{
    for (size_t i = 0; i < n; ++i) {
        volatile float prod = m * u[i];   /* volatile: forbid any fusing */
        volatile float un = prod + g[i];
        volatile float vn = v[i] + un;
        u[i] = un;
        v[i] = vn;
    }
}

/* ------------------------------------------------------------------- top-k */

static int cmp_u64_desc(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return (x < y) - (x > y);
}
static int cmp_u32_asc(const void *a, const void *b)
{
    uint32_t x = *(const uint32_t *)a, y = *(const uint32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Top-k magnitude selection with residual update.
 *
 * Alg. 1 / Alg. 2: threshold = smallest of the top values of |g_l|,
 * mask = |g_l| >= threshold, g~ = mask .* g_l, g_acc keeps (not mask) .* g_l.
 * (The printed residual line adds g_acc once more although g_l already holds
 * it; the reading taken is g_acc <- (not mask) .* g_l.)
 * Sec. V-A fixes the size of g~ at exactly mu values, so ties at the
 * threshold are cut: the order is (magnitude descending, index ascending) and
 * the first k positions of that order are selected.  The selected values are
 * reported in ascending index order, which is what mask .* g_l with the zeros
 * dropped gives.  Momentum-factor masking (DGC): u is zeroed where sent.
 *
 * Plain definition: sort ALL positions, take the first k.
 * u may be NULL.  Returns 0, or -1 on bad arguments / out of memory.
 */
int oracle_topk(float *v, float *u, size_t n, size_t k,
                float *out_vals, uint32_t *out_idx)
{
    if (k > n || n > 0xFFFFFFFFull) return -1;
    if (k == 0) return 0;
    uint64_t *ord = (uint64_t *)malloc(n * sizeof(uint64_t));
    if (!ord) return -1;
    /* composite (key, reversed index): descending order of the pair is
     * key descending, then index ascending */
    for (size_t i = 0; i < n; ++i)
        ord[i] = ((uint64_t)mag_key(v[i]) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)i);
    qsort(ord, n, sizeof(uint64_t), cmp_u64_desc);
    for (size_t j = 0; j < k; ++j)
        out_idx[j] = 0xFFFFFFFFu - (uint32_t)(ord[j] & 0xFFFFFFFFu);
    free(ord);
    qsort(out_idx, k, sizeof(uint32_t), cmp_u32_asc);
    for (size_t j = 0; j < k; ++j) {
        uint32_t i = out_idx[j];
        out_vals[j] = v[i];
        v[i] = 0.0f;
        if (u) u[i] = 0.0f;
    }
    return 0;
}

/* -------------------------------------------------------------- autoencoder */

static double act(double x, double slope) { return x > 0.0 ? x : slope * x; }

/*
 * One 1-D convolution layer (Sec. IV-C, Table I: 1-D kernels of size 3 with
 * stride 2, and a size-1 stride-1 layer).  Padding is not given in the paper;
 * the reading taken is pad = (ksize-1)/2, so
 *     L_out = floor((L_in + 2*pad - ksize) / stride) + 1.
 *     out[co][p] = b[co] + sum_ci sum_t W[co][ci][t] * in[ci][p*stride - pad + t]
 * with taps outside [0, L_in) contributing nothing.  fp64 accumulation, one
 * rounding to fp32 at the end.  apply_act: leaky-ReLU with the given slope
 * (slope 0 = ReLU).
 */
size_t oracle_conv_len(size_t l_in, int ksize, int stride)
{
    int pad = (ksize - 1) / 2;
    if (l_in == 0) return 0;
    return (l_in + 2 * (size_t)pad - (size_t)ksize) / (size_t)stride + 1;
}

void oracle_conv1d(const float *in, int c_in, size_t l_in,
                   const float *w, const float *b, int c_out,
                   int ksize, int stride, int apply_act, float slope,
                   float *out)
{
    int pad = (ksize - 1) / 2;
    size_t l_out = oracle_conv_len(l_in, ksize, stride);
    for (int co = 0; co < c_out; ++co)
        for (size_t p = 0; p < l_out; ++p) {
            double acc = (double)b[co];
            for (int ci = 0; ci < c_in; ++ci)
                for (int t = 0; t < ksize; ++t) {
                    long long q = (long long)p * stride - pad + t;
                    if (q < 0 || q >= (long long)l_in) continue;
                    acc += (double)w[((size_t)co * c_in + ci) * ksize + t] *
                           (double)in[(size_t)ci * l_in + (size_t)q];
                }
            if (apply_act) acc = act(acc, (double)slope);
            out[(size_t)co * l_out + p] = (float)acc;
        }
}

/*
 * One 1-D transposed convolution ("deconvolution", Sec. IV-C, Table II): the
 * adjoint of the layer above.  Input position p sends W[ci][co][t]*in[ci][p]
 * to output position q = p*stride - pad + t; positions outside [0, l_out) are
 * dropped.  l_out is given by the caller (the length the mirrored encoder
 * layer consumed), which fixes the otherwise ambiguous output length.
 * Weight layout W[c_in][c_out][ksize].
 * Returns 0, or -1 if the row of fp64 accumulators cannot be allocated.
 */
int oracle_conv_transpose1d(const float *in, int c_in, size_t l_in,
                             const float *w, const float *b, int c_out,
                             int ksize, int stride, size_t l_out,
                             int apply_act, float slope, float *out)
{
    int pad = (ksize - 1) / 2;
    double *acc = (double *)malloc((l_out ? l_out : 1) * sizeof(double));
    if (!acc) return -1;
    for (int co = 0; co < c_out; ++co) {
        for (size_t q = 0; q < l_out; ++q) acc[q] = (double)b[co];
        for (int ci = 0; ci < c_in; ++ci)
            for (size_t p = 0; p < l_in; ++p)
                for (int t = 0; t < ksize; ++t) {
                    long long q = (long long)p * stride - pad + t;
                    if (q < 0 || q >= (long long)l_out) continue;
                    acc[q] += (double)w[((size_t)ci * c_out + co) * ksize + t] *
                              (double)in[(size_t)ci * l_in + p];
                }
        for (size_t q = 0; q < l_out; ++q) {
            double a = acc[q];
            if (apply_act) a = act(a, (double)slope);
            out[(size_t)co * l_out + q] = (float)a;
        }
    }
    free(acc);
    return 0;
}

/*
 * Encoder E_c: the layers in order, non-linearity after every layer but the
 * last (the latent is not rectified).  Sec. IV, eq. g^c = E_c(g); Table I.
 * chan[0..n_layers], ksize[l], stride[l]; w[l] = W[c_out][c_in][ksize],
 * b[l] = [c_out].  x is [chan[0]][k]; latent is [chan[n_layers]][L_latent].
 * Returns the latent length per channel, or (size_t)-1 on allocation failure.
 */
size_t oracle_encode(const float *x, size_t k, int n_layers, const int *chan,
                     const int *ksize, const int *stride,
                     const float *const *w, const float *const *b,
                     float slope, float *latent)
{
    size_t len = k;
    const float *cur = x;
    float *owned = NULL;
    for (int l = 0; l < n_layers; ++l) {
        size_t l_out = oracle_conv_len(len, ksize[l], stride[l]);
        int last = (l == n_layers - 1);
        float *dst = last ? latent
                          : (float *)malloc(((size_t)chan[l + 1] * l_out + 1) * sizeof(float));
        if (!dst) { free(owned); return (size_t)-1; }
        oracle_conv1d(cur, chan[l], len, w[l], b[l], chan[l + 1], ksize[l], stride[l],
                      !last, slope, dst);
        free(owned);
        owned = last ? NULL : dst;
        cur = dst;
        len = l_out;
    }
    return len;
}

/*
 * Decoder D_c: transposed layers in order, non-linearity after every layer
 * but the last.  Sec. IV, eq. g^rec = D_c(.); Table II.  out_len[l] is the
 * output length of decoder layer l (the caller derives it from the encoder's
 * length chain so that the final length is k again).  A layer with stride 1
 * and ksize 1 is an ordinary 1x1 convolution, which the transposed form with
 * W[c_in][c_out][1] also expresses.
 */
int oracle_decode(const float *latent, size_t l_latent, int n_layers, const int *chan,
                  const int *ksize, const int *stride, const size_t *out_len,
                  const float *const *w, const float *const *b,
                  float slope, float *rec)
{
    size_t len = l_latent;
    const float *cur = latent;
    float *owned = NULL;
    for (int l = 0; l < n_layers; ++l) {
        int last = (l == n_layers - 1);
        float *dst = last ? rec
                          : (float *)malloc(((size_t)chan[l + 1] * out_len[l] + 1) * sizeof(float));
        if (!dst) { free(owned); return -1; }
        int rc = oracle_conv_transpose1d(cur, chan[l], len, w[l], b[l], chan[l + 1], ksize[l], stride[l],
                                         out_len[l], !last, slope, dst);
        if (rc != 0) { if (!last) free(dst); free(owned); return -1; }
        free(owned);
        owned = last ? NULL : dst;
        cur = dst;
        len = out_len[l];
    }
    return 0;
}

/* ------------------------------------------------------------------ scatter */

/*
 * Placement of a node's (reconstructed) values back at their positions and
 * averaging over nodes: Sec. V-B, g^rec = (1/K) sum_k g_k^rec, then the weight
 * update uses the dense result.  One call adds one node's share:
 *     dense[idx[j]] <- dense[idx[j]] + scale*vals[j]
 * product rounded to fp32, then the sum rounded to fp32.
 * Returns -1 if an index is out of range.
 */
int oracle_scatter(const float *vals, const uint32_t *idx, size_t k, float scale,
                   float *dense, size_t n)
{
    for (size_t j = 0; j < k; ++j) {
        if (idx[j] >= n) return -1;
        volatile float s = scale * vals[j];
        volatile float d = dense[idx[j]] + s;
        dense[idx[j]] = d;
    }
    return 0;
}

/* ------------------------------------------------------ per-layer selection */

/*
 * Per-layer top-k — Sec. V-A and the layer loop of Alg. 1 / Alg. 2: the
 * gradient of every layer l (a contiguous segment of n_l elements of the flat
 * vector) is thresholded on its own, mu_l values are kept, and the kept values
 * of all layers are concatenated in layer order.
 *
 * offsets[0..n_seg]: segment l is [offsets[l], offsets[l+1]); offsets[0] = 0,
 * offsets[n_seg] = n.  ks[l] = mu_l <= n_l.  Each segment is selected exactly
 * like the flat vector in oracle_topk (same key, same tie rule); positions are
 * reported in the flat vector's numbering, so the concatenation is ascending.
 * out_vals / out_idx hold sum(ks) entries.
 */
int oracle_topk_segmented(float *v, float *u, size_t n, size_t n_seg,
                          const uint64_t *offsets, const uint64_t *ks,
                          float *out_vals, uint32_t *out_idx)
{
    if (n_seg == 0 || offsets[0] != 0 || offsets[n_seg] != n) return -1;
    size_t o = 0;
    for (size_t l = 0; l < n_seg; ++l) {
        if (offsets[l + 1] < offsets[l]) return -1;
        size_t lo = (size_t)offsets[l], len = (size_t)(offsets[l + 1] - offsets[l]);
        size_t k = (size_t)ks[l];
        if (oracle_topk(v + lo, u ? u + lo : NULL, len, k, out_vals + o, out_idx + o) != 0)
            return -1;
        for (size_t j = 0; j < k; ++j) out_idx[o + j] += (uint32_t)lo;
        o += k;
    }
    return 0;
}

/* --------------------------------------- ring-allreduce: shared positions */

/*
 * Values at positions chosen by another node — Sec. V-A, ring-allreduce
 * pattern: one node selects, sends its positions, and every other node builds
 * its own g~ from the SAME positions.  The mask / residual lines of Alg. 2 then
 * apply with that mask: what is sent leaves the residual (and, with the
 * momentum correction, the momentum buffer).
 *     vals[j] = v[idx[j]] ; v[idx[j]] = +0 ; u[idx[j]] = +0
 * idx must be distinct.  u may be NULL.
 */
int oracle_gather(float *v, float *u, size_t n, const uint32_t *idx, size_t k, float *out_vals)
{
    for (size_t j = 0; j < k; ++j) {
        if (idx[j] >= n) return -1;
        out_vals[j] = v[idx[j]];
        v[idx[j]] = 0.0f;
        if (u) u[idx[j]] = 0.0f;
    }
    return 0;
}

/*
 * Average of the nodes' compressed representations — Sec. V-C / Alg. 2:
 * g^avg = (1/K) sum_k g^c_k.  Reading taken for the rounding: like the
 * scatter, every term is scaled first and the terms are added in node order,
 *     out[i] = (..((0 + scale*x_0[i]) + scale*x_1[i]) + ...) + scale*x_{K-1}[i],
 * each product and each sum rounded to fp32 on its own.  x: [batch][len].
 */
void oracle_average(const float *x, size_t batch, size_t len, float scale, float *out)
{
    for (size_t i = 0; i < len; ++i) {
        float acc = 0.0f;
        for (size_t b = 0; b < batch; ++b) {
            volatile float s = scale * x[b * len + i];
            volatile float a = acc + s;
            acc = a;
        }
        out[i] = acc;
    }
}

/* ------------------------------------------- parameter server: innovation */

/*
 * Innovation component — Alg. 1 (threshold_inv, mask_inv, g~^I = g~ .* mask_inv)
 * and Sec. IV-C: a vector of the size of g~ holding the top-magnitude values
 * of g~ and zeros elsewhere.  Alg. 1 forms it inside the layer loop, so it is
 * taken per layer: segment l of g~ is [offsets[l], offsets[l+1]) and keeps
 * ks[l] values (same key and tie rule as the selection itself, exactly ks[l]
 * kept).  One segment covering everything gives the flat form.
 * vals is not modified.  out: [k], +0 where nothing is kept.
 */
int oracle_innovation(const float *vals, size_t k, size_t n_seg, const uint64_t *offsets,
                      const uint64_t *ks, float *out)
{
    if (n_seg == 0 || offsets[0] != 0 || offsets[n_seg] != k) return -1;
    for (size_t j = 0; j < k; ++j) out[j] = 0.0f;
    for (size_t l = 0; l < n_seg; ++l) {
        if (offsets[l + 1] < offsets[l]) return -1;
        size_t lo = (size_t)offsets[l], len = (size_t)(offsets[l + 1] - offsets[l]);
        size_t kk = (size_t)ks[l];
        if (kk > len) return -1;
        if (kk == 0) continue;
        uint64_t *ord = (uint64_t *)malloc(len * sizeof(uint64_t));
        if (!ord) return -1;
        for (size_t i = 0; i < len; ++i)
            ord[i] = ((uint64_t)mag_key(vals[lo + i]) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)i);
        qsort(ord, len, sizeof(uint64_t), cmp_u64_desc);
        for (size_t j = 0; j < kk; ++j) {
            size_t i = 0xFFFFFFFFu - (uint32_t)(ord[j] & 0xFFFFFFFFu);
            out[lo + i] = vals[lo + i];
        }
        free(ord);
    }
    return 0;
}
