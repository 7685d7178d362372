/* Runs every function of the CPU oracle on small inputs held in exactly-sized heap blocks, so that
 * a build with -fsanitize=address,undefined reports any access outside them, any use of freed or
 * uninitialised-size memory and any undefined arithmetic in the oracle.  Test infrastructure: it
 * checks nothing about the values (the pins do that); it prints one checksum so that the calls
 * cannot be optimised away.  Sizes include the degenerate ones: n = 1, k = 0, k = n, odd lengths. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void oracle_accumulate(const float *g, float *u, float *v, size_t n, float m);
int oracle_topk(float *v, float *u, size_t n, size_t k, float *out_vals, uint32_t *out_idx);
size_t oracle_conv_len(size_t l_in, int ksize, int stride);
size_t oracle_encode(const float *x, size_t k, int n_layers, const int *chan, const int *ksize, const int *stride,
                     const float *const *w, const float *const *b, float slope, float *latent);
int oracle_decode(const float *latent, size_t l_latent, int n_layers, const int *chan, const int *ksize,
                  const int *stride, const size_t *out_len, const float *const *w, const float *const *b,
                  float slope, float *rec);
int oracle_scatter(const float *vals, const uint32_t *idx, size_t k, float scale, float *dense, size_t n);
int oracle_topk_segmented(float *v, float *u, size_t n, size_t n_seg, const uint64_t *offsets, const uint64_t *ks,
                          float *out_vals, uint32_t *out_idx);
int oracle_gather(float *v, float *u, size_t n, const uint32_t *idx, size_t k, float *out_vals);
void oracle_average(const float *x, size_t batch, size_t len, float scale, float *out);
int oracle_innovation(const float *vals, size_t k, size_t n_seg, const uint64_t *offsets, const uint64_t *ks,
                      float *out);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static float rnd(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((int32_t)(state >> 33) % 2001 - 1000) * 1e-3f;   /* few distinct values: ties occur */
}
static float *vec(size_t n)
{
    float *p = (float *)malloc((n ? n : 1) * sizeof(float));
    if (!p) exit(2);
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}

static double checksum = 0.0;
static void fold(const float *p, size_t n) { for (size_t i = 0; i < n; ++i) checksum += p[i]; }

static void selection(size_t n, size_t k)
{
    float *g = vec(n), *u = vec(n), *v = vec(n), *vals = vec(k);
    uint32_t *idx = (uint32_t *)malloc((k ? k : 1) * sizeof(uint32_t));
    oracle_accumulate(g, u, v, n, 0.9f);
    if (oracle_topk(v, u, n, k, vals, idx) != 0) exit(3);
    fold(vals, k);
    if (oracle_topk(v, NULL, n, k, vals, idx) != 0) exit(3);     /* without momentum buffer */
    float *dense = vec(n);
    if (oracle_scatter(vals, idx, k, 0.25f, dense, n) != 0) exit(3);
    float *got = vec(k);
    if (oracle_gather(v, u, n, idx, k, got) != 0) exit(3);
    fold(dense, n); fold(got, k);
    /* per layer: three segments (one possibly empty), keeping nothing / one / everything */
    if (n >= 3) {
        uint64_t off[4] = {0, n / 3, n / 3, n}, ks[3] = {n / 3 ? 1 : 0, 0, n - n / 3};
        size_t total = (size_t)(ks[0] + ks[1] + ks[2]);
        float *sv = vec(total), *inn = vec(total);
        uint32_t *si = (uint32_t *)malloc((total ? total : 1) * sizeof(uint32_t));
        float *v2 = vec(n), *u2 = vec(n);
        if (oracle_topk_segmented(v2, u2, n, 3, off, ks, sv, si) != 0) exit(3);
        uint64_t ooff[4] = {0, ks[0], ks[0] + ks[1], total}, iks[3] = {ks[0], 0, ks[2] / 10};
        if (oracle_innovation(sv, total, 3, ooff, iks, inn) != 0) exit(3);
        fold(sv, total); fold(inn, total);
        free(sv); free(inn); free(si); free(v2); free(u2);
    }
    free(g); free(u); free(v); free(vals); free(idx); free(dense); free(got);
}

/* encoder 1 -> c1 -> c2 (kernel 3, stride 2) and its mirrored decoder, then the same with a
 * kernel-1 / stride-1 layer in the middle */
static void autoencoder(size_t k, int c1, int c2, int with_k1)
{
    int n_layers = with_k1 ? 3 : 2;
    int chan[4] = {1, c1, c2, c2}, ks[3] = {3, 3, 1}, st[3] = {2, 2, 1};
    int dchan[4], dks[3], dst[3];
    size_t len[4];
    len[0] = k;
    for (int l = 0; l < n_layers; ++l) len[l + 1] = oracle_conv_len(len[l], ks[l], st[l]);
    const float *w[3], *b[3], *dw[3], *db[3];
    size_t out_len[3];
    for (int l = 0; l < n_layers; ++l) {
        w[l] = vec((size_t)chan[l + 1] * chan[l] * ks[l]);
        b[l] = vec((size_t)chan[l + 1]);
        int m = n_layers - 1 - l;                       /* decoder layer l mirrors encoder layer m */
        dchan[l] = chan[m + 1]; dks[l] = ks[m]; dst[l] = st[m]; out_len[l] = len[m];
    }
    dchan[n_layers] = chan[0];
    for (int l = 0; l < n_layers; ++l) {
        dw[l] = vec((size_t)dchan[l] * dchan[l + 1] * dks[l]);
        db[l] = vec((size_t)dchan[l + 1]);
    }
    float *x = vec(k), *lat = vec((size_t)chan[n_layers] * len[n_layers]), *rec = vec(k);
    if (oracle_encode(x, k, n_layers, chan, ks, st, w, b, 0.01f, lat) != len[n_layers]) exit(4);
    if (oracle_decode(lat, len[n_layers], n_layers, dchan, dks, dst, out_len, dw, db, 0.0f, rec) != 0) exit(4);
    fold(lat, (size_t)chan[n_layers] * len[n_layers]); fold(rec, k);
    float *avg = vec(k);
    oracle_average(rec, 1, k, 0.5f, avg);
    fold(avg, k);
    for (int l = 0; l < n_layers; ++l) { free((void *)w[l]); free((void *)b[l]); free((void *)dw[l]); free((void *)db[l]); }
    free(x); free(lat); free(rec); free(avg);
}

int main(void)
{
    const size_t ns[] = {1, 2, 3, 7, 64, 1000, 4097};
    for (size_t a = 0; a < sizeof ns / sizeof ns[0]; ++a) {
        size_t n = ns[a];
        const size_t ks[] = {0, 1, n / 2, n > 1 ? n - 1 : 1, n};
        for (size_t c = 0; c < 5; ++c) if (ks[c] <= n) selection(n, ks[c]);
    }
    const size_t lens[] = {1, 2, 3, 4, 5, 17, 130, 1025};
    for (size_t a = 0; a < sizeof lens / sizeof lens[0]; ++a) {
        autoencoder(lens[a], 8, 4, 0);
        autoencoder(lens[a], 3, 5, 1);
    }
    float *x = vec(3 * 100), *out = vec(100);
    oracle_average(x, 3, 100, 1.0f / 3.0f, out);
    fold(out, 100);
    free(x); free(out);
    printf("checksum %.6f\n", checksum);
    return 0;
}
