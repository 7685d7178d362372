// Autoencoder layers (Sec. IV-C, Tables I and II: 1-D convolutions / transposed convolutions,
// kernel size 1 or 3, stride 1 or 2, padding (ksize-1)/2) and the scatter/average step
// (Sec. V-B), for gfx950.  Generic per-layer kernels: one thread computes COT output channels
// at one output position; weights are wave-uniform and come through the scalar cache; the input
// channels are taken in groups of G whose loads are all issued before the group's multiply-adds.
#include "lgc_internal.h"

namespace lgc {

__device__ __forceinline__ float leaky(float x, float slope) { return x > 0.f ? x : slope * x; }

// out[b][co][p] = bias[co] + sum_ci sum_t w[co][ci][t] * in[b][ci][p*stride - pad + t]
template <int COT, int KS, int G>
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
    // input channels in groups of G: all loads of a group are issued before its multiply-adds
    // (the order of the additions per output stays ci ascending, tap ascending)
    for (int ci0 = 0; ci0 < c_in; ci0 += G) {
        float x[G][KS];
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int t = 0; t < KS; ++t) {
                const long long q = q0 + t;
                x[g][t] = (ci0 + g < c_in && q >= 0 && q < (long long)l_in) ? in[(size_t)(ci0 + g) * l_in + q] : 0.f;
            }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (ci0 + g < c_in) {
#pragma unroll
                for (int c = 0; c < COT; ++c) {
                    if (co0 + c < c_out) {
#pragma unroll
                        for (int t = 0; t < KS; ++t)
                            acc[c] = fmaf(w[((size_t)(co0 + c) * c_in + ci0 + g) * KS + t], x[g][t], acc[c]);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int c = 0; c < COT; ++c)
        if (co0 + c < c_out) out[(size_t)(co0 + c) * l_out + p] = act ? leaky(acc[c], slope) : acc[c];
}

// out[b][co][q] = bias[co] + sum_ci sum_{(p,t): p*stride - pad + t = q} w[ci][co][t] * in[b][ci][p]
// With `extra` (decoder with the innovation component, Sec. IV-C): the last of the c_in input
// channels is extra[b][:], the others are in[b][0 .. c_in-2][:].
template <int COT, int KS, int G>
__global__ __launch_bounds__(256) void k_conv_transpose1d(const float *__restrict__ in, float *__restrict__ out,
                                                          const float *__restrict__ w,
                                                          const float *__restrict__ bias, int c_in, int c_out,
                                                          int stride, uint32_t l_in, uint32_t l_out, int act,
                                                          float slope, const float *__restrict__ extra) {
    const uint32_t q = blockIdx.x * 256 + threadIdx.x;
    if (q >= l_out) return;
    const int co0 = blockIdx.y * COT;
    const int b = blockIdx.z;
    constexpr int PAD = (KS - 1) / 2;
    const int c_main = extra ? c_in - 1 : c_in;
    in += (size_t)b * c_main * l_in;
    if (extra) extra += (size_t)b * l_in;
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
    for (int ci0 = 0; ci0 < c_in; ci0 += G) {
        float x[G][KS];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int ci = ci0 + g;
            const float *row = ci < c_main ? in + (size_t)ci * l_in : extra;
#pragma unroll
            for (int t = 0; t < KS; ++t) x[g][t] = (ci < c_in && hit[t]) ? row[src[t]] : 0.f;
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (ci0 + g < c_in) {
#pragma unroll
                for (int c = 0; c < COT; ++c) {
                    if (co0 + c < c_out) {
#pragma unroll
                        for (int t = 0; t < KS; ++t)
                            acc[c] = fmaf(w[((size_t)(ci0 + g) * c_out + co0 + c) * KS + t], x[g][t], acc[c]);
                    }
                }
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
#define LGC_CONV(KS, G) hipLaunchKernelGGL((k_conv1d<kCot, KS, G>), grid, dim3(256), 0, st, in, out, l.w, l.b, l.c_in, \
                                           l.c_out, l.stride, l_in, l_out, (int)act, slope)
    if (l.ksize == 3) { if (l.c_in >= 16) LGC_CONV(3, 16); else if (l.c_in >= 4) LGC_CONV(3, 4); else LGC_CONV(3, 1); }
    else              { if (l.c_in >= 16) LGC_CONV(1, 16); else if (l.c_in >= 4) LGC_CONV(1, 4); else LGC_CONV(1, 1); }
#undef LGC_CONV
}

void launch_conv_transpose1d(const float *in, float *out, const LayerDev &l, uint32_t l_in, uint32_t l_out,
                             int batch, bool act, float slope, hipStream_t st, const float *extra) {
    if (l_out == 0) return;
    dim3 grid((l_out + 255) / 256, (l.c_out + kCot - 1) / kCot, batch);
#define LGC_CONVT(KS, G) hipLaunchKernelGGL((k_conv_transpose1d<kCot, KS, G>), grid, dim3(256), 0, st, in, out, l.w, l.b, \
                                            l.c_in, l.c_out, l.stride, l_in, l_out, (int)act, slope, extra)
    if (l.ksize == 3) { if (l.c_in >= 16) LGC_CONVT(3, 16); else if (l.c_in >= 4) LGC_CONVT(3, 4); else LGC_CONVT(3, 1); }
    else              { if (l.c_in >= 16) LGC_CONVT(1, 16); else if (l.c_in >= 4) LGC_CONVT(1, 4); else LGC_CONVT(1, 1); }
#undef LGC_CONVT
}

// ---- two-layer stacks in one launch ------------------------------------------------------------
// The benchmark autoencoders (1 -> C1 -> C2, both layers kernel 3 / stride 2) are latency-bound
// as separate launches; here one thread produces one latent position (encoder) or four output
// positions (decoder) and recomputes the hidden positions it needs in registers (1.5x the hidden
// layer's arithmetic, no intermediate tensor).  The order of the multiply-adds per output is the
// one of the per-layer kernels above.

// z[b][co][p] = b2[co] + sum_c sum_t w2[co][c][t] * h[c][2p-1+t],
// h[c][s] = act(b1[c] + sum_t w1[c][0][t] * x[b][2s-1+t]); taps outside [0, L) contribute 0.
template <int C1, int C2>
__global__ __launch_bounds__(256) void k_encoder2(const float *__restrict__ x, float *__restrict__ z,
                                                  const float *__restrict__ w1, const float *__restrict__ b1,
                                                  const float *__restrict__ w2, const float *__restrict__ b2,
                                                  uint32_t l0, uint32_t l1, uint32_t l2, float slope) {
    const uint32_t p = blockIdx.x * 256 + threadIdx.x;
    if (p >= l2) return;
    x += (size_t)blockIdx.y * l0;
    z += (size_t)blockIdx.y * C2 * l2;
    float xv[7];   // x[4p-3 .. 4p+3]
#pragma unroll
    for (int i = 0; i < 7; ++i) {
        const long long q = 4ll * p - 3 + i;
        xv[i] = (q >= 0 && q < (long long)l0) ? x[q] : 0.f;
    }
    bool ok[3];    // hidden positions 2p-1, 2p, 2p+1 that exist
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        const long long hp = 2ll * p - 1 + s;
        ok[s] = hp >= 0 && hp < (long long)l1;
    }
    float acc[C2];
#pragma unroll
    for (int co = 0; co < C2; ++co) acc[co] = b2[co];
#pragma unroll
    for (int c = 0; c < C1; ++c) {
        float h[3];
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            float a = b1[c];
#pragma unroll
            for (int t = 0; t < 3; ++t) a = fmaf(w1[c * 3 + t], xv[2 * s + t], a);
            h[s] = ok[s] ? leaky(a, slope) : 0.f;
        }
#pragma unroll
        for (int co = 0; co < C2; ++co)
#pragma unroll
            for (int t = 0; t < 3; ++t) acc[co] = fmaf(w2[(co * C1 + c) * 3 + t], h[t], acc[co]);
    }
#pragma unroll
    for (int co = 0; co < C2; ++co) z[(size_t)co * l2 + p] = acc[co];
}

// y[b][q] = b4 + sum_c sum_{(s,t): 2s-1+t = q} w4[c][0][t] * h[c][s],
// h[c][s] = act(b3[c] + sum_cz sum_{(r,t): 2r-1+t = s} w3[cz][c][t] * z[b][cz][r]).
// Thread r4 writes y[4 r4 .. 4 r4 + 3]; these use h at 2 r4, 2 r4 + 1, 2 r4 + 2 and z at r4, r4 + 1.
template <int CZ, int CH>
__global__ __launch_bounds__(256) void k_decoder2(const float *__restrict__ z, float *__restrict__ y,
                                                  const float *__restrict__ w3, const float *__restrict__ b3,
                                                  const float *__restrict__ w4, const float *__restrict__ b4,
                                                  uint32_t l2, uint32_t l1, uint32_t l0, float slope) {
    const uint32_t r = blockIdx.x * 256 + threadIdx.x;
    if (4ull * r >= l0) return;
    z += (size_t)blockIdx.y * CZ * l2;
    y += (size_t)blockIdx.y * l0;
    const bool z0 = r < l2, z1 = r + 1 < l2;
    float za[CZ], zb[CZ];
#pragma unroll
    for (int cz = 0; cz < CZ; ++cz) {
        za[cz] = z0 ? z[(size_t)cz * l2 + r] : 0.f;
        zb[cz] = z1 ? z[(size_t)cz * l2 + r + 1] : 0.f;
    }
    const uint32_t s0 = 2 * r;
    const bool h0 = s0 < l1, h1 = s0 + 1 < l1, h2 = s0 + 2 < l1;
    const float bias = b4[0];
    float y0 = bias, y1 = bias, y2 = bias, y3 = bias;
    // two hidden channels per round: unrolled over all of them, the weights (wave-uniform, in scalar
    // registers) do not fit and spill into vector lanes, several reads of a lane for every multiply-add
#pragma unroll 2
    for (int c = 0; c < CH; ++c) {
        // hidden position 2r (even): tap 1 from z[r]; 2r+1 (odd): tap 0 from z[r+1], tap 2 from z[r];
        // 2r+2 (even): tap 1 from z[r+1].  Taps that do not reach a position add nothing.
        float a0 = b3[c], a1 = b3[c], a2 = b3[c];
#pragma unroll
        for (int cz = 0; cz < CZ; ++cz) {
            const float t0 = w3[(cz * CH + c) * 3 + 0], t1 = w3[(cz * CH + c) * 3 + 1], t2 = w3[(cz * CH + c) * 3 + 2];
            a0 = fmaf(t1, za[cz], a0);
            a1 = fmaf(t0, zb[cz], a1);
            a1 = fmaf(t2, za[cz], a1);
            a2 = fmaf(t1, zb[cz], a2);
        }
        const float g0 = h0 ? leaky(a0, slope) : 0.f;
        const float g1 = h1 ? leaky(a1, slope) : 0.f;
        const float g2 = h2 ? leaky(a2, slope) : 0.f;
        const float u0 = w4[c * 3 + 0], u1 = w4[c * 3 + 1], u2 = w4[c * 3 + 2];
        y0 = fmaf(u1, g0, y0);                       // q = 4r   : tap 1 from h[2r]
        y1 = fmaf(u0, g1, y1);                       // q = 4r+1 : tap 0 from h[2r+1], tap 2 from h[2r]
        y1 = fmaf(u2, g0, y1);
        y2 = fmaf(u1, g1, y2);                       // q = 4r+2 : tap 1 from h[2r+1]
        y3 = fmaf(u0, g2, y3);                       // q = 4r+3 : tap 0 from h[2r+2], tap 2 from h[2r+1]
        y3 = fmaf(u2, g1, y3);
    }
    const uint64_t q = 4ull * r;
    y[q] = y0;
    if (q + 1 < l0) y[q + 1] = y1;
    if (q + 2 < l0) y[q + 2] = y2;
    if (q + 3 < l0) y[q + 3] = y3;
}

// The parameter-server decoder at the benchmark's shape in one launch (Sec. IV-C, Sec. V-B): two kernel-3 /
// stride-2 transposed layers CZ -> CH -> CM channels as in k_decoder2, then the kernel-1 layer that takes the CM
// channels and the innovation component as one more channel:
//   y[b][q] = b5 + sum_cm w5[cm] * act(m[cm][q]) + w5[CM] * innov[b][q],
//   m[cm][q] = b4[cm] + sum_c sum_{(s,t): 2s-1+t = q} w4[c][cm][t] * h[c][s],   h as in k_decoder2.
// Thread r4 writes y[4 r4 .. 4 r4 + 3].
template <int CZ, int CH, int CM>
__global__ __launch_bounds__(256) void k_decoder3i(const float *__restrict__ z, const float *__restrict__ innov,
                                                   float *__restrict__ y, const float *__restrict__ w3,
                                                   const float *__restrict__ b3, const float *__restrict__ w4,
                                                   const float *__restrict__ b4, const float *__restrict__ w5,
                                                   const float *__restrict__ b5, uint32_t l2, uint32_t l1, uint32_t l0,
                                                   float slope) {
    const uint32_t r = blockIdx.x * 256 + threadIdx.x;
    if (4ull * r >= l0) return;
    z += (size_t)blockIdx.y * CZ * l2;
    y += (size_t)blockIdx.y * l0;
    innov += (size_t)blockIdx.y * l0;
    const uint64_t q = 4ull * r;
    float in[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) in[j] = q + j < l0 ? innov[q + j] : 0.f;
    const bool z0 = r < l2, z1 = r + 1 < l2;
    float za[CZ], zb[CZ];
#pragma unroll
    for (int cz = 0; cz < CZ; ++cz) {
        za[cz] = z0 ? z[(size_t)cz * l2 + r] : 0.f;
        zb[cz] = z1 ? z[(size_t)cz * l2 + r + 1] : 0.f;
    }
    const uint32_t s0 = 2 * r;
    const bool h0 = s0 < l1, h1 = s0 + 1 < l1, h2 = s0 + 2 < l1;
    float m[CM][4];
#pragma unroll
    for (int cm = 0; cm < CM; ++cm) m[cm][0] = m[cm][1] = m[cm][2] = m[cm][3] = b4[cm];
    // one hidden channel per round: the round's 3 CZ + 3 CM wave-uniform weights fit the scalar registers
#pragma unroll 1
    for (int c = 0; c < CH; ++c) {
        float a0 = b3[c], a1 = b3[c], a2 = b3[c];
#pragma unroll
        for (int cz = 0; cz < CZ; ++cz) {
            const float t0 = w3[(cz * CH + c) * 3 + 0], t1 = w3[(cz * CH + c) * 3 + 1], t2 = w3[(cz * CH + c) * 3 + 2];
            a0 = fmaf(t1, za[cz], a0);
            a1 = fmaf(t0, zb[cz], a1);
            a1 = fmaf(t2, za[cz], a1);
            a2 = fmaf(t1, zb[cz], a2);
        }
        const float g0 = h0 ? leaky(a0, slope) : 0.f;
        const float g1 = h1 ? leaky(a1, slope) : 0.f;
        const float g2 = h2 ? leaky(a2, slope) : 0.f;
#pragma unroll
        for (int cm = 0; cm < CM; ++cm) {
            const float u0 = w4[(c * CM + cm) * 3 + 0], u1 = w4[(c * CM + cm) * 3 + 1], u2 = w4[(c * CM + cm) * 3 + 2];
            m[cm][0] = fmaf(u1, g0, m[cm][0]);
            m[cm][1] = fmaf(u0, g1, m[cm][1]);
            m[cm][1] = fmaf(u2, g0, m[cm][1]);
            m[cm][2] = fmaf(u1, g1, m[cm][2]);
            m[cm][3] = fmaf(u0, g2, m[cm][3]);
            m[cm][3] = fmaf(u2, g1, m[cm][3]);
        }
    }
    float out[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float a = b5[0];
#pragma unroll
        for (int cm = 0; cm < CM; ++cm) a = fmaf(w5[cm], leaky(m[cm][j], slope), a);
        out[j] = fmaf(w5[CM], in[j], a);
    }
    y[q] = out[0];
    if (q + 1 < l0) y[q + 1] = out[1];
    if (q + 2 < l0) y[q + 2] = out[2];
    if (q + 3 < l0) y[q + 3] = out[3];
}

static bool two_layer_shape(const LayerDev &a, const LayerDev &b) {
    return a.ksize == 3 && a.stride == 2 && b.ksize == 3 && b.stride == 2;
}

bool launch_encoder2(const float *x, float *z, const LayerDev &a, const LayerDev &b, uint32_t l0, uint32_t l1,
                     uint32_t l2, int batch, float slope, hipStream_t st) {
    if (!two_layer_shape(a, b) || a.c_in != 1 || a.c_out != b.c_in) return false;
    if (l2 == 0) return true;
    dim3 grid((l2 + 255) / 256, batch);
    if (a.c_out == 8 && b.c_out == 4)
        hipLaunchKernelGGL((k_encoder2<8, 4>), grid, dim3(256), 0, st, x, z, a.w, a.b, b.w, b.b, l0, l1, l2, slope);
    else if (a.c_out == 16 && b.c_out == 8)
        hipLaunchKernelGGL((k_encoder2<16, 8>), grid, dim3(256), 0, st, x, z, a.w, a.b, b.w, b.b, l0, l1, l2, slope);
    else
        return false;
    return true;
}

bool launch_decoder2(const float *z, float *y, const LayerDev &a, const LayerDev &b, uint32_t l2, uint32_t l1,
                     uint32_t l0, int batch, float slope, hipStream_t st) {
    if (!two_layer_shape(a, b) || b.c_out != 1 || a.c_out != b.c_in) return false;
    if (l0 == 0) return true;
    dim3 grid(((l0 + 3) / 4 + 255) / 256, batch);
    if (a.c_in == 4 && a.c_out == 8)
        hipLaunchKernelGGL((k_decoder2<4, 8>), grid, dim3(256), 0, st, z, y, a.w, a.b, b.w, b.b, l2, l1, l0, slope);
    else if (a.c_in == 8 && a.c_out == 16)
        hipLaunchKernelGGL((k_decoder2<8, 16>), grid, dim3(256), 0, st, z, y, a.w, a.b, b.w, b.b, l2, l1, l0, slope);
    else
        return false;
    return true;
}

// a, b: the two transposed layers; c: the kernel-1 layer over b's channels and the innovation component
bool launch_decoder3i(const float *z, const float *innov, float *y, const LayerDev &a, const LayerDev &b,
                      const LayerDev &c, uint32_t l2, uint32_t l1, uint32_t l0, int batch, float slope, hipStream_t st) {
    if (!two_layer_shape(a, b) || a.c_out != b.c_in || c.ksize != 1 || c.stride != 1 || c.c_out != 1 ||
        c.c_in != b.c_out + 1)
        return false;
    if (l0 == 0) return true;
    dim3 grid(((l0 + 3) / 4 + 255) / 256, batch);
    if (a.c_in == 4 && a.c_out == 8 && b.c_out == 4)
        hipLaunchKernelGGL((k_decoder3i<4, 8, 4>), grid, dim3(256), 0, st, z, innov, y, a.w, a.b, b.w, b.b, c.w, c.b, l2, l1,
                           l0, slope);
    else if (a.c_in == 8 && a.c_out == 16 && b.c_out == 8)
        hipLaunchKernelGGL((k_decoder3i<8, 16, 8>), grid, dim3(256), 0, st, z, innov, y, a.w, a.b, b.w, b.b, c.w, c.b, l2,
                           l1, l0, slope);
    else
        return false;
    return true;
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

// All nodes in one launch, same result as one k_scatter per node in node order.  Needs every
// node's positions in ascending order.  The thread of (node b, entry j) looks its position up in
// every other node's list; the thread of the first node that holds the position owns it and adds
// the contributions of all holders in node order; the other holders' threads leave it alone.  No
// atomics, no waiting.  A look-up is a chain of dependent loads, so a block does it once for all
// of its 256 entries: 16 lanes per other list and bound find, by 16-way search (log16 k rounds of
// loads), the stretch of that list between the block's first and last position; the stretches are
// copied to LDS (they hold about as many entries as the block's own, the nodes' selections being
// alike) and every thread searches them there.  A stretch too long for LDS is searched in place.
constexpr int kScatterNodes = 8;
constexpr int kScatterWin = 512;

__global__ __launch_bounds__(256) void k_scatter_nodes(const float *__restrict__ vals,
                                                       const uint32_t *__restrict__ idx, uint32_t k, int batch,
                                                       float scale, float *__restrict__ dense, uint32_t n,
                                                       Stats *stats) {
    __shared__ uint32_t win[kScatterNodes][kScatterWin];
    __shared__ uint32_t w_lo[kScatterNodes], w_hi[kScatterNodes];
    const int tid = threadIdx.x, b = blockIdx.y;
    const uint32_t j0 = blockIdx.x * 256, j = j0 + tid;   // j0 < k: the grid has ceil(k / 256) blocks
    const uint32_t *own_list = idx + (size_t)b * k;
    const bool mine = j < k;
    const uint32_t i = mine ? own_list[j] : 0u;
    const uint32_t before = (mine && j > 0) ? own_list[j - 1] : 0u;
    const uint32_t first = own_list[j0], last = own_list[k - j0 > 256 ? j0 + 255 : k - 1];
    // loaded now, used at the end: only the owner of a position ever writes it, and it reads first
    const float base = (mine && i < n) ? dense[i] : 0.f, own = mine ? vals[(size_t)b * k + j] : 0.f;
    {
        // search g = tid / 16: list g / 2, its first entry >= first (even g) or > last (odd g)
        const int g = tid >> 4, t = tid & 15, o = g >> 1;
        const bool active = o < batch && o != b;
        const uint32_t target = (g & 1) ? last + 1 : first;
        const uint32_t *list = idx + (size_t)(active ? o : b) * k;
        // everything below lo is < target, everything from hi on is >= target
        uint32_t lo = 0, hi = active ? k : 0u;
        while (__any(lo < hi)) {   // all lanes of the wavefront take part in the ballot
            const uint32_t len = hi - lo, step = (len + 15) / 16;
            const uint32_t p = lo + (uint32_t)t * step;
            const bool probe = lo < hi && p < hi;
            const uint32_t x = probe ? list[p] : 0xffffffffu;
            const unsigned long long m = __ballot(probe && x < target);
            const uint32_t c = (uint32_t)__popc((uint32_t)(m >> (tid & 48)) & 0xffffu);   // probes of this search below the target
            if (lo < hi) {
                const uint32_t probes = (len + step - 1) / step;
                const uint32_t nlo = c ? lo + (c - 1) * step + 1 : lo;
                hi = c < probes ? lo + c * step : hi;
                lo = nlo;
            }
        }
        if (t == 0 && active) { if (g & 1) w_hi[o] = lo; else w_lo[o] = lo; }
    }
    __syncthreads();
    for (int o = 0; o < batch; ++o) {
        if (o == b) continue;   // uniform
        const uint32_t lo = w_lo[o], hi = w_hi[o], len = hi > lo ? hi - lo : 0u;
        if (len <= (uint32_t)kScatterWin)
            for (uint32_t t = tid; t < len; t += 256) win[o][t] = idx[(size_t)o * k + lo + t];
    }
    __syncthreads();
    if (!mine) return;
    if (j > 0 && before >= i) atomicAdd(&stats->errors, 1u);   // not ascending
    if (i >= n) { atomicAdd(&stats->errors, 1u); return; }
    // per other node: is i in its list, and where
    bool held[kScatterNodes];
    uint32_t at[kScatterNodes];
#pragma unroll
    for (int o = 0; o < kScatterNodes; ++o) {
        held[o] = false; at[o] = 0;
        if (o < batch && o != b) {
            const uint32_t wl = w_lo[o], wh = w_hi[o], len = wh > wl ? wh - wl : 0u;
            uint32_t lo = 0, hi = len;   // first entry of the stretch that is >= i
            if (len <= (uint32_t)kScatterWin) {
                while (lo < hi) {
                    const uint32_t mid = (lo + hi) >> 1;
                    if (win[o][mid] < i) lo = mid + 1; else hi = mid;
                }
                held[o] = lo < len && win[o][lo] == i;
            } else {
                const uint32_t *list = idx + (size_t)o * k + wl;
                while (lo < hi) {
                    const uint32_t mid = (lo + hi) >> 1;
                    if (list[mid] < i) lo = mid + 1; else hi = mid;
                }
                held[o] = lo < len && list[lo] == i;
            }
            at[o] = wl + lo;
        }
    }
    bool owner = true;
#pragma unroll
    for (int o = 0; o < kScatterNodes; ++o) owner = owner && !(o < b && held[o]);
    if (!owner) return;
    float acc = __fadd_rn(base, __fmul_rn(scale, own));
#pragma unroll
    for (int o = 0; o < kScatterNodes; ++o)
        if (o > b && held[o]) acc = __fadd_rn(acc, __fmul_rn(scale, vals[(size_t)o * k + at[o]]));
    dense[i] = acc;
}

bool launch_scatter_nodes(const float *vals, const uint32_t *idx, uint32_t k, int batch, float scale, float *dense,
                          uint32_t n, Stats *stats, hipStream_t st) {
    if (batch > kScatterNodes) return false;
    if (k == 0) return true;
    hipLaunchKernelGGL(k_scatter_nodes, dim3((k + 255) / 256, batch), dim3(256), 0, st, vals, idx, k, batch, scale,
                       dense, n, stats);
    return true;
}

// ---- ring-allreduce pattern ---------------------------------------------------------------------

// out[b][j] = v[b][idx[j]]; v[b][idx[j]] = u[b][idx[j]] = +0.  The positions are shared by the nodes
// and distinct, so every element is touched by one thread only.
__global__ __launch_bounds__(256) void k_gather_at(float *__restrict__ v, float *__restrict__ u, uint64_t stride,
                                                   uint32_t n, const uint32_t *__restrict__ idx, uint32_t k,
                                                   float *__restrict__ out, Stats *stats) {
    const uint32_t j = blockIdx.x * 256 + threadIdx.x;
    if (j >= k) return;
    const size_t off = (size_t)blockIdx.y * stride;
    const uint32_t i = idx[j];
    float *o = out + (size_t)blockIdx.y * k + j;
    if (i >= n) { *o = 0.f; atomicAdd(&stats->errors, 1u); return; }
    *o = v[off + i];
    v[off + i] = 0.f;
    if (u) u[off + i] = 0.f;
}

void launch_gather_at(float *v, float *u, uint64_t stride, uint32_t n, int batch, const uint32_t *idx, uint32_t k,
                      float *out, Stats *stats, hipStream_t st) {
    if (k == 0) return;
    hipLaunchKernelGGL(k_gather_at, dim3((k + 255) / 256, batch), dim3(256), 0, st, v, u, stride, n, idx, k, out, stats);
}

// out[i] = (..((0 + scale*x[0][i]) + scale*x[1][i]) + ..), products and sums rounded one by one
__global__ __launch_bounds__(256) void k_average(const float *__restrict__ x, uint32_t len, int batch, float scale,
                                                 float *__restrict__ out) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i >= len) return;
    float acc = 0.f;
    for (int b = 0; b < batch; ++b) acc = __fadd_rn(acc, __fmul_rn(scale, x[(size_t)b * len + i]));
    out[i] = acc;
}

void launch_average(const float *x, uint32_t len, int batch, float scale, float *out, hipStream_t st) {
    if (len == 0) return;
    hipLaunchKernelGGL(k_average, dim3((len + 255) / 256), dim3(256), 0, st, x, len, batch, scale, out);
}

}  // namespace lgc
