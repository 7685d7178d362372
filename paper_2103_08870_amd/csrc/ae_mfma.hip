// Deep autoencoder layers on the matrix cores (gfx950, wave64, v_mfma_f32_32x32x2_f32).
//
// The paper-size autoencoder (Sec. IV-C, Table I: 1-64-128-256-64-4; Table II: 4-4-32-64-128-32-1)
// has layers that are dense contractions: a kernel-3 / stride-2 convolution from c_in to c_out
// channels is, per output position, a product of a [c_out] x [3 c_in] weight matrix with the
// 3 c_in inputs under the window (contraction depth 192 .. 768), and a kernel-3 / stride-2
// transposed convolution is two such products (even and odd output positions, depth c_in and
// 2 c_in).  These run here as implicit GEMMs in fp32 on the MFMA units (fp32 in, fp32 accumulate:
// the 1e-4 parity bar against the fp64 oracle rules out bf16 / fp16 inputs).  The first and last
// layers of each stack (1 or 4 channels on one side) stay on the per-layer vector kernels.
//
// Operand layout of v_mfma_f32_32x32x2_f32 (checked on the device): lane l supplies
// A[i = l % 32][k = l / 32] and B[k = l / 32][j = l % 32]; of the 16 results of lane l, number r
// is C[i = 8 (r / 4) + 4 (l / 32) + r % 4][j = l % 32].  Here i is the output channel, j the
// position and k the contraction index, so each result register of a half-wavefront is 32
// consecutive positions of one channel: coalesced stores.

#include "lgc_internal.h"

namespace lgc {

typedef float acc16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float leaky_m(float x, float slope) { return x > 0.f ? x : slope * x; }

// ---- weights in contraction-major order -----------------------------------------------------------
// conv:  w [c_out][c_in][3]  ->  wt[(ci*3 + t)][co]
// convT: w [c_in][c_out][3]  ->  wt[(t*c_in + ci)][co]     (tap-major: the kernel takes one tap at a time)
__global__ void k_weights_contraction_major(const float *__restrict__ w, float *__restrict__ wt, int c_in, int c_out,
                                            int transposed) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= c_in * c_out * 3) return;
    if (!transposed) {
        const int t = e % 3, ci = (e / 3) % c_in, co = e / (3 * c_in);
        wt[(size_t)(ci * 3 + t) * c_out + co] = w[e];
    } else {
        const int t = e % 3, co = (e / 3) % c_out, ci = e / (3 * c_out);
        wt[(size_t)(t * c_in + ci) * c_out + co] = w[e];
    }
}

void launch_weights_contraction_major(const float *w, float *wt, int c_in, int c_out, bool transposed, hipStream_t st) {
    const int total = c_in * c_out * 3;
    hipLaunchKernelGGL(k_weights_contraction_major, dim3((total + 255) / 256), dim3(256), 0, st, w, wt, c_in, c_out,
                       (int)transposed);
}

// ---- convolution, kernel 3, stride 2, padding 1 -----------------------------------------------------
// out[b][co][p] = bias[co] + sum_ci sum_t w[co][ci][t] * in[b][ci][2p - 1 + t]
// Block: 256 threads, 64 output channels x 64 positions; wavefront (wm, wn) of 2 x 2 owns one 32 x 32
// MFMA tile.  Small tiles on purpose: the layers are short (a few thousand positions per node), and
// a few hundred blocks are needed to keep 256 compute units evenly busy.  The contraction runs over
// chunks of 16 input channels staged in LDS: inputs split into odd and even positions (so that every
// tap is a unit-stride read), weights as [48][64].  The next chunk is fetched into registers while
// the current one is multiplied.  c_in % 16 == 0 and c_out % 64 == 0.
constexpr int kCiChunk = 16;
constexpr int kPosTile = 64;
constexpr int kRowPad = 136;    // per input channel: odd positions [0..64], even positions [68..131]
constexpr int kEvenOff = 68;
constexpr int kXPerRow = 2 * kPosTile + 1;                           // 129 inputs per channel and tile
constexpr int kXRegs = (kCiChunk * kXPerRow + 255) / 256;            // 9
constexpr int kWRegs = kCiChunk * 3 * 64 / 256;                      // 12

// TAIL: a following kernel-1 / stride-1 layer from these 64 channels (c_out == 64: one block holds all of
// them for its positions) to tail_c <= 4 channels is applied to the activated tile before anything is
// stored; `out` is then that layer's output [b][tail_c][l_out] (Table I: conv4 256->64 and conv5 64->4).
template <bool TAIL>
__global__ __launch_bounds__(256) void k_conv3s2_mfma(const float *__restrict__ in, float *__restrict__ out,
                                                      const float *__restrict__ wt, const float *__restrict__ bias,
                                                      int c_in, int c_out, uint32_t l_in, uint32_t l_out, int act,
                                                      float slope, const float *__restrict__ tail_w /*[tail_c][64]*/,
                                                      const float *__restrict__ tail_b, int tail_c, int tail_act) {
    // the last slot of the input buffer takes the stores of staging slots that hold nothing
    // (a second pair of buffers, with one barrier per chunk, was tried: it costs a resident block per
    // compute unit and gains nothing)
    __shared__ float xs[kCiChunk * kRowPad + 1];
    __shared__ float ws[kCiChunk * 3 * 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, half = lane >> 5, col = lane & 31;
    const uint32_t p0 = blockIdx.x * kPosTile;
    const int co0 = blockIdx.y * 64;
    in += (size_t)blockIdx.z * c_in * l_in;
    out += (size_t)blockIdx.z * (TAIL ? tail_c : c_out) * l_out;

    // staging slots of this thread, fixed for the whole contraction: input slot e = tid + 256 i is
    // (channel e / 129, r = e % 129) with r <= 64: odd[r] = in[2 (p0 + r) - 1] and
    // r > 64: even[r - 65] = in[2 (p0 + r - 65)].  gx = offset inside a chunk of the input (0 where
    // there is nothing to load: the load is made anyway and its result dropped, no branches),
    // lx = LDS slot, bit i of `live` = the slot holds a real input
    // (the LDS slots and the weights' offsets are recomputed where they are used: registers are
    // what limits the number of resident wavefronts here)
    uint32_t gx[kXRegs], live = 0;
#pragma unroll
    for (int i = 0; i < kXRegs; ++i) {
        const int e = tid + 256 * i;
        const int ci = e / kXPerRow, r = e % kXPerRow;
        const long long q = r <= kPosTile ? 2ll * (p0 + r) - 1 : 2ll * (p0 + (r - kPosTile - 1));
        const bool ok = e < kCiChunk * kXPerRow && q >= 0 && q < (long long)l_in;
        gx[i] = ok ? (uint32_t)(ci * (size_t)l_in + q) : 0u;
        live |= (uint32_t)ok << i;
    }
    const uint32_t gw0 = (uint32_t)((tid >> 6) * c_out + co0 + (tid & 63));   // slot e = tid + 256 i: row (tid >> 6) + 4 i
    float xr[kXRegs], wr[kWRegs];
    auto fetch = [&](int c0) {
        const float *xin = in + (size_t)c0 * l_in;
        const float *win = wt + (size_t)c0 * 3 * c_out + gw0;
#pragma unroll
        for (int i = 0; i < kXRegs; ++i) xr[i] = xin[gx[i]];
#pragma unroll
        for (int i = 0; i < kWRegs; ++i) wr[i] = win[(size_t)(4 * i) * c_out];
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < kXRegs; ++i) {
            const int e = tid + 256 * i;
            const int ci = e / kXPerRow, r = e % kXPerRow;
            const int slot = e < kCiChunk * kXPerRow ? ci * kRowPad + (r <= kPosTile ? r : kEvenOff + (r - kPosTile - 1))
                                                     : kCiChunk * kRowPad;
            xs[slot] = ((live >> i) & 1u) ? xr[i] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < kWRegs; ++i) ws[tid + 256 * i] = wr[i];
    };

    acc16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    fetch(0);
    for (int c0 = 0; c0 < c_in; c0 += kCiChunk) {
        __syncthreads();   // the previous chunk's readers are done
        stage();
        __syncthreads();
        if (c0 + kCiChunk < c_in) fetch(c0 + kCiChunk);   // in flight during the multiplications below
        // contraction index of step s: lanes 0..31 take channel s / 3 of the chunk's first eight, lanes
        // 32..63 the same of its last eight, tap s % 3: both halves read at the same constant offsets
        // from their own base, so the reads of two steps pair into one LDS instruction
        const float *xb = xs + half * (kCiChunk / 2) * kRowPad + wn * 32 + col;
        const float *wb = ws + half * (kCiChunk * 3 / 2) * 64 + wm * 32 + col;
#pragma unroll
        for (int s = 0; s < kCiChunk * 3 / 2; ++s) {
            const int off = (s / 3) * kRowPad + ((s % 3) == 1 ? kEvenOff : 0) + ((s % 3) == 2 ? 1 : 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wb[s * 64], xb[off], acc, 0, 0, 0);
        }
    }
    const uint32_t p = p0 + wn * 32 + col;
    if (!TAIL) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int co = co0 + wm * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
            if (p < l_out) {
                const float y = acc[r] + bias[co];
                out[(size_t)co * l_out + p] = act ? leaky_m(y, slope) : y;
            }
        }
        return;
    }
    // this lane's 16 channels of position p, activated; their weighted sums for the tail's channels;
    // then the other half-wavefront's 16 channels, and through LDS the other 32 channels (wm)
    float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int co = wm * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
        const float y0 = acc[r] + bias[co];
        const float y = act ? leaky_m(y0, slope) : y0;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (c < tail_c) part[c] = fmaf(tail_w[c * 64 + co], y, part[c]);
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) part[c] += __shfl_xor(part[c], 32, 64);
    __syncthreads();                        // everyone is done with the staging buffers
    float *red = xs;                        // [wm][c][64 positions]
    if (half == 0) {
#pragma unroll
        for (int c = 0; c < 4; ++c) red[(wm * 4 + c) * 64 + wn * 32 + col] = part[c];
    }
    __syncthreads();
    const int c = tid >> 6, pp = tid & 63;
    if (c < tail_c && p0 + pp < l_out) {
        const float z = tail_b[c] + red[c * 64 + pp] + red[(4 + c) * 64 + pp];
        out[(size_t)c * l_out + p0 + pp] = tail_act ? leaky_m(z, slope) : z;
    }
}

bool conv3s2_mfma_covers(const LayerDev &l, uint32_t l_in) {
    if (!l.wt || l.ksize != 3 || l.stride != 2 || l.c_in % kCiChunk != 0 || l.c_out % 64 != 0) return false;
    return (uint64_t)l_in * kCiChunk < (1ull << 32) && (uint64_t)l.c_in * 3 * l.c_out < (1ull << 32);   // 32-bit offsets inside a chunk
}

// tail (nullable): a kernel-1 / stride-1 layer from l.c_out == 64 to at most 4 channels, applied in the same
// launch; `out` is then the tail's output
bool launch_conv3s2_mfma(const float *in, float *out, const LayerDev &l, uint32_t l_in, uint32_t l_out, int batch,
                         bool act, float slope, hipStream_t st, const LayerDev *tail, bool tail_act) {
    if (!conv3s2_mfma_covers(l, l_in)) return false;
    if (tail && !(tail->ksize == 1 && tail->stride == 1 && tail->c_in == 64 && l.c_out == 64 && tail->c_out <= 4)) return false;
    if (l_out == 0) return true;
    dim3 grid((l_out + kPosTile - 1) / kPosTile, l.c_out / 64, batch);
    if (tail)
        hipLaunchKernelGGL(k_conv3s2_mfma<true>, grid, dim3(256), 0, st, in, out, l.wt, l.b, l.c_in, l.c_out, l_in, l_out,
                           (int)act, slope, tail->w, tail->b, tail->c_out, (int)tail_act);
    else
        hipLaunchKernelGGL(k_conv3s2_mfma<false>, grid, dim3(256), 0, st, in, out, l.wt, l.b, l.c_in, l.c_out, l_in, l_out,
                           (int)act, slope, nullptr, nullptr, 0, 0);
    return true;
}

// ---- transposed convolution, kernel 3, stride 2, padding 1 ------------------------------------------
// out[b][co][q] = bias[co] + sum_ci sum_{(p,t): 2p - 1 + t = q} w[ci][co][t] * in[b][ci][p]
//   even q = 2m:     sum_ci w[ci][co][1] in[ci][m]
//   odd  q = 2m + 1: sum_ci ( w[ci][co][0] in[ci][m+1] + w[ci][co][2] in[ci][m] )
// Block: 256 threads, 32 output channels x 128 input positions m (256 output positions); wavefront w
// owns the 32 channels x 32 positions m = 32 w .. 32 w + 31, with one accumulator tile for the even
// and one for the odd outputs.  Chunks of 16 input channels in LDS: inputs [16][129] (unit stride for
// both taps), weights [3][16][32] (tap-major); the next chunk is fetched into registers during the
// multiplications.  c_in % 16 == 0 and c_out % 32 == 0.
constexpr int kTPosTile = 128;
constexpr int kTRowPad = 132;
constexpr int kTXRegs = (kCiChunk * (kTPosTile + 1) + 255) / 256;    // 9
constexpr int kTWRegs = 3 * kCiChunk * 32 / 256;                      // 6

// TAIL: a following kernel-1 / stride-1 layer from these 32 channels (c_out == 32) to one channel is applied
// to the activated tiles before anything is stored; `out` is then [b][1][l_out] (Table II: deconv5 128->32
// and the last layer 32->1).
template <bool TAIL>
__global__ __launch_bounds__(256) void k_convt3s2_mfma(const float *__restrict__ in, float *__restrict__ out,
                                                       const float *__restrict__ wt, const float *__restrict__ bias,
                                                       int c_in, int c_out, uint32_t l_in, uint32_t l_out, int act,
                                                       float slope, const float *__restrict__ tail_w /*[32]*/,
                                                       const float *__restrict__ tail_b, int tail_act) {
    __shared__ float xs[kCiChunk * kTRowPad + 1];
    __shared__ float ws[3 * kCiChunk * 32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const uint32_t m0 = blockIdx.x * kTPosTile;
    const int co0 = blockIdx.y * 32;
    in += (size_t)blockIdx.z * c_in * l_in;
    out += (size_t)blockIdx.z * (TAIL ? 1 : c_out) * l_out;

    // staging slots of this thread, fixed for the whole contraction (see the convolution above)
    uint32_t gx[kTXRegs], gw[kTWRegs], live = 0;
    int lx[kTXRegs];
#pragma unroll
    for (int i = 0; i < kTXRegs; ++i) {
        const int e = tid + 256 * i;
        const int ci = e / (kTPosTile + 1), r = e % (kTPosTile + 1);
        const bool slot = e < kCiChunk * (kTPosTile + 1);
        const bool ok = slot && m0 + r < l_in;
        gx[i] = ok ? (uint32_t)(ci * (size_t)l_in + m0 + r) : 0u;
        live |= (uint32_t)ok << i;
        lx[i] = slot ? ci * kTRowPad + r : kCiChunk * kTRowPad;
    }
#pragma unroll
    for (int i = 0; i < kTWRegs; ++i) {
        const int e = tid + 256 * i;
        const int t = e / (kCiChunk * 32), ci = (e / 32) % kCiChunk, co = e & 31;
        gw[i] = (uint32_t)((t * c_in + ci) * c_out + co0 + co);
    }
    float xr[kTXRegs], wr[kTWRegs];
    auto fetch = [&](int c0) {
        const float *xin = in + (size_t)c0 * l_in;
        const float *win = wt + (size_t)c0 * c_out;
#pragma unroll
        for (int i = 0; i < kTXRegs; ++i) xr[i] = xin[gx[i]];
#pragma unroll
        for (int i = 0; i < kTWRegs; ++i) wr[i] = win[gw[i]];
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < kTXRegs; ++i) xs[lx[i]] = ((live >> i) & 1u) ? xr[i] : 0.f;
#pragma unroll
        for (int i = 0; i < kTWRegs; ++i) ws[tid + 256 * i] = wr[i];
    };

    acc16 even, odd;
#pragma unroll
    for (int r = 0; r < 16; ++r) { even[r] = 0.f; odd[r] = 0.f; }

    fetch(0);
    for (int c0 = 0; c0 < c_in; c0 += kCiChunk) {
        __syncthreads();
        stage();
        __syncthreads();
        if (c0 + kCiChunk < c_in) fetch(c0 + kCiChunk);
        // lanes 0..31 take the chunk's first eight input channels, lanes 32..63 its last eight
        const float *xb = xs + half * (kCiChunk / 2) * kTRowPad + wave * 32 + col;
        const float *wb = ws + half * (kCiChunk / 2) * 32 + col;
#pragma unroll
        for (int s = 0; s < kCiChunk / 2; ++s) {
            const float x0 = xb[s * kTRowPad];          // in[ci][m]
            const float x1 = xb[s * kTRowPad + 1];      // in[ci][m + 1]
            const float w0 = wb[(0 * kCiChunk + s) * 32];
            const float w1 = wb[(1 * kCiChunk + s) * 32];
            const float w2 = wb[(2 * kCiChunk + s) * 32];
            even = __builtin_amdgcn_mfma_f32_32x32x2f32(w1, x0, even, 0, 0, 0);
            odd = __builtin_amdgcn_mfma_f32_32x32x2f32(w0, x1, odd, 0, 0, 0);
            odd = __builtin_amdgcn_mfma_f32_32x32x2f32(w2, x0, odd, 0, 0, 0);
        }
    }
    const uint32_t m = m0 + wave * 32 + col;
    if (TAIL) {
        // weighted sums over this lane's 16 channels, then the other half-wavefront's 16
        float se = 0.f, so = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int co = (r >> 2) * 8 + half * 4 + (r & 3);
            const float bv = bias[co], wv = tail_w[co];
            const float ye = even[r] + bv, yo = odd[r] + bv;
            se = fmaf(wv, act ? leaky_m(ye, slope) : ye, se);
            so = fmaf(wv, act ? leaky_m(yo, slope) : yo, so);
        }
        se += __shfl_xor(se, 32, 64);
        so += __shfl_xor(so, 32, 64);
        const uint64_t q = 2ull * m + half;              // lanes 0..31 store the even, lanes 32..63 the odd output
        if (q < l_out) {
            const float z = tail_b[0] + (half ? so : se);
            out[q] = tail_act ? leaky_m(z, slope) : z;
        }
        return;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int co = co0 + (r >> 2) * 8 + half * 4 + (r & 3);
        const float bv = bias[co];
        const uint64_t q = 2ull * m;
        if (q < l_out) {
            const float y = even[r] + bv;
            out[(size_t)co * l_out + q] = act ? leaky_m(y, slope) : y;
        }
        if (q + 1 < l_out) {
            const float y = odd[r] + bv;
            out[(size_t)co * l_out + q + 1] = act ? leaky_m(y, slope) : y;
        }
    }
}

// tail (nullable): a kernel-1 / stride-1 layer from l.c_out == 32 channels to one, applied in the same launch
bool launch_convt3s2_mfma(const float *in, float *out, const LayerDev &l, uint32_t l_in, uint32_t l_out, int batch,
                          bool act, float slope, hipStream_t st, const LayerDev *tail, bool tail_act) {
    if (!l.wt || l.ksize != 3 || l.stride != 2 || l.c_in % kCiChunk != 0 || l.c_out % 32 != 0) return false;
    if ((uint64_t)l_in * kCiChunk >= (1ull << 32) || (uint64_t)l.c_in * 3 * l.c_out >= (1ull << 32)) return false;   // 32-bit offsets inside a chunk
    if (tail && !(tail->ksize == 1 && tail->stride == 1 && tail->c_in == 32 && l.c_out == 32 && tail->c_out == 1)) return false;
    if (l_out == 0) return true;
    // input positions that reach an output: m < ceil(l_out / 2) (and the odd tap of m = that - 1 reads m + 1)
    const uint32_t m_count = (l_out + 1) / 2;
    dim3 grid((m_count + kTPosTile - 1) / kTPosTile, l.c_out / 32, batch);
    if (tail)
        hipLaunchKernelGGL(k_convt3s2_mfma<true>, grid, dim3(256), 0, st, in, out, l.wt, l.b, l.c_in, l.c_out, l_in, l_out,
                           (int)act, slope, tail->w, tail->b, (int)tail_act);
    else
        hipLaunchKernelGGL(k_convt3s2_mfma<false>, grid, dim3(256), 0, st, in, out, l.wt, l.b, l.c_in, l.c_out, l_in, l_out,
                           (int)act, slope, nullptr, nullptr, 0);
    return true;
}

}  // namespace lgc
