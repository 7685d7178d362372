// Deep autoencoder layers on the matrix cores (gfx950, wave64, v_mfma_f32_32x32x2_f32).
//
// The paper-size autoencoder (Sec. IV-C, Table I: 1-64-128-256-64-4; Table II: 4-4-32-64-128-32-1)
// has layers that are dense contractions: a kernel-3 / stride-2 convolution from c_in to c_out
// channels is, per output position, a product of a [c_out] x [3 c_in] weight matrix with the
// 3 c_in inputs under the window (contraction depth 192 .. 768), and a kernel-3 / stride-2
// transposed convolution is two such products (even and odd output positions, depth c_in and
// 2 c_in).  These run here as implicit GEMMs in fp32 on the MFMA units (fp32 in, fp32 accumulate:
// the 1e-4 parity bar against the fp64 oracle rules out bf16 / fp16 inputs).  The narrow first
// layers of each stack (1 or 4 channels on one side) are evaluated inside the input staging of the
// deep layer after them, the kernel-1 layers that end the stacks in the epilogue of the deep layer
// before them.
//
// Operand layout of v_mfma_f32_32x32x2_f32 (checked on the device): lane l supplies
// A[i = l % 32][k = l / 32] and B[k = l / 32][j = l % 32]; of the 16 results of lane l, number r
// is C[i = 8 (r / 4) + 4 (l / 32) + r % 4][j = l % 32].  Here i is the output channel, j the
// position and k the contraction index, so each result register of a half-wavefront is 32
// consecutive positions of one channel: coalesced stores.

#include "lgc_internal.h"

namespace lgc {

typedef float acc16 __attribute__((ext_vector_type(16)));
typedef float f4v __attribute__((ext_vector_type(4)));

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
constexpr int kHeadMaxC = 256;                                        // most channels of a fused one-channel first layer
constexpr int kXRegs = (kCiChunk * kXPerRow + 255) / 256;            // 9
constexpr int kWRegs = kCiChunk * 3 * 64 / 256;                      // 12

// TAIL: a following kernel-1 / stride-1 layer from these 64 channels (c_out == 64: one block holds all of
// them for its positions) to tail_c <= 4 channels is applied to the activated tile before anything is
// stored; `out` is then that layer's output [b][tail_c][l_out] (Table I: conv4 256->64 and conv5 64->4).
// HEAD: the layer's input is not read but made on the fly from a preceding kernel-3 / stride-2 layer with ONE
// input channel (Table I: conv1 1->64 in front of conv2 64->128): `in` is then that layer's input
// [b][1][l_head], head_w [c_in][1][3] and head_b [c_in] its weights, and every staged input h[ci][q] =
// act(head_b[ci] + sum_t head_w[ci][t] x[2q - 1 + t]) comes from a 259-value stretch of x kept in LDS: no
// intermediate tensor, no launch for the first layer, no global loads of inputs in the contraction loop.
// SPLIT: the contraction is cut into `splits` equal runs of input channels, one block each (blockIdx.y =
// split * (c_out / 64) + channel block); a block then stores its raw partial sums (no bias, no non-linearity) to
// out[b][split][co][p], and k_splitk_finish adds them up.  For layers with too few output tiles to fill the
// device (Table I: conv4 256 -> 64 has 25 tiles per node).
template <bool TAIL, bool HEAD, bool SPLIT = false>
__global__ __launch_bounds__(256) void k_conv3s2_mfma(const float *__restrict__ in, float *__restrict__ out,
                                                      const float *__restrict__ wt, const float *__restrict__ bias,
                                                      int c_in, int c_out, uint32_t l_in, uint32_t l_out, int act,
                                                      float slope, const float *__restrict__ tail_w /*[tail_c][64]*/,
                                                      const float *__restrict__ tail_b, int tail_c, int tail_act,
                                                      const float *__restrict__ head_w, const float *__restrict__ head_b,
                                                      uint32_t l_head, int splits) {
    // the last slot of the input buffer takes the stores of staging slots that hold nothing
    // (a second pair of buffers, with one barrier per chunk, was tried: it costs a resident block per
    // compute unit and gains nothing)
    __shared__ float xs[kCiChunk * kRowPad + 1];
    __shared__ __align__(16) float ws[kCiChunk * 3 * 64];
    __shared__ float head_x[HEAD ? 4 * kPosTile + 4 : 1];   // x[4 p0 - 3 .. 4 p0 + 255], zeros outside [0, l_head)
    __shared__ float head_p[HEAD ? 4 * kHeadMaxC : 1];      // per channel: the three taps, then the bias
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, half = lane >> 5, col = lane & 31;
    const uint32_t p0 = blockIdx.x * kPosTile;
    const int co_blocks = c_out / 64;
    const int co0 = (SPLIT ? (int)blockIdx.y % co_blocks : (int)blockIdx.y) * 64;
    const int split = SPLIT ? (int)blockIdx.y / co_blocks : 0;
    const int c_per = SPLIT ? c_in / splits : c_in;          // a multiple of kCiChunk (the launcher sees to it)
    const int c_lo = split * c_per, c_hi = c_lo + c_per;
    in += (size_t)blockIdx.z * (HEAD ? (size_t)l_head : (size_t)c_in * l_in);
    out += SPLIT ? ((size_t)blockIdx.z * splits + split) * c_out * l_out
                 : (size_t)blockIdx.z * (TAIL ? tail_c : c_out) * l_out;
    if (HEAD) {
        for (int i = tid; i < 4 * kPosTile + 3; i += 256) {
            const long long q = 4ll * p0 - 3 + i;
            head_x[i] = (q >= 0 && q < (long long)l_head) ? in[q] : 0.f;
        }
        for (int i = tid; i < c_in; i += 256) {   // c_in <= kHeadMaxC (the launcher sees to it)
            head_p[4 * i] = head_w[3 * i]; head_p[4 * i + 1] = head_w[3 * i + 1]; head_p[4 * i + 2] = head_w[3 * i + 2];
            head_p[4 * i + 3] = head_b[i];
        }
        // the first barrier of the contraction loop orders these stores before their first use in stage()
    }

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
    // weights: 16-byte loads (the load instructions' issue rate, not their bytes, is what the staging costs);
    // group f = tid + 256 i of four channels: row f / 16 = (tid >> 4) + 16 i of the chunk's 48, channels 4 (f % 16) ..
    const uint32_t gw0 = (uint32_t)((tid >> 4) * c_out + co0 + (tid & 15) * 4);
    float xr[HEAD ? 1 : kXRegs];
    f4v wr[kWRegs / 4];
    auto fetch = [&](int c0) {
        const float *win = wt + (size_t)c0 * 3 * c_out + gw0;
        if (!HEAD) {
            const float *xin = in + (size_t)c0 * l_in;
#pragma unroll
            for (int i = 0; i < kXRegs; ++i) xr[i] = xin[gx[i]];
        }
#pragma unroll
        for (int i = 0; i < kWRegs / 4; ++i) wr[i] = *(const f4v *)(win + (size_t)(16 * i) * c_out);
    };
    auto stage = [&](int c0) {
#pragma unroll
        for (int i = 0; i < kXRegs; ++i) {
            const int e = tid + 256 * i;
            const int ci = e / kXPerRow, r = e % kXPerRow;
            const int slot = e < kCiChunk * kXPerRow ? ci * kRowPad + (r <= kPosTile ? r : kEvenOff + (r - kPosTile - 1))
                                                     : kCiChunk * kRowPad;
            float x;
            if (HEAD) {
                // h[c0 + ci][q], q = 2 (p0 + r) - 1 (odd slots) or 2 (p0 + r - 65) (even slots): its window starts
                // at x[2 q - 1] = head_x[4 r] or head_x[4 (r - 65) + 2]
                const int x0 = r <= kPosTile ? 4 * r : 4 * (r - kPosTile - 1) + 2;
                const float *hp = head_p + 4 * (c0 + (e < kCiChunk * kXPerRow ? ci : 0));
                float a = hp[3];
                a = fmaf(hp[0], head_x[x0], a);
                a = fmaf(hp[1], head_x[x0 + 1], a);
                a = fmaf(hp[2], head_x[x0 + 2], a);
                x = leaky_m(a, slope);
            } else {
                x = xr[i];
            }
            xs[slot] = ((live >> i) & 1u) ? x : 0.f;
        }
#pragma unroll
        for (int i = 0; i < kWRegs / 4; ++i) *(f4v *)(ws + (tid + 256 * i) * 4) = wr[i];
    };

    acc16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    fetch(c_lo);
    for (int c0 = c_lo; c0 < c_hi; c0 += kCiChunk) {
        __syncthreads();   // the previous chunk's readers are done
        stage(c0);
        __syncthreads();
        if (c0 + kCiChunk < c_hi) fetch(c0 + kCiChunk);   // in flight during the multiplications below
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
    if (SPLIT) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int co = co0 + wm * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
            if (p < l_out) out[(size_t)co * l_out + p] = acc[r];
        }
        return;
    }
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
        hipLaunchKernelGGL((k_conv3s2_mfma<true, false>), grid, dim3(256), 0, st, in, out, l.wt, l.b, l.c_in, l.c_out, l_in,
                           l_out, (int)act, slope, tail->w, tail->b, tail->c_out, (int)tail_act, nullptr, nullptr, 0u, 1);
    else
        hipLaunchKernelGGL((k_conv3s2_mfma<false, false>), grid, dim3(256), 0, st, in, out, l.wt, l.b, l.c_in, l.c_out, l_in,
                           l_out, (int)act, slope, nullptr, nullptr, 0, 0, nullptr, nullptr, 0u, 1);
    return true;
}

// ---- split contraction for layers with few output tiles ----------------------------------------------
// How many runs the contraction of layer `l` is cut into for outputs of length l_out and `batch` nodes: 1 (no
// split) unless the unsplit launch would leave most compute units without a block and the layer is deep.
int conv3s2_mfma_splits(const LayerDev &l, uint32_t l_out, int batch) {
    if (!l.wt || l.ksize != 3 || l.stride != 2 || l.c_in % kCiChunk != 0 || l.c_out % 64 != 0 || l.c_in < 128) return 1;
    const uint64_t blocks = (uint64_t)((l_out + kPosTile - 1) / kPosTile) * (l.c_out / 64) * batch;
    if (blocks == 0 || blocks >= 192) return 1;
    int best = 1;
    for (int s = 2; s <= 8; s *= 2)   // 2, 4 or 8 equal runs of whole chunks, at most about two blocks per compute unit
        if ((l.c_in / kCiChunk) % s == 0 && blocks * s <= 512) best = s;
    return best;
}

// Adds up the partial sums of a split contraction: y[co][p] = act(bias[co] + sum_s part[b][s][co][p]), summed in
// the order s = 0, 1, ..  (fixed, so the result does not depend on which block ran when).  tail_c == 0: out is
// [b][c_out][l_out].  tail_c > 0 (<= 4): a following kernel-1 / stride-1 layer to tail_c channels is applied here
// as well and out is [b][tail_c][l_out].  Block: 64 positions (one per lane) x 16 wavefronts that take every
// sixteenth channel each (all of a thread's loads are independent and in flight together: the kernel is a
// latency chain otherwise); the tail's sums of the sixteen meet in LDS.
template <int SPLITS>
__global__ __launch_bounds__(1024) void k_splitk_finish(const float *__restrict__ part, float *__restrict__ out,
                                                        const float *__restrict__ bias, int c_out, uint32_t l_out, int act,
                                                        float slope, const float *__restrict__ tail_w /*[tail_c][c_out]*/,
                                                        const float *__restrict__ tail_b, int tail_c, int tail_act) {
    __shared__ float red[16][4][64];   // [wavefront][tail channel][position]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t p = blockIdx.x * 64 + lane;
    const bool live = p < l_out;
    part += (size_t)blockIdx.y * SPLITS * c_out * l_out;
    out += (size_t)blockIdx.y * (tail_c ? tail_c : c_out) * l_out;
    float t[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int co = wave; co < c_out; co += 16) {
        float x[SPLITS];
#pragma unroll
        for (int s = 0; s < SPLITS; ++s) x[s] = live ? part[((size_t)s * c_out + co) * l_out + p] : 0.f;
        float y = x[0];
#pragma unroll
        for (int s = 1; s < SPLITS; ++s) y += x[s];
        y += bias[co];
        if (act) y = leaky_m(y, slope);
        if (tail_c) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (c < tail_c) t[c] = fmaf(tail_w[c * c_out + co], y, t[c]);
        } else if (live) {
            out[(size_t)co * l_out + p] = y;
        }
    }
    if (tail_c == 0) return;   // the same for the whole block
#pragma unroll
    for (int c = 0; c < 4; ++c) red[wave][c][lane] = t[c];
    __syncthreads();
    if (wave < tail_c && live) {   // wavefront c finishes tail channel c
        float z = tail_b[wave];
#pragma unroll
        for (int w = 0; w < 16; ++w) z += red[w][wave][lane];
        out[(size_t)wave * l_out + p] = tail_act ? leaky_m(z, slope) : z;
    }
}

// Layer `l` with its contraction split `splits` ways (conv3s2_mfma_splits): partial sums to `part`
// ([batch][splits][c_out][l_out] floats), then the finish kernel to `out`.  tail (nullable): a kernel-1 /
// stride-1 layer from l.c_out to at most 4 channels applied in the finish kernel; `out` is then its output.
bool launch_conv3s2_mfma_splitk(const float *in, float *part, float *out, const LayerDev &l, uint32_t l_in, uint32_t l_out,
                                int batch, int splits, bool act, float slope, hipStream_t st, const LayerDev *tail,
                                bool tail_act) {
    if (!conv3s2_mfma_covers(l, l_in) || (splits != 2 && splits != 4 && splits != 8) || (l.c_in / kCiChunk) % splits != 0) return false;
    if (tail && !(tail->ksize == 1 && tail->stride == 1 && tail->c_in == l.c_out && tail->c_out <= 4)) return false;
    if (l_out == 0) return true;
    dim3 grid((l_out + kPosTile - 1) / kPosTile, (l.c_out / 64) * splits, batch);
    hipLaunchKernelGGL((k_conv3s2_mfma<false, false, true>), grid, dim3(256), 0, st, in, part, l.wt, l.b, l.c_in, l.c_out, l_in,
                       l_out, 0, slope, nullptr, nullptr, 0, 0, nullptr, nullptr, 0u, splits);
    const dim3 fgrid((l_out + 63) / 64, batch);
#define LGC_FINISH(S) hipLaunchKernelGGL(k_splitk_finish<S>, fgrid, dim3(1024), 0, st, part, out, l.b, l.c_out, l_out, (int)act, slope, \
                                         tail ? tail->w : nullptr, tail ? tail->b : nullptr, tail ? tail->c_out : 0, (int)tail_act)
    if (splits == 2) LGC_FINISH(2); else if (splits == 4) LGC_FINISH(4); else LGC_FINISH(8);
#undef LGC_FINISH
    return true;
}

// The two first layers of a stack in one launch: `head` (one input channel, kernel 3, stride 2, always
// followed by the non-linearity) is evaluated inside the staging of `l`.  x: [batch][1][l_x]; l_in, l_out:
// input and output length of `l` (l_in is the head's output length).
bool launch_conv3s2_mfma_head(const float *x, float *out, const LayerDev &head, const LayerDev &l, uint32_t l_x,
                              uint32_t l_in, uint32_t l_out, int batch, bool act, float slope, hipStream_t st) {
    if (!conv3s2_mfma_covers(l, l_in)) return false;
    if (!(head.c_in == 1 && head.ksize == 3 && head.stride == 2 && head.c_out == l.c_in && l.c_in <= kHeadMaxC)) return false;
    if (l_out == 0) return true;
    dim3 grid((l_out + kPosTile - 1) / kPosTile, l.c_out / 64, batch);
    hipLaunchKernelGGL((k_conv3s2_mfma<false, true>), grid, dim3(256), 0, st, x, out, l.wt, l.b, l.c_in, l.c_out, l_in, l_out,
                       (int)act, slope, nullptr, nullptr, 0, 0, head.w, head.b, l_x, 1);
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
// HEAD: the layer's input is made on the fly from the two narrow layers in front of it (Table II: deconv1
// 4->4, kernel 3 / stride 1, and deconv2 4->32, kernel 3 / stride 2, in front of deconv3 32->64): `in` is then
// the first of them's input z [b][hd.c0][hd.l_z].  A block first evaluates the stride-1 layer on the 65
// positions its tile needs (into LDS), and every staged input h2[ci][m] is the stride-2 layer evaluated there:
// even m = 2p from h1[.][p], odd m = 2p + 1 from h1[.][p] and h1[.][p + 1].  No intermediate tensors, two
// launches fewer, no global loads of inputs in the contraction loop.
struct ConvtHead {
    const float *w1, *b1;   // [c0][c1][3], [c1]    kernel 3, stride 1
    const float *w2, *b2;   // [c1][c_in][3], [c_in] kernel 3, stride 2
    int c0, c1;             // both <= kHeadNarrow
    uint32_t l_z;           // length of z and of the stride-1 layer's output
};
constexpr int kHeadNarrow = 8;
constexpr int kHeadWide = 64;     // most channels out of the stride-2 head layer (= c_in of the deep layer)
constexpr int kHeadPos = kTPosTile / 2 + 1;   // 65 positions of h1 per tile

template <bool TAIL, int HC1>   // HC1: 0 = no head, else the channels between the two head layers (hd.c1)
__global__ __launch_bounds__(256) void k_convt3s2_mfma(const float *__restrict__ in, float *__restrict__ out,
                                                       const float *__restrict__ wt, const float *__restrict__ bias,
                                                       int c_in, int c_out, uint32_t l_in, uint32_t l_out, int act,
                                                       float slope, const float *__restrict__ tail_w /*[32]*/,
                                                       const float *__restrict__ tail_b, int tail_act, ConvtHead hd) {
    __shared__ float xs[kCiChunk * kTRowPad + 1];
    __shared__ float ws[3 * kCiChunk * 32];
    constexpr bool HEAD = HC1 > 0;
    __shared__ float hz[HEAD ? kHeadNarrow * (kHeadPos + 2) : 1];        // z[c][m0/2 - 1 .. m0/2 + 65]
    __shared__ float h1[HEAD ? kHeadNarrow * kHeadPos : 1];              // h1[c][m0/2 .. m0/2 + 64]
    __shared__ float hw1[HEAD ? kHeadNarrow * kHeadNarrow * 3 + kHeadNarrow : 1];
    __shared__ float hw2[HEAD ? kHeadNarrow * kHeadWide * 3 + kHeadWide : 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const uint32_t m0 = blockIdx.x * kTPosTile;
    const int co0 = blockIdx.y * 32;
    in += (size_t)blockIdx.z * (HEAD ? (size_t)hd.c0 * hd.l_z : (size_t)c_in * l_in);
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
    float xr[HEAD ? 1 : kTXRegs], wr[kTWRegs];
    auto fetch = [&](int c0) {
        const float *win = wt + (size_t)c0 * c_out;
        if (!HEAD) {
            const float *xin = in + (size_t)c0 * l_in;
#pragma unroll
            for (int i = 0; i < kTXRegs; ++i) xr[i] = xin[gx[i]];
        }
#pragma unroll
        for (int i = 0; i < kTWRegs; ++i) wr[i] = win[gw[i]];
    };
    auto stage = [&](int c0) {
#pragma unroll
        for (int i = 0; i < kTXRegs; ++i) {
            float x;
            if (HEAD) {
                // h2[c][m0 + r] of the stride-2 head layer (m0 is even): r = 2j from h1[.][j], r = 2j + 1 from
                // h1[.][j] (tap 2) and h1[.][j + 1] (tap 0)
                const int e = tid + 256 * i;
                const bool slot = e < kCiChunk * (kTPosTile + 1);
                const int c = c0 + (slot ? e / (kTPosTile + 1) : 0), r = e % (kTPosTile + 1), j = r >> 1;
                float a = hw2[kHeadNarrow * kHeadWide * 3 + c];
                const bool odd = r & 1;   // no branch: both forms are evaluated and one is kept
#pragma unroll
                for (int c1 = 0; c1 < HC1; ++c1) {
                    const float *w = hw2 + (c1 * c_in + c) * 3;
                    const float *h = h1 + c1 * kHeadPos + j;
                    const float h0 = h[0], hn = h[odd ? 1 : 0];
                    const float even_a = fmaf(w[1], h0, a);
                    const float odd_a = fmaf(w[2], h0, fmaf(w[0], hn, a));
                    a = odd ? odd_a : even_a;
                }
                x = leaky_m(a, slope);
            } else {
                x = xr[i];
            }
            xs[lx[i]] = ((live >> i) & 1u) ? x : 0.f;
        }
#pragma unroll
        for (int i = 0; i < kTWRegs; ++i) ws[tid + 256 * i] = wr[i];
    };

    acc16 even, odd;
#pragma unroll
    for (int r = 0; r < 16; ++r) { even[r] = 0.f; odd[r] = 0.f; }

    fetch(0);
    if (HEAD) {   // after the first fetch, so that the deep layer's weights are on their way meanwhile
        const long long pz = (long long)(m0 / 2) - 1;   // first position of the z stretch
        for (int i = tid; i < hd.c0 * (kHeadPos + 2); i += 256) {
            const int c = i / (kHeadPos + 2), j = i % (kHeadPos + 2);
            const long long q = pz + j;
            hz[i] = (q >= 0 && q < (long long)hd.l_z) ? in[(size_t)c * hd.l_z + q] : 0.f;
        }
        for (int i = tid; i < hd.c0 * hd.c1 * 3; i += 256) hw1[i] = hd.w1[i];
        for (int i = tid; i < hd.c1; i += 256) hw1[kHeadNarrow * kHeadNarrow * 3 + i] = hd.b1[i];
        for (int i = tid; i < hd.c1 * c_in * 3; i += 256) hw2[i] = hd.w2[i];
        for (int i = tid; i < c_in; i += 256) hw2[kHeadNarrow * kHeadWide * 3 + i] = hd.b2[i];
        __syncthreads();
        // stride-1 transposed layer: h1[c][p] = act(b1[c] + sum_cz (w1[cz][c][0] z[cz][p+1] + w1[cz][c][1] z[cz][p]
        // + w1[cz][c][2] z[cz][p-1])); positions outside [0, l_z) hold 0
        for (int i = tid; i < hd.c1 * kHeadPos; i += 256) {
            const int c = i / kHeadPos, j = i % kHeadPos;   // p = m0/2 + j, z stretch index of p is j + 1
            float a = hw1[kHeadNarrow * kHeadNarrow * 3 + c];
            for (int cz = 0; cz < hd.c0; ++cz) {
                const float *w = hw1 + (cz * hd.c1 + c) * 3;
                const float *z = hz + cz * (kHeadPos + 2) + j;
                a = fmaf(w[0], z[2], a);
                a = fmaf(w[1], z[1], a);
                a = fmaf(w[2], z[0], a);
            }
            h1[i] = (uint64_t)(m0 / 2) + j < hd.l_z ? leaky_m(a, slope) : 0.f;
        }
        // the first barrier of the contraction loop orders these stores before their first use in stage()
    }
    for (int c0 = 0; c0 < c_in; c0 += kCiChunk) {
        __syncthreads();
        stage(c0);
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
        hipLaunchKernelGGL((k_convt3s2_mfma<true, 0>), grid, dim3(256), 0, st, in, out, l.wt, l.b, l.c_in, l.c_out, l_in,
                           l_out, (int)act, slope, tail->w, tail->b, (int)tail_act, ConvtHead{});
    else
        hipLaunchKernelGGL((k_convt3s2_mfma<false, 0>), grid, dim3(256), 0, st, in, out, l.wt, l.b, l.c_in, l.c_out, l_in,
                           l_out, (int)act, slope, nullptr, nullptr, 0, ConvtHead{});
    return true;
}

// The first three layers of a decoder in one launch: h1 (kernel 3, stride 1) and h2 (kernel 3, stride 2), both
// narrow and both followed by the non-linearity, are evaluated inside the staging of the deep layer `l`.
// z: [batch][h1.c_in][l_z]; l_in: input length of `l` (= output length of h2, 2 l_z or 2 l_z - 1); l_out: its
// output length.
bool launch_convt3s2_mfma_head(const float *z, float *out, const LayerDev &h1, const LayerDev &h2, const LayerDev &l,
                               uint32_t l_z, uint32_t l_in, uint32_t l_out, int batch, bool act, float slope,
                               hipStream_t st) {
    if (!l.wt || l.ksize != 3 || l.stride != 2 || l.c_in % kCiChunk != 0 || l.c_out % 32 != 0) return false;
    if ((uint64_t)l_in * kCiChunk >= (1ull << 32) || (uint64_t)l.c_in * 3 * l.c_out >= (1ull << 32)) return false;
    if (!(h1.ksize == 3 && h1.stride == 1 && h2.ksize == 3 && h2.stride == 2 && h1.c_out == h2.c_in && h2.c_out == l.c_in &&
          h1.c_in <= kHeadNarrow && (h1.c_out == 4 || h1.c_out == 8) && l.c_in <= kHeadWide))
        return false;
    if (!(l_in == 2 * l_z || l_in + 1 == 2 * l_z)) return false;
    if (l_out == 0) return true;
    const uint32_t m_count = (l_out + 1) / 2;
    dim3 grid((m_count + kTPosTile - 1) / kTPosTile, l.c_out / 32, batch);
    const ConvtHead hd{h1.w, h1.b, h2.w, h2.b, h1.c_in, h1.c_out, l_z};
    if (h1.c_out == 4)
        hipLaunchKernelGGL((k_convt3s2_mfma<false, 4>), grid, dim3(256), 0, st, z, out, l.wt, l.b, l.c_in, l.c_out, l_in, l_out,
                           (int)act, slope, nullptr, nullptr, 0, hd);
    else
        hipLaunchKernelGGL((k_convt3s2_mfma<false, 8>), grid, dim3(256), 0, st, z, out, l.wt, l.b, l.c_in, l.c_out, l_in, l_out,
                           (int)act, slope, nullptr, nullptr, 0, hd);
    return true;
}

}  // namespace lgc
