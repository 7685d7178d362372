// Thresholds carried from one selection to the next (the record type is Carry in lgc_internal.h).
//
// Alg. 1 / Alg. 2 select every iteration from the same residuals, whose k-th largest magnitude T* moves smoothly
// once the residuals have piled up.  A record holds log2 |T*| of up to three selections in a row.  T* of the next
// selection is predicted on the line through the last two; the candidate threshold offered to it lies below the
// prediction by a margin, the larger of
//   * the distance that holds `target` times k candidates, from the slope that this selection measured itself:
//     its candidates above t_est were `total`, so log2(count) falls by log2(total / k) over log2 T* - log2 t_est;
//   * four times the recent miss: how far T* lay from what the two selections before it predicted, the largest
//     of the recent selections (each selection's own, or 0.85 of the value before).
// The offer is made only if that margin is expected to hold no more than `most` times k candidates, after four
// selections in a row (two misses on record), and after offers that failed only after twice as many each time
// (8, 16, ... 128).  A wrong offer costs the next selection its fast path (too few candidates, or too many for
// the list), never its result.
#pragma once
#include "lgc_internal.h"

namespace lgc {

// ok: the selection was served from the candidates above t_est (`total` of them, >= k); carried: t_est had been
// offered by the record.  target, most: log2 of the candidate counts over k (aimed at / at most).  fresh: the
// record is not the previous selection's (another kind of selection came between).
__device__ __forceinline__ void carry_update(Carry *c, const uint32_t n, const uint32_t k, const bool fresh, const bool ok,
                                             const bool carried, const uint32_t thr, const uint32_t t_est,
                                             const uint32_t total, const float target, const float most) {
    const bool same = !fresh && c->n == n && c->k == k;     // the record is the previous selection's, of this shape
    const bool follows = same && c->len > 0;
    const float l1 = c->log2_t[0], l2 = c->log2_t[1];
    uint32_t len = 0, next = 0, fails = same ? c->fails : 0u, held = same ? c->held : 0u;
    if (carried) {
        if (!ok) { fails = fails < 5 ? fails + 1 : 5u; held = 0; }
        else if (++held >= 64) { fails = fails ? fails - 1 : 0u; held = 0; }
    }
    float l0 = 0.f, miss = 0.f;
    constexpr uint32_t kMinNormal = 0x00800000u, kInf = 0x7f800000u;
    if (ok && thr >= kMinNormal && thr < kInf && t_est >= kMinNormal && t_est < thr) {
        l0 = log2f(__uint_as_float(thr));
        len = follows ? (c->len < 255 ? c->len + 1 : 255u) : 1u;
        if (len >= 3) miss = fmaxf(fabsf(l0 - (2.f * l1 - l2)), len > 3 ? 0.85f * c->miss : 0.f);
        const float ratio = total > k ? log2f((float)total / (float)k) : 0.f;
        const float used = l0 - log2f(__uint_as_float(t_est));
        if (len >= (4u << fails) && ratio >= 0.05f && used > 0.f) {
            const float slope = ratio / used;                // log2(count) per log2(threshold)
            const float gap = fmaxf(fminf(fmaxf(target / slope, 0.25f * used), 4.f * used), 4.f * miss);
            if (gap <= 0.25f && gap * slope <= most) {
                const uint32_t t = __float_as_uint(exp2f(2.f * l0 - l1 - gap));
                if (t >= kMinNormal && t < kInf) next = t;
            }
        }
    }
    c->n = n; c->k = k; c->len = len;
    c->log2_t[0] = l0; c->log2_t[1] = l1; c->log2_t[2] = l2;
    c->next_t_est = next; c->fails = fails; c->held = held; c->miss = miss;
}

}  // namespace lgc
