// Top-k selection of Alg. 2 ("top-k indices" line, Appendix C) inside one wavefront.
#pragma once

#include "stream_common.h"

namespace stream {

// Order-preserving map of a float's bit pattern to an unsigned integer (-inf lowest).
__device__ __forceinline__ unsigned sortable_bits(float v)
{
    const unsigned u = __builtin_bit_cast(unsigned, v + 0.f);   // -0 -> +0: equal as scores
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Keeps the k valid branches with the largest scores, equal scores going to the lower position.
// A lane holds NB branches (NB = 2: lane j holds positions 2j and 2j+1, the children of node j;
// NB = 1: lane j holds position j); s[] / v[] are their scores and validity, keep[] the result.
//
// The k-th largest score is found by a binary search over the 32 bits of the order-preserving
// integer image of the scores, most significant bit first: a bit stays set if at least k
// branches are >= the candidate.  A step is one vector compare per branch of a lane, whose lane
// mask is counted on the scalar unit.  The search stops as soon as exactly k branches are >= the
// candidate (they are the answer); with distinct scores that happens at the first bit in which
// the k-th and the (k+1)-th largest differ.  Only rows whose k-th and (k+1)-th largest scores are
// equal run all 32 steps; they keep what lies above the threshold and, of the branches equal
// to it, the first (k - number above) in position order.
template <int NB>
__device__ __forceinline__ void select_topk_wave(const float (&s)[NB], const bool (&v)[NB], int k, int lane,
                                                 bool (&keep)[NB])
{
    unsigned u[NB];
    int n_valid = 0;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const unsigned b = sortable_bits(s[i]);
        u[i] = v[i] ? (b ? b : 1u) : 0u;         // 0 marks "not a candidate": below every threshold
        n_valid += __popcll(__ballot(v[i]));
    }
    if (n_valid <= k) {                           // wave-uniform
#pragma unroll
        for (int i = 0; i < NB; ++i) keep[i] = v[i];
        return;
    }
    unsigned thr = 0;
    bool exact = false;
    for (int bit = 31; bit >= 0; --bit) {
        const unsigned t = thr | (1u << bit);
        int ge = 0;
#pragma unroll
        for (int i = 0; i < NB; ++i) ge += __popcll(__ballot(u[i] >= t));
        if (ge >= k) {
            thr = t;
            if (ge == k) { exact = true; break; }
        }
    }
    if (exact) {
#pragma unroll
        for (int i = 0; i < NB; ++i) keep[i] = u[i] >= thr;
        return;
    }
    // ties at the threshold
    const unsigned long long lt = (1ull << lane) - 1ull;
    int n_gt = 0;
#pragma unroll
    for (int i = 0; i < NB; ++i) n_gt += __popcll(__ballot(u[i] > thr));
    const int need = k - n_gt;
    int before = 0;                               // equal branches at lower positions
#pragma unroll
    for (int i = 0; i < NB; ++i) before += __popcll(__ballot(u[i] == thr) & lt);
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const bool eq = u[i] == thr;
        keep[i] = u[i] > thr || (eq && before < need);
        before += eq ? 1 : 0;                     // this lane's own lower position
    }
}

}  // namespace stream
