// Score-function stage shared by the bf16 matrix-core forward kernels: turns one 32-key x
// 32-query tile of raw dot products (transposed C layout: the lane owns one query, 16 keys)
// into packed bf16 weights P^T, ready to be the B operand of O^T += V^T P^T.
//   activation heads (Eq. (GDPA)):  P = Act(S * scale), zero outside the visible keys
//   softmax heads (Eq. (PMA), Eq. (seed-level attention), Eq. (sliding window)):  online
//   softmax with a running reference maximum and sum per query; the O^T accumulators are
//   rescaled when the reference moves.
#pragma once
#include "mfma_tile.h"

namespace kunlun {

constexpr float LOG2E = 1.4426950408889634f;

// Largest growth of a row maximum (log2 units) that is tolerated before the running
// reference of the online softmax is moved: weights stay below 2^8, and the accumulators are
// rescaled only when some query of the wave exceeds it.  The result is unchanged in exact
// arithmetic because numerator and denominator use the same reference.
constexpr float SOFTMAX_LAZY_LOG2 = 8.f;

// sacc: raw scores of this lane's query for keys key_base + 8*(v/4) + 4g + (v%4).
// Key k is visible iff (unsigned)(k - key_lo) <= key_span; rel0 = key_base + 4g - key_lo.
// need_mask (wave-uniform): some (query, key) pair of the tile is not visible.
// sc = scale (activation heads) or scale * log2(e) (softmax heads; scale > 0).
// FRESH: the first tile of a query block under softmax - m_ref = -inf, l_run = 0 and the accumulators hold nothing
// yet (they need not even be initialised), so the reference simply becomes the tile's maximum and nothing is
// rescaled; the result is the same, bit for bit, as that of the general path on zeroed accumulators.
template <int ACT, int DB, int NQB, bool FRESH = false>
__device__ __forceinline__ void score_to_weights(const f32x16& sacc, bool need_mask, unsigned rel0, unsigned key_span,
                                                 float sc, float& m_ref, float& l_run, f32x16 (&oacc)[DB][NQB], int qb,
                                                 bf16x8 (&pf)[2]) {
    constexpr bool SOFTMAX = ACT == KUNLUN_ACT_SOFTMAX;
    float pv[16];  // raw scores, then weights
#pragma unroll
    for (int v = 0; v < 16; ++v) pv[v] = sacc[v];
    if (SOFTMAX) {
        if (need_mask) {
            // (an empty volatile statement: the compiler must keep this a branch; folded into selects, the 48
            // compare / select / add operations below would run for every tile, and few tiles need them)
            asm volatile("");
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const bool ok = rel0 + (unsigned)(8 * (v >> 2) + (v & 3)) <= key_span;
                pv[v] = ok ? pv[v] : -INFINITY;
            }
        }
        // scale > 0 (checked on the host), so the maximum commutes with the scaling;
        // scores are handled in log2 units (scale * log2 e folded into sc)
        float mx = pv[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, pv[v]);
        mx = halves_max(mx) * sc;  // the other lane half holds the other 16 keys
        const bool grow = mx > m_ref + SOFTMAX_LAZY_LOG2;
        if (FRESH) {
            m_ref = mx;
        } else if (__builtin_amdgcn_ballot_w64(grow) != 0) {
            const float corr = grow ? fast_exp2(m_ref - mx) : 1.f;
            m_ref = grow ? mx : m_ref;
            l_run *= corr;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[db][qb][v] *= corr;
        }
        const float neg_m = m_ref == -INFINITY ? 0.f : -m_ref;
        float sum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            pv[v] = fast_exp2(fmaf(pv[v], sc, neg_m));
            sum += pv[v];
        }
        l_run += sum;
    } else if (need_mask) {
        asm volatile("");  // a branch, as above
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const bool ok = rel0 + (unsigned)(8 * (v >> 2) + (v & 3)) <= key_span;
            const float w = act_fast<ACT>(pv[v] * sc);
            pv[v] = ok ? w : 0.f;
        }
    } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) pv[v] = act_fast<ACT>(pv[v] * sc);
    }
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[c][e] = (bf16_t)pv[8 * c + e];
}

}  // namespace kunlun
