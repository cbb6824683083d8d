// Algorithm 1 of the paper for the weights one lane holds: shared by the whole-matrix kernel
// (mq_quant.hip) and the column loop (mq_gptq.hip), so that both take bit-identical decisions.
//
// The argmin is decided in floating point, so the operations are fixed: binary32, each rounded on
// its own (contraction into fused multiply-adds is switched off here), in the order
//     t = S - zero;  D = scale * t;  e = w - D;  p = e * e;  E = E + lambda_r * p      (r ascending)
// and the smallest q wins a tie.  What is saved against evaluating 256 x |R| terms is only work
// whose result is the same bit for bit: S(q, r) is constant on runs of 2^(8-r) candidates, so the
// term of width r is recomputed only where its slice changes, and the partial sum over the widths
// below the lowest one that changed is reused.  The candidate loop is unrolled completely: which
// slice changes at which q is known at compile time.
#pragma once
#include "mq_internal.h"
#include "mq_static_for.h"

namespace mq {

struct QuantLambda {
    float v[kC];  // lambda of width r at v[r - 1]; 0 = not a target width
};

// the slice of candidate Q at width r changes against candidate Q - 1 (Eq. 1, round half up, clamp)
constexpr int slice_index_of(int q, int r) {
    const int sh = kC - r;
    const int t = sh ? (q + (1 << (sh - 1))) >> sh : q;
    return t < (1 << r) - 1 ? t : (1 << r) - 1;
}
constexpr bool slice_changes(int q, int r) { return q == 0 || slice_index_of(q, r) != slice_index_of(q - 1, r); }
constexpr int popc8(uint32_t m) { int c = 0; for (int i = 0; i < 8; ++i) c += (m >> i) & 1; return c; }
// position of width r among the widths of MASK, ascending
constexpr int level_of(uint32_t mask, int r) { return popc8(mask & ((1u << (r - 1)) - 1)); }

// MASK: bit r-1 set = the term of width r is evaluated (widths outside MASK must have lambda 0).
// VEC consecutive weights of one row (same group: same scale and zero) per lane.
template <uint32_t MASK, int VEC>
__device__ __forceinline__ void choose_codes(const float (&w)[VEC], float s, float z, const QuantLambda &lam,
                                             uint32_t (&qbest)[VEC]) {
#pragma clang fp contract(off)
    constexpr int NL = popc8(MASK);
    float err[NL][VEC];   // lambda_r * (w - D_r)^2 of the current slice of each width
    float pre[NL][VEC];   // pre[i] = err[0] + ... + err[i], added in this order
    float best[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        best[v] = __builtin_inff();
        qbest[v] = 0;
    }
    static_for<256>([&](auto qc) {
#pragma clang fp contract(off)
        constexpr int q = qc;
        bool dirty = false;  // compile-time after unrolling: a lower width changed at this q
        static_for<kC>([&](auto rc) {
#pragma clang fp contract(off)
            constexpr int r = rc + 1;
            if constexpr ((MASK >> rc) & 1) {
                constexpr int i = level_of(MASK, r);
                constexpr bool ch = slice_changes(q, r);
                if constexpr (ch) {
                    constexpr float S = (float)(slice_index_of(q, r) << (kC - r));
                    const float t = S - z;
                    const float D = s * t;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        const float e = w[v] - D;
                        const float p = e * e;
                        err[i][v] = lam.v[rc] * p;
                    }
                }
                if (ch || dirty) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        if constexpr (i == 0)
                            pre[i][v] = err[i][v];
                        else
                            pre[i][v] = pre[i - 1][v] + err[i][v];
                    }
                    dirty = true;
                }
            }
        });
        if (dirty) {  // otherwise E(q) == E(q - 1): cannot be a new strict minimum
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const bool lt = pre[NL - 1][v] < best[v];
                best[v] = lt ? pre[NL - 1][v] : best[v];
                qbest[v] = lt ? (uint32_t)q : qbest[v];
                // select now: the compiler would otherwise keep all 256 comparison masks for later
                asm volatile("" : "+v"(qbest[v]));
            }
        }
    });
}

// The same decision with the 256 candidates spread over several lanes: this lane evaluates the CPL
// candidates q_base .. q_base + CPL - 1 (q_base a multiple of CPL) and returns its best (E, q);
// the caller takes the lexicographic minimum of (E, q) over the lanes that share the weight, which
// is the first minimum over all 256.  E(q) is computed by exactly the operations of choose_codes,
// so the result is bit-identical.  A slice can change inside the run only at compile-time known
// offsets (runs no longer than CPL) or at its start (longer runs), where every term is computed.
template <uint32_t MASK, int CPL>
__device__ __forceinline__ void choose_codes_part(float w, float s, float z, const QuantLambda &lam, uint32_t q_base,
                                                  float &best, uint32_t &qbest) {
#pragma clang fp contract(off)
    constexpr int NL = popc8(MASK);
    static_assert(CPL >= 1 && 256 % CPL == 0, "candidates per lane divide 256");
    float err[NL], pre[NL];
    best = __builtin_inff();
    qbest = q_base;
    static_for<CPL>([&](auto qc) {
#pragma clang fp contract(off)
        constexpr int ql = qc;
        const uint32_t q = q_base + ql;
        bool dirty = false;
        static_for<kC>([&](auto rc) {
#pragma clang fp contract(off)
            constexpr int r = rc + 1;
            if constexpr ((MASK >> rc) & 1) {
                constexpr int i = level_of(MASK, r);
                constexpr int sh = kC - r, step = 1 << sh;
                constexpr bool ch = ql == 0 || (step <= CPL && (ql + step / 2) % step == 0);
                if constexpr (ch) {
                    uint32_t t = sh ? (q + (step >> 1)) >> sh : q;
                    constexpr uint32_t top = (1u << r) - 1;
                    t = t < top ? t : top;
                    const float S = (float)(t << sh);
                    const float d0 = S - z;
                    const float D = s * d0;
                    const float e = w - D;
                    const float p = e * e;
                    err[i] = lam.v[rc] * p;
                }
                if (ch || dirty) {
                    if constexpr (i == 0)
                        pre[i] = err[i];
                    else
                        pre[i] = pre[i - 1] + err[i];
                    dirty = true;
                }
            }
        });
        if (dirty) {
            const bool lt = pre[NL - 1] < best;
            best = lt ? pre[NL - 1] : best;
            qbest = lt ? q : qbest;
            asm volatile("" : "+v"(qbest));
        }
    });
}

// Built variants: {8} (plain rounding to the nearest code), {3,4,8} (the paper's experiments),
// {2,3,4,6,8} (the widths this library packs), and all eight widths for anything else.
inline uint32_t quant_variant_mask(uint32_t need) {
    if (!(need & ~0x80u)) return 0x80u;
    if (!(need & ~0x8Cu)) return 0x8Cu;
    if (!(need & ~0xAEu)) return 0xAEu;
    return 0xFFu;
}

}  // namespace mq
