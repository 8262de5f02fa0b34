// Device helpers for stage 2: raw-bit access to f32 / bf16 weights and the
// in-register N:M selection on exact scores.
#pragma once

#include "dass_internal.h"

namespace dass {

// 32-bit words that hold `n` consecutive elements of dtype DT.
template <int DT>
__host__ __device__ constexpr int words_for(int n)
{
    return DT == DASS_BF16 ? n / 2 : n;
}

// |element e| of a run of elements packed in `words`, widened to float (exact).
template <int DT>
__device__ __forceinline__ float abs_elem(const uint32_t *words, int e)
{
    if constexpr (DT == DASS_BF16) {
        const uint32_t w = words[e >> 1];
        const uint32_t bits = (e & 1) ? (w & 0x7fff0000u) : ((w << 16) & 0x7fff0000u);
        return __uint_as_float(bits);
    } else {
        return __uint_as_float(words[e] & 0x7fffffffu);
    }
}

// Overwrite element e with +0.
template <int DT>
__device__ __forceinline__ void zero_elem(uint32_t *words, int e)
{
    if constexpr (DT == DASS_BF16)
        words[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
    else
        words[e] = 0u;
}

// Keep-bits of one group of M exact scores s[0..M).  Position a "wins" against b
// when s[a] > s[b], or s[a] == s[b] and a < b; this is a strict total order, so
// the win counts are a permutation of 0..M-1 and position a is among the
// n_keep best exactly when wins[a] >= M - n_keep =: min_wins.
// (Sec. 3 "Extension to N:M Sparsity"; ties: lower index kept.)
template <int M>
__device__ __forceinline__ uint32_t nm_keep_bits(const double *s, int min_wins)
{
    int wins[M];
#pragma unroll
    for (int a = 0; a < M; ++a)
        wins[a] = 0;
#pragma unroll
    for (int a = 0; a < M; ++a) {
#pragma unroll
        for (int b = a + 1; b < M; ++b) {
            const int c = s[a] >= s[b] ? 1 : 0;
            wins[a] += c;
            wins[b] += 1 - c;
        }
    }
    uint32_t bits = 0;
#pragma unroll
    for (int a = 0; a < M; ++a)
        bits |= (wins[a] >= min_wins ? 1u : 0u) << a;
    return bits;
}

// ---------------------------------------------------------------------------
// Fast exact selection for the n_keep = m / 2 patterns (1:2, 2:4, 4:8).
//
// The exact score |w| * f of an f32 (or bf16) weight and an f32 factor is kept
// as the unevaluated sum p + q of two f32: p = fl(|w| f) and q = fma(|w|, f, -p),
// the rounding error of p, which is itself an f32 whenever no underflow gets in
// the way (callers check that).  Rounding is monotonic, so scores order like
// the pairs (p, q) taken lexicographically.
//
// A comparison of two scores is made for all 64 lanes at once and lands in a
// scalar register as a lane mask; everything after it (who beats whom, who has
// enough wins) is bitwise logic on such masks, done by the scalar unit.
// ---------------------------------------------------------------------------
typedef uint64_t lanemask_t;

enum { kCmpEq = 1, kCmpGt = 2, kCmpGe = 3, kCmpLt = 4 };   // ordered f32 predicates of the compare builtin

// Lanes where score a >= score b (a sits before b in its group, so a also wins ties).
__device__ __forceinline__ lanemask_t score_ge(float pa, float qa, float pb, float qb)
{
    const lanemask_t gt = __builtin_amdgcn_fcmpf(pa, pb, kCmpGt);
    const lanemask_t eq = __builtin_amdgcn_fcmpf(pa, pb, kCmpEq);
    const lanemask_t ge = __builtin_amdgcn_fcmpf(qa, qb, kCmpGe);
    return gt | (eq & ge);
}

__device__ __forceinline__ lanemask_t majority3(lanemask_t x, lanemask_t y, lanemask_t z)
{
    return (x & y) | (z & (x | y));
}

// Calls apply(a, keep) for every position a of a group, where keep = lanes in which position
// a is among the M / 2 best, i.e. beats at least M / 2 of the other M - 1 positions.  p, q: the
// M scores of the group.  Positions are finished one after the other (for M = 8 with a
// scheduling fence in between) so that only the comparisons with later positions stay live:
// all 28 masks of an 8-group and their complements would not fit the scalar registers.
template <int M, typename Apply>
__device__ __forceinline__ void keep_top_half(const float *p, const float *q, Apply apply)
{
    static_assert(M == 2 || M == 4 || M == 8, "patterns 1:2, 2:4 and 4:8");
    lanemask_t beats[M][M];   // beats[a][b] for a < b: a ranks above b
#pragma unroll
    for (int a = 0; a < M; ++a) {
        lanemask_t x[M - 1];
        int n = 0;
#pragma unroll
        for (int b = 0; b < a; ++b)
            x[n++] = ~beats[b][a];
#pragma unroll
        for (int b = a + 1; b < M; ++b) {
            beats[a][b] = score_ge(p[a], q[a], p[b], q[b]);
            x[n++] = beats[a][b];
        }
        lanemask_t keep;
        if constexpr (M == 2) {
            keep = x[0];
        } else if constexpr (M == 4) {
            keep = majority3(x[0], x[1], x[2]);
        } else {
            // at least 4 of 7: carry-save adders; the weight-4 bit of the count is the answer
            const lanemask_t s1 = x[0] ^ x[1] ^ x[2], c1 = majority3(x[0], x[1], x[2]);
            const lanemask_t s2 = x[3] ^ x[4] ^ x[5], c2 = majority3(x[3], x[4], x[5]);
            const lanemask_t c3 = majority3(s1, s2, x[6]);
            keep = majority3(c1, c2, c3);
        }
        apply(a, keep);
        if constexpr (M == 8)
            __builtin_amdgcn_sched_barrier(0);
    }
}

// 16-byte vector of raw words, the unit of every global access of stage 2.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

struct alignas(16) Vec16 {
    uint32_t w[4];
};

__device__ __forceinline__ Vec16 load16(const void *p)
{
    return *reinterpret_cast<const Vec16 *>(p);
}
__device__ __forceinline__ void store16(void *p, const Vec16 &v)
{
    *reinterpret_cast<Vec16 *>(p) = v;
}

}  // namespace dass
