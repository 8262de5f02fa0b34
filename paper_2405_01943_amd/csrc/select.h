// Device helpers for stage 2: raw-bit access to f32 / bf16 weights and the
// in-register N:M selection on exact scores.
#pragma once

#include "dass_internal.h"

// Stage 2 compares exact scores built from individually rounded products and differences: the
// compiler must not fuse a multiply into a neighbouring add or subtract anywhere in this code.
#pragma clang fp contract(off)

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
// The exact score |w| * f of an f32 (or bf16) weight and an f32 factor is kept as the
// unevaluated sum p + q of two f32: p = fl(|w| f') and q = fma(|w|, f', -p), the rounding
// error of p, with f' = 2^64 f.  The error term is a multiple of ulp(w) ulp(f'); with
// f' >= 2^23 (f >= 2^-41) that is at least 2^-149 even for a subnormal weight, so q is always
// an f32 and p + q is the exact product.  Factors outside [2^-41, 2^64) other than 0, and
// products that overflow, send a wavefront to the f64 path instead (callers check).
//
// Rounding is monotonic, so scores order like the pairs (p, q) taken lexicographically:
// with d = pa - pb and dq = qa - qb, both correctly signed, t = 4 d + dq has the sign of the
// difference of the exact scores (|dq| < 2 |d| whenever d != 0, and t = dq when d == 0).
//
// One thread holds G groups of M positions.  For every pair of positions the outcome in
// group g is bit g of one 32-bit word, so the logic that turns outcomes into keep flags runs
// on all of the thread's groups at once.
// ---------------------------------------------------------------------------
constexpr float kFactorScale = 0x1p+64f;
constexpr float kFactorMin = 0x1p-41f, kFactorMax = 0x1p+64f;   // nonzero factors the fast path takes: [min, max)

__device__ __forceinline__ bool factor_in_fast_range(float f)
{
    return f == 0.0f || (f >= kFactorMin && f < kFactorMax);
}

template <int M>
struct PairWords {
    uint32_t w[M * (M - 1) / 2];   // pair (a, b), a < b, in the order (0,1) (0,2) .. (M-2,M-1)
};

// Shift the outcomes of one more group into the pair words: the new bit 0 of pair (a, b) is
// set iff b's score is strictly greater than a's (on a tie the earlier position, a, ranks higher).
template <int M>
__device__ __forceinline__ void push_group(PairWords<M> &pw, const float *p, const float *q)
{
    int n = 0;
#pragma unroll
    for (int a = 0; a < M; ++a)
#pragma unroll
        for (int b = a + 1; b < M; ++b) {
            const float t = fmaf(p[a] - p[b], 4.0f, q[a] - q[b]);
            pw.w[n] = __builtin_amdgcn_alignbit(pw.w[n], __float_as_uint(t), 31);   // (w << 1) | sign(t)
            // Pin the word here: otherwise the compiler sinks every push below the caller's
            // range check and keeps all scores of the thread live until then.
            asm volatile("" : "+v"(pw.w[n]));
            ++n;
        }
}

__device__ __forceinline__ uint32_t majority3(uint32_t x, uint32_t y, uint32_t z)
{
    return (x & y) | (z & (x | y));
}

// keep[a]: bit g set iff position a of group g is among the M / 2 best of its group, i.e.
// ranks above at least M / 2 of the other M - 1 positions.  Bits above the thread's group
// count are garbage.
template <int M>
__device__ __forceinline__ void keep_words(const PairWords<M> &pw, uint32_t *keep)
{
    static_assert(M == 2 || M == 4 || M == 8, "patterns 1:2, 2:4 and 4:8");
    auto pair_index = [](int a, int b) { return a * (2 * M - a - 1) / 2 + (b - a - 1); };   // a < b
#pragma unroll
    for (int a = 0; a < M; ++a) {
        uint32_t x[M - 1];   // x[.]: a ranks above the other position
        int n = 0;
#pragma unroll
        for (int b = 0; b < a; ++b)
            x[n++] = pw.w[pair_index(b, a)];
#pragma unroll
        for (int b = a + 1; b < M; ++b)
            x[n++] = ~pw.w[pair_index(a, b)];
        if constexpr (M == 2) {
            keep[a] = x[0];
        } else if constexpr (M == 4) {
            keep[a] = majority3(x[0], x[1], x[2]);
        } else {
            // at least 4 of 7: carry-save adders; the weight-4 bit of the count is the answer
            const uint32_t s1 = x[0] ^ x[1] ^ x[2], c1 = majority3(x[0], x[1], x[2]);
            const uint32_t s2 = x[3] ^ x[4] ^ x[5], c2 = majority3(x[3], x[4], x[5]);
            const uint32_t c3 = majority3(s1, s2, x[6]);
            keep[a] = majority3(c1, c2, c3);
        }
    }
}

// ---------------------------------------------------------------------------
// The cut of a group: the M / 2-th largest leading term (`cut`), the next one below it in
// rank (`next`) and the largest (`top`), from min/max networks (no comparisons of pairs).
//
// Rounding is monotonic: s_a <= s_b for the exact scores implies p_a <= p_b for their leading
// terms.  So when next < cut strictly, the M / 2 positions with p >= cut are exactly the M / 2
// best by exact score and no two scores tie across the cut: the group is decided by M
// comparisons against `cut`, whatever the error terms and the indices are.  When next == cut
// the leading terms do not decide the group and the caller takes the exact pairwise path.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void sort2(float &lo, float &hi)
{
    const float a = __builtin_fminf(lo, hi), b = __builtin_fmaxf(lo, hi);
    lo = a;
    hi = b;
}
// ascending order of four
__device__ __forceinline__ void sort4(float &a, float &b, float &c, float &d)
{
    sort2(a, b);
    sort2(c, d);
    sort2(a, c);   // a: least of the four
    sort2(b, d);   // d: greatest
    sort2(b, c);
}
template <int M>
__device__ __forceinline__ void group_cut(const float *p, float &cut, float &next, float &top)
{
    static_assert(M == 2 || M == 4 || M == 8, "patterns 1:2, 2:4 and 4:8");
    if constexpr (M == 2) {
        cut = top = __builtin_fmaxf(p[0], p[1]);
        next = __builtin_fminf(p[0], p[1]);
    } else if constexpr (M == 4) {
        float a = p[0], b = p[1], c = p[2], d = p[3];
        sort2(a, b);
        sort2(c, d);
        top = __builtin_fmaxf(b, d);
        const float h = __builtin_fminf(b, d), l = __builtin_fmaxf(a, c);   // the two middle ones, in some order
        cut = __builtin_fmaxf(h, l);
        next = __builtin_fminf(h, l);
    } else {
        float a0 = p[0], a1 = p[1], a2 = p[2], a3 = p[3], b0 = p[4], b1 = p[5], b2 = p[6], b3 = p[7];
        sort4(a0, a1, a2, a3);
        sort4(b0, b1, b2, b3);
        top = __builtin_fmaxf(a3, b3);
        // a ascending followed by b descending is bitonic: element i against element i + 4 splits the
        // eight into the four largest (the maxima) and the four smallest (the minima)
        cut = __builtin_fminf(__builtin_fminf(__builtin_fmaxf(a0, b3), __builtin_fmaxf(a1, b2)),
                              __builtin_fminf(__builtin_fmaxf(a2, b1), __builtin_fmaxf(a3, b0)));
        next = __builtin_fmaxf(__builtin_fmaxf(__builtin_fminf(a0, b3), __builtin_fminf(a1, b2)),
                               __builtin_fmaxf(__builtin_fminf(a2, b1), __builtin_fminf(a3, b0)));
    }
}

// Two bf16 elements, each held as f32 bits with the low half clear, packed into one word:
// `lo` becomes the low half, `hi` the high half.
__device__ __forceinline__ uint32_t pack_bf16_pair(uint32_t lo, uint32_t hi)
{
    return (lo >> 16) | hi;
}

// All-ones if bit `bit` of `word` is set, else 0.
__device__ __forceinline__ uint32_t spread_bit(uint32_t word, int bit)
{
    return (uint32_t)__builtin_amdgcn_sbfe((int)word, bit, 1);
}

// 16-byte vector of raw words, the unit of every global access of stage 2.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

enum { kFactorOne = 0, kFactorNorm = 1, kFactorSqrt = 2 };

// f = norm^alpha for alpha = 0, 1, 0.5.  sqrtf is the correctly rounded f32 square root
// (this file is built without fast-math), which equals the f64 square root rounded to f32.
__device__ __forceinline__ float factor_of(float norm, int fmode)
{
    if (fmode == kFactorSqrt)
        return sqrtf(norm);
    return fmode == kFactorNorm ? norm : 1.0f;
}

template <int DT>
__device__ __forceinline__ float elem_of(const u32x4 &v, int e)   // element e of a 16-byte vector, as f32
{
    if constexpr (DT == DASS_BF16) {
        const uint32_t w = v[e >> 1];
        return __uint_as_float((e & 1) ? (w & 0xffff0000u) : (w << 16));
    } else {
        return __uint_as_float(v[e]);
    }
}

// Element e of a 16-byte vector becomes +0 when `drop` is set; plain mask arithmetic, no branch.
template <int DT>
__device__ __forceinline__ void zero_lane_if(u32x4 &v, int e, bool drop)
{
    if constexpr (DT == DASS_BF16)
        v[e >> 1] &= drop ? ((e & 1) ? 0x0000ffffu : 0xffff0000u) : 0xffffffffu;
    else
        v[e] &= drop ? 0u : 0xffffffffu;
}

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
