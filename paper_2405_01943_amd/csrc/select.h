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
