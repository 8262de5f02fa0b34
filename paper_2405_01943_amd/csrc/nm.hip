// Stage 2, N:M: score every weight as |W| * f (Sec. 3 Eq. 4 / Eq. 5), keep the
// n_keep best of every m consecutive positions along the group axis (Sec. 3
// "Extension to N:M Sparsity"), write +0 over the rest in place.
//
// One streaming pass: every weight is read once and written once with 16-byte
// accesses; selection happens in registers on exact scores.
//
// Two families of kernels:
//   nm_half_*   the patterns the paper uses, n_keep = m / 2 for m = 2, 4, 8, with
//               alpha in {0, 0.5, 1}: the factor is computed in the kernel; a group
//               is decided by its cut (the m / 2-th largest leading term, from a
//               min/max network) whenever the leading terms decide it, else by
//               pairwise comparison of exact two-term f32 scores, bit-sliced over
//               the thread's groups; accesses are non-temporal and every thread
//               makes a single pass (many small workgroups keep HBM busier than a
//               resident grid that loops).
//   nm_*        every other (n_keep, m, alpha): factor vector from a helper kernel,
//               scores as f64 products, selection by counting wins per lane.
#include "select.h"

#include <cstdio>
#include <vector>

#include <type_traits>

#include <mutex>

namespace dass {

constexpr int kBlock = 256;
constexpr int kHalfColsRows = 4;   // 16-byte vectors per thread of nm_half_cols_kernel

// ---------------------------------------------------------------------------
// n_keep = m / 2, factor computed in the kernel
// ---------------------------------------------------------------------------
// N factors at once from the norms at src[0..N): all loads are issued before the first use,
// and the exponent is tested once.  ok is cleared when a factor is outside the fast range;
// the factors come back scaled by kFactorScale.  VEC: src is 16-byte aligned and differs from
// lane to lane (16-byte loads); otherwise it is the same for the whole wavefront (scalar loads).
template <int N, bool VEC>
__device__ __forceinline__ void scaled_factors(const float *__restrict__ src, int fmode, float *f, bool &ok)
{
    float nrm[N];
    if constexpr (VEC) {
        static_assert(N % 4 == 0, "whole 16-byte vectors");
#pragma unroll
        for (int i = 0; i < N / 4; ++i) {
            const u32x4 q = *reinterpret_cast<const u32x4 *>(src + 4 * i);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                nrm[4 * i + k] = __uint_as_float(q[k]);
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i)
            nrm[i] = src[i];
    }
    if (fmode == kFactorSqrt) {
#pragma unroll
        for (int i = 0; i < N; ++i)
            f[i] = sqrtf(nrm[i]);
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i)
            f[i] = fmode == kFactorNorm ? nrm[i] : 1.0f;
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
        ok &= factor_in_fast_range(f[i]);
        f[i] *= kFactorScale;
    }
}

// |W[r, c]| straight from memory, and W[r, c] = +0: the element-wise accesses of the rare f64 path.
template <int DT>
__device__ __forceinline__ float abs_at(const char *W, int64_t r, int64_t c, int64_t ld)
{
    if constexpr (DT == DASS_BF16)
        return __uint_as_float(((uint32_t) * reinterpret_cast<const uint16_t *>(W + (r * ld + c) * 2) << 16) & 0x7fffffffu);
    else
        return __uint_as_float(*reinterpret_cast<const uint32_t *>(W + (r * ld + c) * 4) & 0x7fffffffu);
}
template <int DT>
__device__ __forceinline__ void zero_at(char *W, int64_t r, int64_t c, int64_t ld)
{
    if constexpr (DT == DASS_BF16)
        *reinterpret_cast<uint16_t *>(W + (r * ld + c) * 2) = 0;
    else
        *reinterpret_cast<uint32_t *>(W + (r * ld + c) * 4) = 0u;
}

// Groups run down a column (stride ld): Gate-Proj and Up-Proj.  A thread owns the EPV
// columns of one 16-byte vector and M rows (2 x M for M = 2): EPV (or 2 EPV) groups.  A
// workgroup covers up to 256 such column slots, so rows are read and written in contiguous
// pieces of up to 4 KB; every thread makes one pass and the grid covers the matrix (many small workgroups
// keep HBM busier than a resident grid that loops).
// (`bid`: the workgroup's number inside this matrix.)
template <int DT, int M, bool NORM_ROWS, bool WITH_MASK, bool CUT_FIRST>
__device__ __forceinline__ void nm_half_rows_body(
    void *__restrict__ Wv, int64_t rows, int64_t cols, int64_t ld, const float *__restrict__ norms,
    int fmode, uint8_t *__restrict__ mask, uint32_t nbx, uint32_t bid)
{
    constexpr int EPV = DT == DASS_BF16 ? 8 : 4;
    constexpr int GB = M >= 4 ? 1 : 2;   // row groups per thread
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;

    const int64_t bx = bid % nbx, by = bid / nbx;   // 32-bit division
    const int64_t slot = bx * blockDim.x + threadIdx.x;
    // Lanes past the last column slot leave.  (With f32 two neighbouring lanes share a mask byte
    // and exchange their halves at the end; cols is a multiple of 8, so they leave or stay together.)
    if (slot >= cols / EPV)
        return;
    constexpr bool active = true;
    const int64_t c0 = slot * EPV;
    const int64_t n_groups = rows / M;
    char *W = static_cast<char *>(Wv);

    u32x4 v[GB][M];
#pragma unroll
    for (int g = 0; g < GB; ++g)
        if (by * GB + g < n_groups) {
#pragma unroll
            for (int a = 0; a < M; ++a)
                v[g][a] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4 *>(W + (((by * GB + g) * M + a) * ld + c0) * EB));
        }

    bool fast_ok = true;
    float fc[EPV];   // scaled factors of the thread's columns, or ...
    if constexpr (!NORM_ROWS)
        scaled_factors<EPV, true>(norms + c0, fmode, fc, fast_ok);   // c0 is a multiple of 4: 16-byte loads

#pragma unroll
    for (int g = 0; g < GB; ++g) {
        if (by * GB + g >= n_groups)
            break;
        const int64_t r0 = (by * GB + g) * M;
        float fr[M];   // ... of the group's rows
        if constexpr (NORM_ROWS)
            scaled_factors<M, false>(norms + r0, fmode, fr, fast_ok);

        if constexpr (CUT_FIRST) {
            // Every column's group against its cut (select.h): M comparisons instead of M (M - 1) / 2
            // pairs, the result written over the weights in their registers.  A wavefront in which some
            // group is not decided by its leading terms, or some product left the f32 range, fetches
            // its weights again (memory still holds them) and takes the pairwise code below.
            uint32_t kept_cols[M];
#pragma unroll
            for (int a = 0; a < M; ++a)
                kept_cols[a] = 0;
            bool undecided = false;
            float top_all = 0.0f;
            constexpr int EPW = DT == DASS_BF16 ? 2 : 1;   // elements per 32-bit word
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t part[EPW][M];
#pragma unroll
                for (int h = 0; h < EPW; ++h) {
                    const int e = j * EPW + h;
                    float x[M], p[M];
#pragma unroll
                    for (int a = 0; a < M; ++a) {
                        x[a] = elem_of<DT>(v[g][a], e);
                        p[a] = fabsf(x[a]) * (NORM_ROWS ? fr[a] : fc[e]);
                    }
                    float cut, next, top;
                    group_cut<M>(p, cut, next, top);
                    undecided |= next == cut;
                    top_all = fmaxf(top_all, top);
#pragma unroll
                    for (int a = 0; a < M; ++a) {
                        const bool keep = p[a] >= cut;
                        part[h][a] = keep ? __float_as_uint(x[a]) : 0u;
                        if constexpr (WITH_MASK)
                            kept_cols[a] |= keep ? 1u << e : 0u;
                    }
                }
#pragma unroll
                for (int a = 0; a < M; ++a) {
                    if constexpr (DT == DASS_BF16)
                        v[g][a][j] = pack_bf16_pair(part[0][a], part[1][a]);
                    else
                        v[g][a][j] = part[0][a];
                }
                __builtin_amdgcn_sched_barrier(0);   // one word of columns at a time keeps the register count down
            }
            if (__builtin_amdgcn_ballot_w64(undecided || !fast_ok || !(top_all < INFINITY)) == 0) {
#pragma unroll
                for (int a = 0; a < M; ++a) {
                    __builtin_nontemporal_store(v[g][a], reinterpret_cast<u32x4 *>(W + ((r0 + a) * ld + c0) * EB));
                    if constexpr (WITH_MASK) {
                        if constexpr (EPV == 8) {
                            mask[(r0 + a) * (cols / 8) + slot] = (uint8_t)kept_cols[a];
                        } else {   // two lanes share a byte: the even lane writes both halves
                            const uint32_t other = __shfl_xor(kept_cols[a], 1, 64);
                            if ((slot & 1) == 0)
                                mask[(r0 + a) * (cols / 8) + slot / 2] = (uint8_t)(kept_cols[a] | (other << 4));
                        }
                    }
                }
                continue;
            }
#pragma unroll
            for (int a = 0; a < M; ++a)
                v[g][a] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(W + ((r0 + a) * ld + c0) * EB));
        }

        // Outcomes of all pairs of rows, one bit per column (column e ends up in bit e).
        PairWords<M> pw;
        float pmax = 0.0f;
#pragma unroll
        for (int e = EPV - 1; e >= 0; --e) {
            float p[M], q[M];
#pragma unroll
            for (int a = 0; a < M; ++a) {
                const float w = fabsf(elem_of<DT>(v[g][a], e)), f = NORM_ROWS ? fr[a] : fc[e];
                p[a] = w * f;
                q[a] = fmaf(w, f, -p[a]);
                pmax = fmaxf(pmax, p[a]);
            }
            push_group<M>(pw, p, q);
            __builtin_amdgcn_sched_barrier(0);   // one column at a time keeps the register count down
        }
        uint32_t keep[M];
        keep_words<M>(pw, keep);

        // A factor outside the fast range or a product that overflowed (in any lane): the
        // whole wavefront redoes its groups element by element on the weights still in memory,
        // with f64 products, which are exact over the whole f32 range, and writes the zeros itself.
        const bool exact_path = __builtin_amdgcn_ballot_w64(!fast_ok || !(pmax < INFINITY)) != 0;
        if (exact_path) {
#pragma unroll
            for (int a = 0; a < M; ++a)
                keep[a] = 0;
#pragma unroll 1
            for (int e = 0; e < EPV; ++e) {
                double sc[M];
#pragma unroll
                for (int a = 0; a < M; ++a)
                    sc[a] = (double)abs_at<DT>(W, r0 + a, c0 + e, ld) *
                            (double)factor_of(norms[NORM_ROWS ? r0 + a : c0 + e], fmode);
                const uint32_t bits = nm_keep_bits<M>(sc, M / 2);
#pragma unroll
                for (int a = 0; a < M; ++a) {
                    if (active && !((bits >> a) & 1u))
                        zero_at<DT>(W, r0 + a, c0 + e, ld);
                    keep[a] |= ((bits >> a) & 1u) << e;
                }
            }
        } else {
#pragma unroll
            for (int a = 0; a < M; ++a) {
                if constexpr (DT == DASS_BF16) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t lo = spread_bit(keep[a], 2 * j), hi = spread_bit(keep[a], 2 * j + 1);
                        v[g][a][j] &= (lo & 0x0000ffffu) | (hi & 0xffff0000u);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        v[g][a][j] &= spread_bit(keep[a], j);
                }
                if (active)
                    __builtin_nontemporal_store(v[g][a], reinterpret_cast<u32x4 *>(W + ((r0 + a) * ld + c0) * EB));
            }
        }
        if constexpr (WITH_MASK) {
#pragma unroll
            for (int a = 0; a < M; ++a) {
                const uint32_t kept = keep[a] & ((1u << EPV) - 1u);
                if constexpr (EPV == 8) {
                    if (active)
                        mask[(r0 + a) * (cols / 8) + slot] = (uint8_t)kept;
                } else {   // two lanes share a byte: the even lane writes both halves
                    const uint32_t other = __shfl_xor(kept, 1, 64);
                    if (active && (slot & 1) == 0)
                        mask[(r0 + a) * (cols / 8) + slot / 2] = (uint8_t)(kept | (other << 4));
                }
            }
        }
    }
}

// Groups run along a row (contiguous): Down-Proj.  A thread owns the UW = max(EPV, M)
// consecutive columns of NV 16-byte vectors and RB rows, RB * UW / M groups; the factors of
// its columns are computed once.
template <int DT, int M, bool NORM_COLS, bool WITH_MASK, bool CUT_FIRST>
__device__ __forceinline__ void nm_half_cols_body(
    void *__restrict__ Wv, int64_t rows, int64_t cols, int64_t ld, const float *__restrict__ norms,
    int fmode, uint8_t *__restrict__ mask, uint32_t nbx, uint32_t bid)
{
    constexpr int EPV = DT == DASS_BF16 ? 8 : 4;
    constexpr int UW = M > EPV ? M : EPV;
    constexpr int NV = UW / EPV;
    constexpr int RB = kHalfColsRows / NV;
    constexpr int GPR = UW / M;   // groups per row
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;

    const int64_t bx = bid % nbx, by = bid / nbx;   // 32-bit division
    const int64_t slot = bx * blockDim.x + threadIdx.x;
    // Lanes past the last column slot read column 0 and write nothing.  (Measured: letting them
    // leave early instead makes this kernel slower.)
    const bool active = slot < cols / UW;
    const int64_t c0 = (active ? slot : 0) * UW;
    char *W = static_cast<char *>(Wv);

    u32x4 v[RB][NV];
#pragma unroll
    for (int k = 0; k < RB; ++k)
        if (by * RB + k < rows) {
#pragma unroll
            for (int j = 0; j < NV; ++j)
                v[k][j] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4 *>(W + ((by * RB + k) * ld + c0) * EB + 16 * j));
        }

    bool fast_ok = true;
    float fc[UW];
    if constexpr (NORM_COLS)
        scaled_factors<UW, true>(norms + c0, fmode, fc, fast_ok);   // c0 is a multiple of 4: 16-byte loads
    float frow[RB];
    if constexpr (!NORM_COLS) {   // rows past the end (last batch only) reuse the last row's norm
#pragma unroll
        for (int k = 0; k < RB; ++k)
            scaled_factors<1, false>(norms + (by * RB + k < rows ? by * RB + k : rows - 1), fmode, frow + k, fast_ok);
    }

    if constexpr (CUT_FIRST) {
        // Every group against its cut, as in nm_half_rows_body: the result overwrites the weights in
        // their registers and is stored only if every group of the wavefront was decided by its
        // leading terms; otherwise the weights are fetched again.
        uint32_t kept_row[RB];
        bool undecided = false;
        float top_all = 0.0f;
        const int rows_here = rows - by * RB < RB ? (int)(rows - by * RB) : RB;   // uniform in the workgroup
#pragma unroll
        for (int k = 0; k < RB; ++k) {
            kept_row[k] = 0;
            if (k >= rows_here)
                break;
            const float fr = NORM_COLS ? 0.0f : frow[k];
            uint32_t part[UW];
#pragma unroll
            for (int g = 0; g < GPR; ++g) {
                float x[M], p[M];
#pragma unroll
                for (int a = 0; a < M; ++a) {
                    const int e = g * M + a;
                    x[a] = elem_of<DT>(v[k][e / EPV], e % EPV);
                    p[a] = fabsf(x[a]) * (NORM_COLS ? fc[e] : fr);
                }
                float cut, next, top;
                group_cut<M>(p, cut, next, top);
                undecided |= next == cut;
                top_all = fmaxf(top_all, top);
#pragma unroll
                for (int a = 0; a < M; ++a) {
                    const bool keep = p[a] >= cut;
                    part[g * M + a] = keep ? __float_as_uint(x[a]) : 0u;
                    if constexpr (WITH_MASK)
                        kept_row[k] |= keep ? 1u << (g * M + a) : 0u;
                }
                __builtin_amdgcn_sched_barrier(0);   // one group at a time keeps the register count down
            }
#pragma unroll
            for (int j = 0; j < NV; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if constexpr (DT == DASS_BF16)
                        v[k][j][i] = pack_bf16_pair(part[j * 8 + 2 * i], part[j * 8 + 2 * i + 1]);
                    else
                        v[k][j][i] = part[j * 4 + i];
                }
        }
        if (__builtin_amdgcn_ballot_w64(undecided || !fast_ok || !(top_all < INFINITY)) == 0) {
#pragma unroll
            for (int k = 0; k < RB; ++k) {
                if (k >= rows_here)
                    break;
                const int64_t r = by * RB + k;
                if (active) {
#pragma unroll
                    for (int j = 0; j < NV; ++j)
                        __builtin_nontemporal_store(v[k][j], reinterpret_cast<u32x4 *>(W + (r * ld + c0) * EB + 16 * j));
                }
                if constexpr (WITH_MASK) {
                    if constexpr (UW >= 8) {
                        if (active) {
#pragma unroll
                            for (int b = 0; b < UW / 8; ++b)
                                mask[r * (cols / 8) + c0 / 8 + b] = (uint8_t)(kept_row[k] >> (8 * b));
                        }
                    } else {
                        const uint32_t other = __shfl_xor(kept_row[k], 1, 64);
                        if (active && (slot & 1) == 0)
                            mask[r * (cols / 8) + slot / 2] = (uint8_t)(kept_row[k] | (other << 4));
                    }
                }
            }
            return;
        }
#pragma unroll
        for (int k = 0; k < RB; ++k)
            if (k < rows_here) {
#pragma unroll
                for (int j = 0; j < NV; ++j)
                    v[k][j] = __builtin_nontemporal_load(
                        reinterpret_cast<const u32x4 *>(W + ((by * RB + k) * ld + c0) * EB + 16 * j));
            }
    }

    // Outcomes of all pairs of positions; group g of row k ends up in bit k * GPR + g.
    PairWords<M> pw;
    float pmax = 0.0f;
#pragma unroll
    for (int k = RB - 1; k >= 0; --k) {
        const float fr = NORM_COLS ? 0.0f : frow[k];
#pragma unroll
        for (int g = GPR - 1; g >= 0; --g) {
            float p[M], q[M];
#pragma unroll
            for (int a = 0; a < M; ++a) {
                const int e = g * M + a;
                const float w = fabsf(elem_of<DT>(v[k][e / EPV], e % EPV)), f = NORM_COLS ? fc[e] : fr;
                p[a] = w * f;
                q[a] = fmaf(w, f, -p[a]);
                pmax = fmaxf(pmax, p[a]);
            }
            push_group<M>(pw, p, q);
            __builtin_amdgcn_sched_barrier(0);   // one group at a time keeps the register count down
        }
    }
    uint32_t keep[M];
    keep_words<M>(pw, keep);

    // as in nm_half_rows_kernel
    const bool exact_path = __builtin_amdgcn_ballot_w64(!fast_ok || !(pmax < INFINITY)) != 0;
#pragma unroll
    for (int k = 0; k < RB; ++k) {
        const int64_t r = by * RB + k;
        if (r >= rows)
            break;
        uint32_t kept = 0;   // keep flags of the row's UW columns
        if (exact_path) {
#pragma unroll 1
            for (int g = 0; g < GPR; ++g) {
                double sc[M];
#pragma unroll
                for (int a = 0; a < M; ++a)
                    sc[a] = (double)abs_at<DT>(W, r, c0 + g * M + a, ld) *
                            (double)factor_of(norms[NORM_COLS ? c0 + g * M + a : r], fmode);
                const uint32_t bits = nm_keep_bits<M>(sc, M / 2);
#pragma unroll
                for (int a = 0; a < M; ++a)
                    if (active && !((bits >> a) & 1u))
                        zero_at<DT>(W, r, c0 + g * M + a, ld);
                kept |= bits << (g * M);
            }
        } else {
            uint32_t m[UW];   // all-ones where column e of the row is kept
#pragma unroll
            for (int e = 0; e < UW; ++e)
                m[e] = spread_bit(keep[e % M], k * GPR + e / M);
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                if constexpr (DT == DASS_BF16) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        v[k][j][i] &= (m[j * 8 + 2 * i] & 0x0000ffffu) | (m[j * 8 + 2 * i + 1] & 0xffff0000u);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        v[k][j][i] &= m[j * 4 + i];
                }
                if (active)
                    __builtin_nontemporal_store(v[k][j], reinterpret_cast<u32x4 *>(W + (r * ld + c0) * EB + 16 * j));
            }
            if constexpr (WITH_MASK) {
#pragma unroll
                for (int e = 0; e < UW; ++e)
                    kept |= m[e] & (1u << e);
            }
        }
        if constexpr (WITH_MASK) {
            if constexpr (UW >= 8) {
                if (active) {
#pragma unroll
                    for (int b = 0; b < UW / 8; ++b)
                        mask[r * (cols / 8) + c0 / 8 + b] = (uint8_t)(kept >> (8 * b));
                }
            } else {
                const uint32_t other = __shfl_xor(kept, 1, 64);
                if (active && (slot & 1) == 0)
                    mask[r * (cols / 8) + slot / 2] = (uint8_t)(kept | (other << 4));
            }
        }
    }
}

// ===========================================================================
// General path: any (n_keep, m, alpha)
// ===========================================================================

// One matrix per launch.
template <int DT, int M, bool NORM_ROWS, bool WITH_MASK, bool CUT_FIRST>
__global__ __launch_bounds__(kBlock) void nm_half_rows_kernel(
    void *__restrict__ Wv, int64_t rows, int64_t cols, int64_t ld, const float *__restrict__ norms,
    int fmode, uint8_t *__restrict__ mask, uint32_t nbx)
{
    nm_half_rows_body<DT, M, NORM_ROWS, WITH_MASK, CUT_FIRST>(Wv, rows, cols, ld, norms, fmode, mask, nbx,
                                                               blockIdx.x);
}
template <int DT, int M, bool NORM_COLS, bool WITH_MASK, bool CUT_FIRST>
__global__ __launch_bounds__(kBlock) void nm_half_cols_kernel(
    void *__restrict__ Wv, int64_t rows, int64_t cols, int64_t ld, const float *__restrict__ norms,
    int fmode, uint8_t *__restrict__ mask, uint32_t nbx)
{
    nm_half_cols_body<DT, M, NORM_COLS, WITH_MASK, CUT_FIRST>(Wv, rows, cols, ld, norms, fmode, mask, nbx,
                                                               blockIdx.x);
}

// Many matrices of one shape per launch (the layers of a model): the table travels in the
// kernel arguments, a workgroup finds its matrix by one division.  The launch gaps that separate
// single-matrix kernels of ~30 us disappear.
constexpr int kBatchMax = 96;
struct NmBatch {
    void *W[kBatchMax];
    const float *norms[kBatchMax];
    uint8_t *mask[kBatchMax];   // all null unless WITH_MASK
    int64_t rows, cols, ld;
    int fmode;
    uint32_t nbx, blocks_per_matrix;
};
template <int DT, int M, bool GROUPS_DOWN_ROWS, bool NORM_ALONG, bool WITH_MASK, bool CUT_FIRST>
__global__ __launch_bounds__(kBlock) void nm_half_batched_kernel(const NmBatch b)
{
    const uint32_t k = blockIdx.x / b.blocks_per_matrix, bid = blockIdx.x - k * b.blocks_per_matrix;
    if constexpr (GROUPS_DOWN_ROWS)
        nm_half_rows_body<DT, M, NORM_ALONG, WITH_MASK, CUT_FIRST>(b.W[k], b.rows, b.cols, b.ld, b.norms[k], b.fmode,
                                                                    WITH_MASK ? b.mask[k] : nullptr, b.nbx, bid);
    else
        nm_half_cols_body<DT, M, NORM_ALONG, WITH_MASK, CUT_FIRST>(b.W[k], b.rows, b.cols, b.ld, b.norms[k], b.fmode,
                                                                    WITH_MASK ? b.mask[k] : nullptr, b.nbx, bid);
}

// ---------------------------------------------------------------------------
// Groups run along a row (contiguous in memory): Down-Proj.
// A thread owns UW = max(8, M) consecutive columns and walks down rows, so the
// factors of its columns are loaded once.  Rows are taken RB at a time so RB
// 16-byte loads per thread are in flight before the first is used.
// ---------------------------------------------------------------------------
template <int DT, int M, bool NORM_COLS>
__global__ __launch_bounds__(kBlock) void nm_cols_kernel(
    void *__restrict__ Wv, int64_t rows, int64_t cols, int64_t ld, const float *__restrict__ f,
    int min_wins, uint8_t *__restrict__ mask, int64_t nbx, int64_t nby)
{
    constexpr int UW = M > 8 ? M : 8;
    constexpr int NW = words_for<DT>(UW);  // words per thread per row
    constexpr int NV = NW / 4;             // 16-byte vectors per thread per row
    constexpr int RB = 4;
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;

    const int64_t bx = blockIdx.x % nbx, by = blockIdx.x / nbx;
    const int64_t slot = bx * kBlock + threadIdx.x;
    if (slot >= cols / UW)
        return;
    const int64_t c0 = slot * UW;
    char *W = static_cast<char *>(Wv);

    double fc[UW];
    if constexpr (NORM_COLS) {
#pragma unroll
        for (int v = 0; v < UW / 4; ++v) {
            const Vec16 q = load16(f + c0 + 4 * v);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                fc[4 * v + k] = (double)__uint_as_float(q.w[k]);
        }
    }

    for (int64_t rb = by * RB; rb < rows; rb += nby * RB) {
        uint32_t words[RB][NW];
#pragma unroll
        for (int k = 0; k < RB; ++k) {
            if (rb + k < rows) {
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const Vec16 q = load16(W + ((rb + k) * ld + c0) * EB + 16 * v);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        words[k][4 * v + j] = q.w[j];
                }
            }
        }
#pragma unroll
        for (int k = 0; k < RB; ++k) {
            if (rb + k < rows) {
                double fr = 0.0;
                if constexpr (!NORM_COLS)
                    fr = (double)f[rb + k];
                uint32_t kept = 0;
#pragma unroll
                for (int g = 0; g < UW / M; ++g) {
                    double s[M];
#pragma unroll
                    for (int a = 0; a < M; ++a)
                        s[a] = (double)abs_elem<DT>(words[k], g * M + a) *
                               (NORM_COLS ? fc[g * M + a] : fr);
                    const uint32_t bits = nm_keep_bits<M>(s, min_wins);
#pragma unroll
                    for (int a = 0; a < M; ++a)
                        if (!((bits >> a) & 1u))
                            zero_elem<DT>(words[k], g * M + a);
                    kept |= bits << (g * M);
                }
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    Vec16 q;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        q.w[j] = words[k][4 * v + j];
                    store16(W + ((rb + k) * ld + c0) * EB + 16 * v, q);
                }
                if (mask) {
#pragma unroll
                    for (int b = 0; b < UW / 8; ++b)
                        mask[(rb + k) * (cols / 8) + c0 / 8 + b] = (uint8_t)(kept >> (8 * b));
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Groups run down a column (stride ld): Gate-Proj and Up-Proj.
// A thread owns 8 consecutive columns and takes GB row-groups (GB * M rows) at a
// time; each row is one 16-byte access per 8 bf16 columns, contiguous across the
// lanes of a wavefront.  With the factor per row (DaSS), all lanes of a
// wavefront read the same M factors.
// ---------------------------------------------------------------------------
template <int DT, int M, bool NORM_ROWS>
__global__ __launch_bounds__(kBlock) void nm_rows_kernel(
    void *__restrict__ Wv, int64_t rows, int64_t cols, int64_t ld, const float *__restrict__ f,
    int min_wins, uint8_t *__restrict__ mask, int64_t nbx, int64_t nby)
{
    constexpr int NW = words_for<DT>(8);
    constexpr int NV = NW / 4;
    constexpr int GB = M >= 8 ? 1 : 8 / M;
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;

    const int64_t bx = blockIdx.x % nbx, by = blockIdx.x / nbx;
    const int64_t slot = bx * kBlock + threadIdx.x;
    if (slot >= cols / 8)
        return;
    const int64_t c0 = slot * 8;
    const int64_t n_groups = rows / M;
    char *W = static_cast<char *>(Wv);

    double fc[8];
    if constexpr (!NORM_ROWS) {
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            const Vec16 q = load16(f + c0 + 4 * v);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                fc[4 * v + k] = (double)__uint_as_float(q.w[k]);
        }
    }

    for (int64_t gb = by * GB; gb < n_groups; gb += nby * GB) {
        uint32_t words[GB][M][NW];
#pragma unroll
        for (int g = 0; g < GB; ++g) {
            if (gb + g < n_groups) {
#pragma unroll
                for (int a = 0; a < M; ++a) {
                    const int64_t r = (gb + g) * M + a;
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const Vec16 q = load16(W + (r * ld + c0) * EB + 16 * v);
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            words[g][a][4 * v + j] = q.w[j];
                    }
                }
            }
        }
#pragma unroll
        for (int g = 0; g < GB; ++g) {
            if (gb + g < n_groups) {
                const int64_t r0 = (gb + g) * M;
                double fr[M];
                if constexpr (NORM_ROWS) {
#pragma unroll
                    for (int a = 0; a < M; ++a)
                        fr[a] = (double)f[r0 + a];
                }
                uint32_t kept[M];
#pragma unroll
                for (int a = 0; a < M; ++a)
                    kept[a] = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    double s[M];
#pragma unroll
                    for (int a = 0; a < M; ++a)
                        s[a] = (double)abs_elem<DT>(words[g][a], e) * (NORM_ROWS ? fr[a] : fc[e]);
                    const uint32_t bits = nm_keep_bits<M>(s, min_wins);
#pragma unroll
                    for (int a = 0; a < M; ++a) {
                        if (!((bits >> a) & 1u))
                            zero_elem<DT>(words[g][a], e);
                        kept[a] |= ((bits >> a) & 1u) << e;
                    }
                }
#pragma unroll
                for (int a = 0; a < M; ++a) {
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        Vec16 q;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            q.w[j] = words[g][a][4 * v + j];
                        store16(W + ((r0 + a) * ld + c0) * EB + 16 * v, q);
                    }
                    if (mask)
                        mask[(r0 + a) * (cols / 8) + slot] = (uint8_t)kept[a];
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------

// Blocks of `kernel` that fit on the device at once (CUs x blocks per CU).
static int64_t resident_blocks(const void *kernel)
{
    static std::mutex mu;
    static int n_cu = 0;
    std::lock_guard<std::mutex> lock(mu);
    if (n_cu == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
            return 0;
        n_cu = prop.multiProcessorCount;
    }
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kBlock, 0) != hipSuccess ||
        per_cu <= 0)
        return 0;
    return (int64_t)n_cu * per_cu;
}

using nm_kernel_t = void (*)(void *, int64_t, int64_t, int64_t, const float *, int, uint8_t *,
                             int64_t, int64_t);

template <int DT, int M>
static nm_kernel_t pick_kernel(int group_axis, int norm_axis)
{
    if (group_axis == DASS_AXIS_COLS)
        return norm_axis == DASS_AXIS_COLS ? nm_cols_kernel<DT, M, true>
                                           : nm_cols_kernel<DT, M, false>;
    return norm_axis == DASS_AXIS_ROWS ? nm_rows_kernel<DT, M, true>
                                       : nm_rows_kernel<DT, M, false>;
}

template <int DT>
static nm_kernel_t pick_kernel_m(int m, int group_axis, int norm_axis)
{
    switch (m) {
    case 2: return pick_kernel<DT, 2>(group_axis, norm_axis);
    case 4: return pick_kernel<DT, 4>(group_axis, norm_axis);
    case 8: return pick_kernel<DT, 8>(group_axis, norm_axis);
    case 16: return pick_kernel<DT, 16>(group_axis, norm_axis);
    }
    return nullptr;
}

using nm_half_kernel_t = void (*)(void *, int64_t, int64_t, int64_t, const float *, int, uint8_t *,
                                  uint32_t);

// When the factor varies inside a group (it runs along the group axis and alpha is not 0: the
// DaSS configuration) two leading terms of a group are almost never equal, and the kernels decide
// every group by its cut first (CUT_FIRST, select.h): M comparisons per group where the pairwise
// form needs M (M - 1) / 2, which at 8 positions per group is the difference between a kernel
// bound by memory and one bound by its arithmetic.  A factor that is constant inside the groups
// (magnitude pruning, groups across the norm axis) leaves bf16 magnitudes to tie at the cut all
// the time; those kernels compare pairs with both score terms straight away.
template <int DT, int M, bool WITH_MASK>
static nm_half_kernel_t pick_half_kernel(int group_axis, int norm_axis, bool varying_factor)
{
    if (varying_factor)
        return group_axis == DASS_AXIS_COLS ? nm_half_cols_kernel<DT, M, true, WITH_MASK, true>
                                            : nm_half_rows_kernel<DT, M, true, WITH_MASK, true>;
    if (group_axis == DASS_AXIS_COLS)
        return norm_axis == DASS_AXIS_COLS ? nm_half_cols_kernel<DT, M, true, WITH_MASK, false>
                                           : nm_half_cols_kernel<DT, M, false, WITH_MASK, false>;
    return norm_axis == DASS_AXIS_ROWS ? nm_half_rows_kernel<DT, M, true, WITH_MASK, false>
                                       : nm_half_rows_kernel<DT, M, false, WITH_MASK, false>;
}

template <int DT, bool WITH_MASK>
static nm_half_kernel_t pick_half_kernel_m(int m, int group_axis, int norm_axis, bool varying_factor)
{
    switch (m) {
    case 2: return pick_half_kernel<DT, 2, WITH_MASK>(group_axis, norm_axis, varying_factor);
    case 4: return pick_half_kernel<DT, 4, WITH_MASK>(group_axis, norm_axis, varying_factor);
    case 8: return pick_half_kernel<DT, 8, WITH_MASK>(group_axis, norm_axis, varying_factor);
    }
    return nullptr;
}

template <int DT>
static nm_half_kernel_t pick_half_kernel_mask(bool with_mask, int m, int group_axis, int norm_axis,
                                              bool varying_factor)
{
    return with_mask ? pick_half_kernel_m<DT, true>(m, group_axis, norm_axis, varying_factor)
                     : pick_half_kernel_m<DT, false>(m, group_axis, norm_axis, varying_factor);
}

using nm_batched_kernel_t = void (*)(const NmBatch);

template <int DT, int M, bool WITH_MASK>
static nm_batched_kernel_t pick_batched_kernel(int group_axis, int norm_axis, bool varying_factor)
{
    const bool down_rows = group_axis == DASS_AXIS_ROWS, along = norm_axis == group_axis;
    if (varying_factor)   // see pick_half_kernel
        return down_rows ? nm_half_batched_kernel<DT, M, true, true, WITH_MASK, true>
                         : nm_half_batched_kernel<DT, M, false, true, WITH_MASK, true>;
    if (down_rows)
        return along ? nm_half_batched_kernel<DT, M, true, true, WITH_MASK, false>
                     : nm_half_batched_kernel<DT, M, true, false, WITH_MASK, false>;
    return along ? nm_half_batched_kernel<DT, M, false, true, WITH_MASK, false>
                 : nm_half_batched_kernel<DT, M, false, false, WITH_MASK, false>;
}

template <int DT, bool WITH_MASK>
static nm_batched_kernel_t pick_batched_kernel_m(int m, int group_axis, int norm_axis, bool varying_factor)
{
    switch (m) {
    case 2: return pick_batched_kernel<DT, 2, WITH_MASK>(group_axis, norm_axis, varying_factor);
    case 4: return pick_batched_kernel<DT, 4, WITH_MASK>(group_axis, norm_axis, varying_factor);
    case 8: return pick_batched_kernel<DT, 8, WITH_MASK>(group_axis, norm_axis, varying_factor);
    }
    return nullptr;
}

// Launch geometry of the one-pass kernels: one thread per (column slot, row batch), no loop.
struct HalfGeometry {
    int block;
    int64_t nbx, batches;
};
static HalfGeometry half_geometry(int64_t rows, int64_t cols, int dt, int group_axis, int m)
{
    const int epv = vec_elems(dt);
    int64_t slots, batches;
    if (group_axis == DASS_AXIS_COLS) {
        const int uw = m > epv ? m : epv, rb = kHalfColsRows / (uw / epv);
        slots = cols / uw;
        batches = (rows + rb - 1) / rb;
    } else {
        slots = cols / epv;
        const int gb = m >= 4 ? 1 : 2;
        batches = (rows / m + gb - 1) / gb;
    }
    // Workgroup width: the widest of 256, 128, 64 that leaves the fewest idle lanes in the
    // last workgroup of a row (e.g. 1376 slots: 6 x 256 idles 10 %, 11 x 128 only 2 %).
    int block = kBlock;
    for (int cand = kBlock / 2; cand >= 64; cand /= 2)
        if ((slots + cand - 1) / cand * cand < (slots + block - 1) / block * block)
            block = cand;
    return {block, (slots + block - 1) / block, batches};
}

static bool half_path(double alpha, int n_keep, int m)
{
    return 2 * n_keep == m && m <= 8 && (alpha == 0.0 || alpha == 0.5 || alpha == 1.0);
}

}  // namespace dass

extern "C" size_t dass_nm_workspace_bytes(int64_t rows, int64_t cols, dass_axis norm_axis)
{
    const int64_t n = norm_axis == DASS_AXIS_ROWS ? rows : cols;
    return n > 0 ? dass::round_up((size_t)n * sizeof(float), 256) : 0;
}

namespace dass {
static dass_status check_nm_args(const char *fn, void *W, int64_t rows, int64_t cols, int64_t ld, int dt,
                                 const float *norms, int norm_axis, int group_axis, double alpha, int n_keep,
                                 int m, void *workspace, size_t workspace_bytes)
{
    dass_status st = check_score_args(fn, W, rows, cols, ld, dt, norms, norm_axis, group_axis, alpha,
                                      workspace, workspace_bytes,
                                      dass_nm_workspace_bytes(rows, cols, (dass_axis)norm_axis));
    if (st != DASS_OK)
        return st;
    if (!(m == 2 || m == 4 || m == 8 || m == 16))
        return fail(DASS_ERR_ARG, "%s: m=%d must be 2, 4, 8 or 16", fn, m);
    if (n_keep <= 0 || n_keep >= m)
        return fail(DASS_ERR_ARG, "%s: need 0 < n_keep < m, got %d:%d", fn, n_keep, m);
    const int64_t len = group_axis == DASS_AXIS_ROWS ? rows : cols;
    if (len % m != 0)
        return fail(DASS_ERR_SHAPE, "%s: group axis length %lld is not a multiple of m=%d", fn,
                    (long long)len, m);
    return DASS_OK;
}
}  // namespace dass

extern "C" dass_status dass_score_mask_nm(void *W, int64_t rows, int64_t cols, int64_t ld,
                                          dass_dtype dt, const float *norms, dass_axis norm_axis,
                                          dass_axis group_axis, double alpha, int n_keep, int m,
                                          uint8_t *mask_out, void *workspace,
                                          size_t workspace_bytes, void *hip_stream)
{
    using namespace dass;
    const char *fn = "dass_score_mask_nm";
    dass_status st = check_nm_args(fn, W, rows, cols, ld, dt, norms, norm_axis, group_axis, alpha, n_keep, m,
                                   workspace, workspace_bytes);
    if (st != DASS_OK)
        return st;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    // The paper's patterns with an exponent whose factor has an exact f32 recipe: one kernel.
    if (half_path(alpha, n_keep, m)) {
        const int fmode = alpha == 0.0 ? kFactorOne : alpha == 1.0 ? kFactorNorm : kFactorSqrt;
        const bool varying = norm_axis == group_axis && alpha != 0.0;
        nm_half_kernel_t kernel =
            dt == DASS_BF16 ? pick_half_kernel_mask<DASS_BF16>(mask_out != nullptr, m, group_axis, norm_axis, varying)
                            : pick_half_kernel_mask<DASS_F32>(mask_out != nullptr, m, group_axis, norm_axis, varying);
        const HalfGeometry g = half_geometry(rows, cols, dt, group_axis, m);
        const int block = g.block;
        const int64_t nbx = g.nbx, batches = g.batches;
        if (nbx * batches > 0x7fffffffLL)
            return fail(DASS_ERR_SHAPE, "%s: matrix too large for one launch", fn);
        hipLaunchKernelGGL(kernel, dim3((unsigned)(nbx * batches)), dim3(block), 0, stream, W, rows, cols, ld,
                           norms, fmode, mask_out, (uint32_t)nbx);
        return check_launch("N:M kernel");
    }

    float *f = static_cast<float *>(workspace);
    const int64_t n_norm = norm_axis == DASS_AXIS_ROWS ? rows : cols;
    st = launch_factor(norms, n_norm, alpha, f, stream);
    if (st != DASS_OK)
        return st;

    nm_kernel_t kernel = dt == DASS_BF16 ? pick_kernel_m<DASS_BF16>(m, group_axis, norm_axis)
                                         : pick_kernel_m<DASS_F32>(m, group_axis, norm_axis);
    // Work items along x: column slots; along y: row batches, grid-strided so
    // that the whole grid is resident at once and every block does equal work.
    int64_t slots, batches;
    if (group_axis == DASS_AXIS_COLS) {
        slots = cols / (m > 8 ? m : 8);
        batches = (rows + 3) / 4;
    } else {
        slots = cols / 8;
        const int gb = m >= 8 ? 1 : 8 / m;
        batches = (rows / m + gb - 1) / gb;
    }
    const int64_t nbx = (slots + kBlock - 1) / kBlock;
    int64_t resident = resident_blocks(reinterpret_cast<const void *>(kernel));
    if (resident <= 0)
        resident = 1024;
    int64_t nby = resident / nbx;
    if (nby < 1)
        nby = 1;
    if (nby > batches)
        nby = batches;
    if (nbx * nby > 0x7fffffffLL)
        return fail(DASS_ERR_SHAPE, "%s: matrix too wide for one launch", fn);
    hipLaunchKernelGGL(kernel, dim3((unsigned)(nbx * nby)), dim3(kBlock), 0, stream, W, rows, cols,
                       ld, (const float *)f, m - n_keep, mask_out, nbx, nby);
    return check_launch("N:M kernel");
}

extern "C" size_t dass_nm_batched_workspace_bytes(const dass_nm_task *tasks, int64_t n_tasks)
{
    size_t need = 0;
    for (int64_t i = 0; tasks && i < n_tasks; ++i) {
        const size_t n = dass_nm_workspace_bytes(tasks[i].rows, tasks[i].cols, tasks[i].norm_axis);
        need = n > need ? n : need;
    }
    return need;
}

extern "C" dass_status dass_score_mask_nm_batched(const dass_nm_task *tasks, int64_t n_tasks, dass_dtype dt,
                                                  int n_keep, int m, void *workspace,
                                                  size_t workspace_bytes, void *hip_stream)
{
    using namespace dass;
    const char *fn = "dass_score_mask_nm_batched";
    if (n_tasks < 0 || (n_tasks > 0 && !tasks))
        return fail(DASS_ERR_NULL, "%s: tasks must not be NULL", fn);
    for (int64_t i = 0; i < n_tasks; ++i) {   // validate everything before the first launch
        const dass_nm_task &t = tasks[i];
        const dass_status st = check_nm_args(fn, t.W, t.rows, t.cols, t.ld, dt, t.norms, t.norm_axis, t.group_axis,
                                             t.alpha, n_keep, m, workspace, workspace_bytes);
        if (st != DASS_OK) {
            char detail[kErrorBufferSize];
            snprintf(detail, sizeof detail, "%s", error_buffer());
            return fail(st, "task %lld: %s", (long long)i, detail);
        }
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    auto same_launch = [&](const dass_nm_task &a, const dass_nm_task &b) {
        return a.rows == b.rows && a.cols == b.cols && a.ld == b.ld && a.norm_axis == b.norm_axis &&
               a.group_axis == b.group_axis && a.alpha == b.alpha && (a.mask_out != nullptr) == (b.mask_out != nullptr);
    };
    std::vector<char> done((size_t)n_tasks, 0);
    for (int64_t i = 0; i < n_tasks; ++i) {
        if (done[(size_t)i])
            continue;
        const dass_nm_task &t = tasks[i];
        if (!half_path(t.alpha, n_keep, m)) {
            const dass_status st = dass_score_mask_nm(t.W, t.rows, t.cols, t.ld, dt, t.norms, t.norm_axis, t.group_axis,
                                                      t.alpha, n_keep, m, t.mask_out, workspace, workspace_bytes,
                                                      hip_stream);
            if (st != DASS_OK)
                return st;
            done[(size_t)i] = 1;
            continue;
        }
        const HalfGeometry g = half_geometry(t.rows, t.cols, dt, t.group_axis, m);
        const int64_t per_matrix = g.nbx * g.batches;
        if (per_matrix > 0x7fffffffLL)
            return fail(DASS_ERR_SHAPE, "%s: task %lld: matrix too large for one launch", fn, (long long)i);
        const bool varying = t.norm_axis == t.group_axis && t.alpha != 0.0;
        const bool with_mask = t.mask_out != nullptr;
        nm_batched_kernel_t kernel =
            dt == DASS_BF16 ? (with_mask ? pick_batched_kernel_m<DASS_BF16, true>(m, t.group_axis, t.norm_axis, varying)
                                         : pick_batched_kernel_m<DASS_BF16, false>(m, t.group_axis, t.norm_axis, varying))
                            : (with_mask ? pick_batched_kernel_m<DASS_F32, true>(m, t.group_axis, t.norm_axis, varying)
                                         : pick_batched_kernel_m<DASS_F32, false>(m, t.group_axis, t.norm_axis, varying));
        NmBatch b;
        b.rows = t.rows;
        b.cols = t.cols;
        b.ld = t.ld;
        b.fmode = t.alpha == 0.0 ? kFactorOne : t.alpha == 1.0 ? kFactorNorm : kFactorSqrt;
        b.nbx = (uint32_t)g.nbx;
        b.blocks_per_matrix = (uint32_t)per_matrix;
        const int64_t fit = 0x7fffffffLL / per_matrix;   // matrices one grid can hold
        const int cap = (int)(fit < kBatchMax ? fit : kBatchMax);
        int n = 0;
        auto flush = [&]() -> dass_status {
            if (n == 0)
                return DASS_OK;
            for (int k = n; k < kBatchMax; ++k) {
                b.W[k] = nullptr;
                b.norms[k] = nullptr;
                b.mask[k] = nullptr;
            }
            hipLaunchKernelGGL(kernel, dim3((unsigned)(per_matrix * n)), dim3(g.block), 0, stream, b);
            n = 0;
            return check_launch("batched N:M kernel");
        };
        for (int64_t j = i; j < n_tasks; ++j) {   // every later task that can share this launch
            if (done[(size_t)j] || !same_launch(t, tasks[j]))
                continue;
            b.W[n] = tasks[j].W;
            b.norms[n] = tasks[j].norms;
            b.mask[n] = tasks[j].mask_out;
            done[(size_t)j] = 1;
            if (++n == cap) {
                const dass_status st = flush();
                if (st != DASS_OK)
                    return st;
            }
        }
        const dass_status st = flush();
        if (st != DASS_OK)
            return st;
    }
    return DASS_OK;
}
