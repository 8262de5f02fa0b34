// Stage 2, unstructured: every full line along the group axis is one comparison
// group (Sec. 3 "Pruning Granularity": per input for Gate/Up, per output for
// Down); its n_prune lowest scores |W| * f (Eq. 4 / Eq. 5) become +0 in place.
//
// Selection is an MSB-first radix select over a composite integer key that
// orders positions exactly like (score descending, index ascending):
//   high 64 bits: the bit pattern of the f64 product |w| * f  (non-negative
//                 doubles order like their bit patterns, and the product of an
//                 f32/bf16 weight and an f32 factor is exact in f64);
//   low 24 bits : 0xFFFFFF - index along the line  (lower index = larger key).
// The composite keys of a line are all different, so "the n_keep largest" is a
// unique set: find the n_keep-th largest composite T digit by digit (8 bits per
// pass, 256-bin histogram in LDS), then keep exactly the positions whose
// composite is >= T.  When the key digits alone already isolate exactly the
// wanted number of positions the index passes are skipped.
#include "select.h"

namespace dass {

constexpr int kUBlock = 256;
constexpr int kKeyPasses = 8;  // 64-bit score key, 8 bits per pass
constexpr int kIdxPasses = 3;  // 24-bit inverted index
constexpr uint32_t kIdxMax = 0xFFFFFFu;

__device__ __forceinline__ uint64_t score_key(float a, double f)
{
    return (uint64_t)__double_as_longlong((double)a * f);
}

// Inclusive prefix sum of `v` over the 64 lanes of a wavefront.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t u = __shfl_up(v, o, 64);
        if (lane >= o)
            v += u;
    }
    return v;
}

// State of one line's selection, updated after every pass.
struct SelectState {
    uint64_t key_prefix;   // decided high digits of the score key
    uint32_t idx_prefix;   // decided high digits of the inverted index
    uint32_t need;         // rank still wanted inside the current candidate set
    uint32_t done;         // 1: threshold fully known
};

// One 256-bin histogram (descending bins) -> the bin that holds the need-th
// largest candidate.  Called by one wavefront; lane l owns bins 255-4l .. 252-4l.
// Returns (through refs, valid on every lane) the chosen digit, the candidates
// above it and the count inside it.
__device__ __forceinline__ void pick_bin(const uint32_t *hist, uint32_t need, uint32_t &digit,
                                         uint32_t &above, uint32_t &inside)
{
    const int lane = threadIdx.x & 63;
    uint32_t h[4], sum = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        h[j] = hist[255 - 4 * lane - j];
        sum += h[j];
    }
    const uint32_t incl = wave_inclusive_scan(sum);
    uint32_t excl = incl - sum;
    uint32_t my_digit = 0xFFFFFFFFu, my_above = 0, my_inside = 0;
    if (excl < need && need <= incl) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (my_digit == 0xFFFFFFFFu && need <= excl + h[j]) {
                my_digit = 255 - 4 * lane - j;
                my_above = excl;
                my_inside = h[j];
            }
            excl += h[j];
        }
    }
    // exactly one lane found it (1 <= need <= total); broadcast from that lane
    const uint64_t found = __ballot(my_digit != 0xFFFFFFFFu);
    const int src = found ? __ffsll((long long)found) - 1 : 0;
    digit = __shfl(my_digit, src, 64);
    above = __shfl(my_above, src, 64);
    inside = __shfl(my_inside, src, 64);
}

// ---------------------------------------------------------------------------
// Lines are rows (contiguous): one block per row.
// ---------------------------------------------------------------------------
template <int DT, bool NORM_COLS>
__global__ __launch_bounds__(kUBlock) void unstructured_cols_kernel(
    void *__restrict__ Wv, int64_t rows, int64_t cols, int64_t ld, const float *__restrict__ f,
    uint32_t n_keep, uint8_t *__restrict__ mask)
{
    constexpr int NW = words_for<DT>(8);
    constexpr int NV = NW / 4;
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    __shared__ uint32_t hist[256];
    __shared__ SelectState st;

    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x;
    char *Wrow = static_cast<char *>(Wv) + row * ld * EB;
    const int64_t n_vec = cols / 8;
    const double f_row = NORM_COLS ? 0.0 : (double)f[row];

    auto load_unit = [&](int64_t v, uint32_t *words, double *fv) {
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            const Vec16 x = load16(Wrow + v * 8 * EB + 16 * q);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                words[4 * q + j] = x.w[j];
        }
        if constexpr (NORM_COLS) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const Vec16 x = load16(f + v * 8 + 4 * q);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    fv[4 * q + j] = (double)__uint_as_float(x.w[j]);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                fv[e] = f_row;
        }
    };

    uint64_t thr_key = 0;
    uint32_t thr_idx = 0;  // inverted-index threshold
    const bool keep_all = n_keep >= (uint32_t)cols;
    const bool keep_none = n_keep == 0;

    if (!keep_all && !keep_none) {
        if (tid == 0) {
            st.key_prefix = 0;
            st.idx_prefix = 0;
            st.need = n_keep;
            st.done = 0;
        }
        for (int pass = 0; pass < kKeyPasses + kIdxPasses; ++pass) {
            hist[tid] = 0;
            __syncthreads();
            const SelectState s = st;
            if (s.done)
                break;  // uniform: st is the same for every thread
            const bool key_pass = pass < kKeyPasses;
            const int shift = key_pass ? 8 * (kKeyPasses - 1 - pass)
                                       : 8 * (kKeyPasses + kIdxPasses - 1 - pass);
            // bits above the current digit must match the decided prefix
            const uint64_t key_mask =
                key_pass ? (shift == 56 ? 0ull : ~0ull << (shift + 8)) : ~0ull;
            const uint32_t idx_mask = key_pass ? 0u : (~0u << (shift + 8)) & kIdxMax;
            for (int64_t v = tid; v < n_vec; v += kUBlock) {
                uint32_t words[NW];
                double fv[8];
                load_unit(v, words, fv);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint64_t key = score_key(abs_elem<DT>(words, e), fv[e]);
                    const uint32_t inv = kIdxMax - (uint32_t)(v * 8 + e);
                    if ((key & key_mask) == (s.key_prefix & key_mask) &&
                        (inv & idx_mask) == (s.idx_prefix & idx_mask)) {
                        const uint32_t digit =
                            key_pass ? (uint32_t)(key >> shift) & 255u : (inv >> shift) & 255u;
                        atomicAdd(&hist[digit], 1u);
                    }
                }
            }
            __syncthreads();
            if (tid < 64) {
                uint32_t digit, above, inside;
                pick_bin(hist, s.need, digit, above, inside);
                if (tid == 0) {
                    SelectState n = s;
                    n.need = s.need - above;
                    if (key_pass) {
                        n.key_prefix = s.key_prefix | ((uint64_t)digit << shift);
                        // last key digit and every tied position is wanted: no index passes
                        if (pass == kKeyPasses - 1 && n.need == inside)
                            n.done = 1;
                    } else {
                        n.idx_prefix = s.idx_prefix | (digit << shift);
                    }
                    st = n;
                }
            }
            __syncthreads();
        }
        __syncthreads();
        thr_key = st.key_prefix;
        thr_idx = st.idx_prefix;  // 0 when the index passes were skipped: keeps every tie
    }

    for (int64_t v = tid; v < n_vec; v += kUBlock) {
        uint32_t words[NW];
        double fv[8];
        load_unit(v, words, fv);
        uint32_t kept = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            bool keep;
            if (keep_all) {
                keep = true;
            } else if (keep_none) {
                keep = false;
            } else {
                const uint64_t key = score_key(abs_elem<DT>(words, e), fv[e]);
                const uint32_t inv = kIdxMax - (uint32_t)(v * 8 + e);
                keep = key > thr_key || (key == thr_key && inv >= thr_idx);
            }
            if (!keep)
                zero_elem<DT>(words, e);
            kept |= (keep ? 1u : 0u) << e;
        }
        if (!keep_all) {
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                Vec16 x;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    x.w[j] = words[4 * q + j];
                store16(Wrow + v * 8 * EB + 16 * q, x);
            }
        }
        if (mask)
            mask[row * (cols / 8) + v] = (uint8_t)kept;
    }
}

// ---------------------------------------------------------------------------
// Lines are columns (stride ld): one block per slab of kSlabCols columns; a
// thread owns one 8-column slot and every kRowPhases-th row, so a wavefront
// reads 64-byte (bf16) row segments of 16 consecutive rows.
// ---------------------------------------------------------------------------
constexpr int kSlabCols = 32;
constexpr int kSlabSlots = kSlabCols / 8;
constexpr int kRowPhases = kUBlock / kSlabSlots;

template <int DT, bool NORM_ROWS>
__global__ __launch_bounds__(kUBlock) void unstructured_rows_kernel(
    void *__restrict__ Wv, int64_t rows, int64_t cols, int64_t ld, const float *__restrict__ f,
    uint32_t n_keep, uint8_t *__restrict__ mask)
{
    constexpr int NW = words_for<DT>(8);
    constexpr int NV = NW / 4;
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    __shared__ uint32_t hist[kSlabCols][256];
    __shared__ SelectState st[kSlabCols];
    __shared__ uint32_t any_open;

    const int tid = threadIdx.x;
    const int sl = tid % kSlabSlots, rp = tid / kSlabSlots;
    const int64_t slot = (int64_t)blockIdx.x * kSlabSlots + sl;
    const bool active = slot < cols / 8;
    const int64_t c0 = slot * 8;
    char *W = static_cast<char *>(Wv);

    double fc[8];
    if constexpr (!NORM_ROWS) {
        if (active) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const Vec16 x = load16(f + c0 + 4 * q);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    fc[4 * q + j] = (double)__uint_as_float(x.w[j]);
            }
        }
    }

    auto load_unit = [&](int64_t r, uint32_t *words) {
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            const Vec16 x = load16(W + (r * ld + c0) * EB + 16 * q);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                words[4 * q + j] = x.w[j];
        }
    };

    const bool keep_all = n_keep >= (uint32_t)rows;
    const bool keep_none = n_keep == 0;

    if (!keep_all && !keep_none) {
        if (tid < kSlabCols) {
            SelectState s;
            s.key_prefix = 0;
            s.idx_prefix = 0;
            s.need = n_keep;
            // columns past the matrix edge have nothing to select
            s.done = ((int64_t)blockIdx.x * kSlabCols + tid) < cols ? 0u : 1u;
            st[tid] = s;
        }
        for (int pass = 0; pass < kKeyPasses + kIdxPasses; ++pass) {
            for (int i = tid; i < kSlabCols * 256; i += kUBlock)
                (&hist[0][0])[i] = 0;
            if (tid == 0)
                any_open = 0;
            __syncthreads();
            const bool key_pass = pass < kKeyPasses;
            const int shift = key_pass ? 8 * (kKeyPasses - 1 - pass)
                                       : 8 * (kKeyPasses + kIdxPasses - 1 - pass);
            const uint64_t key_mask =
                key_pass ? (shift == 56 ? 0ull : ~0ull << (shift + 8)) : ~0ull;
            const uint32_t idx_mask = key_pass ? 0u : (~0u << (shift + 8)) & kIdxMax;
            if (active) {
                SelectState s[8];
                bool open = false;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    s[e] = st[sl * 8 + e];
                    open |= s[e].done == 0;
                }
                if (open) {
                    for (int64_t r = rp; r < rows; r += kRowPhases) {
                        uint32_t words[NW];
                        load_unit(r, words);
                        const double fr = NORM_ROWS ? (double)f[r] : 0.0;
                        const uint32_t inv = kIdxMax - (uint32_t)r;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const uint64_t key =
                                score_key(abs_elem<DT>(words, e), NORM_ROWS ? fr : fc[e]);
                            if (!s[e].done && (key & key_mask) == (s[e].key_prefix & key_mask) &&
                                (inv & idx_mask) == (s[e].idx_prefix & idx_mask)) {
                                const uint32_t digit = key_pass ? (uint32_t)(key >> shift) & 255u
                                                                : (inv >> shift) & 255u;
                                atomicAdd(&hist[sl * 8 + e][digit], 1u);
                            }
                        }
                    }
                }
            }
            __syncthreads();
            // each wavefront settles kSlabCols / 4 columns
            const int wave = tid / 64;
            for (int c = wave; c < kSlabCols; c += kUBlock / 64) {
                const SelectState s = st[c];
                if (s.done)
                    continue;  // uniform inside the wavefront
                uint32_t digit, above, inside;
                pick_bin(hist[c], s.need, digit, above, inside);
                if ((tid & 63) == 0) {
                    SelectState n = s;
                    n.need = s.need - above;
                    if (key_pass) {
                        n.key_prefix = s.key_prefix | ((uint64_t)digit << shift);
                        if (pass == kKeyPasses - 1 && n.need == inside)
                            n.done = 1;
                    } else {
                        n.idx_prefix = s.idx_prefix | (digit << shift);
                    }
                    if (pass == kKeyPasses + kIdxPasses - 1)
                        n.done = 1;
                    st[c] = n;
                    if (!n.done)
                        any_open = 1;
                }
            }
            __syncthreads();
            if (!any_open)
                break;  // uniform
            __syncthreads();  // any_open is rewritten at the top of the next pass
        }
        __syncthreads();
    }

    if (!active)
        return;
    uint64_t thr_key[8];
    uint32_t thr_idx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        thr_key[e] = (keep_all || keep_none) ? 0 : st[sl * 8 + e].key_prefix;
        thr_idx[e] = (keep_all || keep_none) ? 0 : st[sl * 8 + e].idx_prefix;
    }
    for (int64_t r = rp; r < rows; r += kRowPhases) {
        uint32_t words[NW];
        load_unit(r, words);
        const double fr = NORM_ROWS ? (double)f[r] : 0.0;
        const uint32_t inv = kIdxMax - (uint32_t)r;
        uint32_t kept = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            bool keep;
            if (keep_all) {
                keep = true;
            } else if (keep_none) {
                keep = false;
            } else {
                const uint64_t key = score_key(abs_elem<DT>(words, e), NORM_ROWS ? fr : fc[e]);
                keep = key > thr_key[e] || (key == thr_key[e] && inv >= thr_idx[e]);
            }
            if (!keep)
                zero_elem<DT>(words, e);
            kept |= (keep ? 1u : 0u) << e;
        }
        if (!keep_all) {
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                Vec16 x;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    x.w[j] = words[4 * q + j];
                store16(W + (r * ld + c0) * EB + 16 * q, x);
            }
        }
        if (mask)
            mask[r * (cols / 8) + slot] = (uint8_t)kept;
    }
}

}  // namespace dass

extern "C" size_t dass_unstructured_workspace_bytes(int64_t rows, int64_t cols, dass_dtype dt,
                                                    dass_axis norm_axis, dass_axis group_axis)
{
    (void)dt;
    (void)group_axis;
    const int64_t n = norm_axis == DASS_AXIS_ROWS ? rows : cols;
    return n > 0 ? dass::round_up((size_t)n * sizeof(float), 256) : 0;
}

extern "C" dass_status dass_score_mask_unstructured(void *W, int64_t rows, int64_t cols, int64_t ld,
                                                    dass_dtype dt, const float *norms,
                                                    dass_axis norm_axis, dass_axis group_axis,
                                                    double alpha, int64_t n_prune,
                                                    uint8_t *mask_out, void *workspace,
                                                    size_t workspace_bytes, void *hip_stream)
{
    using namespace dass;
    const char *fn = "dass_score_mask_unstructured";
    dass_status s = check_score_args(
        fn, W, rows, cols, ld, dt, norms, norm_axis, group_axis, alpha, workspace, workspace_bytes,
        dass_unstructured_workspace_bytes(rows, cols, dt, norm_axis, group_axis));
    if (s != DASS_OK)
        return s;
    const int64_t len = group_axis == DASS_AXIS_ROWS ? rows : cols;
    const int64_t lines = group_axis == DASS_AXIS_ROWS ? cols : rows;
    if (n_prune < 0 || n_prune > len)
        return fail(DASS_ERR_ARG, "%s: n_prune=%lld outside [0, %lld]", fn, (long long)n_prune,
                    (long long)len);
    if (len > (int64_t)kIdxMax)
        return fail(DASS_ERR_SHAPE, "%s: line length %lld exceeds %u", fn, (long long)len, kIdxMax);
    const int64_t blocks =
        group_axis == DASS_AXIS_COLS ? lines : (cols + kSlabCols - 1) / kSlabCols;
    if (blocks > 0x7fffffffLL)
        return fail(DASS_ERR_SHAPE, "%s: too many lines for one launch", fn);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    float *f = static_cast<float *>(workspace);
    s = launch_factor(norms, norm_axis == DASS_AXIS_ROWS ? rows : cols, alpha, f, stream);
    if (s != DASS_OK)
        return s;

    const uint32_t n_keep = (uint32_t)(len - n_prune);
    const bool bf16 = dt == DASS_BF16;
    const dim3 grid((unsigned)blocks), block(kUBlock);
    if (group_axis == DASS_AXIS_COLS) {
        auto k = bf16 ? (norm_axis == DASS_AXIS_COLS ? unstructured_cols_kernel<DASS_BF16, true>
                                                     : unstructured_cols_kernel<DASS_BF16, false>)
                      : (norm_axis == DASS_AXIS_COLS ? unstructured_cols_kernel<DASS_F32, true>
                                                     : unstructured_cols_kernel<DASS_F32, false>);
        hipLaunchKernelGGL(k, grid, block, 0, stream, W, rows, cols, ld, (const float *)f, n_keep,
                           mask_out);
    } else {
        auto k = bf16 ? (norm_axis == DASS_AXIS_ROWS ? unstructured_rows_kernel<DASS_BF16, true>
                                                     : unstructured_rows_kernel<DASS_BF16, false>)
                      : (norm_axis == DASS_AXIS_ROWS ? unstructured_rows_kernel<DASS_F32, true>
                                                     : unstructured_rows_kernel<DASS_F32, false>);
        hipLaunchKernelGGL(k, grid, block, 0, stream, W, rows, cols, ld, (const float *)f, n_keep,
                           mask_out);
    }
    return check_launch("unstructured kernel");
}
