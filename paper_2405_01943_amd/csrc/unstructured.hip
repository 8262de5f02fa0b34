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
#include "unstructured_tiled.h"

#include <mutex>
#include <type_traits>

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
    uint32_t n_keep, uint8_t *__restrict__ mask, const uint32_t *__restrict__ gate, uint32_t gate_rows)
{
    constexpr int NW = words_for<DT>(8);
    constexpr int NV = NW / 4;
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    __shared__ uint32_t hist[256];
    __shared__ SelectState st;
    if (gate && gate[blockIdx.x / gate_rows] == 0)
        return;   // the launch before this one has done this row (uniform)

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
    uint32_t n_keep, uint8_t *__restrict__ mask, const uint32_t *__restrict__ gate)
{
    constexpr int NW = words_for<DT>(8);
    constexpr int NV = NW / 4;
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    __shared__ uint32_t hist[kSlabCols][256];
    if (gate && *gate == 0)
        return;   // the launches before this one have done the work (uniform)
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


// ===========================================================================
// Line-resident kernels, alpha in {0, 0.5, 1}: a 1024-thread workgroup holds up to 8 lines in its
// registers (131072 bf16 / 65536 f32 weights in all), so the weights are read once and written
// once; all selection passes run on the registers.  Column lines: up to 16384 (bf16) / 8192 (f32)
// rows; row lines: any length below 65536 whose factors fit LDS beside the histograms (8, 4, 2 or
// 1 lines per workgroup).
//
// Order of positions in a line: (score descending, index ascending), encoded as a composite
// of three 32-bit fields (A, B, C) compared lexicographically, larger = kept first:
//   A, B  the exact score: the two-term f32 form of select.h (A = bits of p, B = the error term
//         q mapped to an unsigned integer that grows with q; rounding is monotonic, so p orders
//         the scores and q orders those with equal p), or, when a factor or a product leaves
//         the range in which that form is exact, the high and low words of the f64 product;
//   C     0xFFFF - index (lines are shorter than 65536).
// The threshold (the n_keep-th largest composite) is found digit by digit, most significant
// first: 11 + 11 + 10 bits for A and for B, 11 + 5 for C, with one 2048-bin histogram per line
// and pass.  The search stops as soon as every candidate left in the chosen bin is wanted, and
// after two passes (22 bits of A) the candidates left are so few that they are listed and ranked
// directly; only a line with more than 64 of them goes on with the third pass.
// ===========================================================================
constexpr int kLrBins = 2048;
constexpr int kLrLines = 8;
constexpr int kLrPasses = 8;
constexpr int kLrThreads = 1024;
constexpr int kLrVecs = 16;   // 16-byte vectors held by a thread
constexpr size_t kFlagBytes = 256;   // the block of the workspace that holds the flag word of the tiled passes
constexpr int kLrTies = 64;   // scores of the threshold's bin that are listed and ranked directly, per line

struct LrState {
    uint32_t a, b, c;   // decided digits of the threshold, undecided bits 0
    uint32_t need;      // rank still wanted among the candidates (>= 1)
    uint32_t open;      // 1 until the threshold is known
    uint32_t pad[3];
};

struct LrPass {
    int field, shift, width;
};
__device__ __forceinline__ LrPass lr_pass(int pass)
{
    if (pass < 6) {
        const int k = pass % 3;
        return {pass / 3, k == 0 ? 21 : k == 1 ? 10 : 0, k == 2 ? 10 : 11};
    }
    return {2, pass == 6 ? 5 : 0, pass == 6 ? 11 : 5};
}

__device__ __forceinline__ uint32_t lr_mono(float q)   // unsigned integer that grows with q
{
    const uint32_t b = __float_as_uint(q);
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}

__device__ __forceinline__ bool lr_keep(const LrState &st, uint32_t a, uint32_t b, uint32_t c)
{
    // all three fields are read and compared unconditionally: straight-line code
    const uint32_t ta = st.a, tb = st.b, tc = st.c;
    return (a > ta) | ((a == ta) & ((b > tb) | ((b == tb) & (c >= tc))));
}

__device__ __forceinline__ uint32_t lr_uniform(uint32_t x)   // a value every lane agrees on, in a scalar register
{
    return __builtin_amdgcn_readfirstlane(x);
}

// One wavefront finds, in the 2048-bin histogram of a line, the bin that holds the need-th
// largest candidate and updates the line's state.  Lane l owns bins 2047 - 32 l .. 2016 - 32 l.
// Returns (on every lane) whether a bin at or above `alarm_bin` is occupied.
__device__ __forceinline__ bool lr_settle(const uint32_t *hist, LrState *state, const LrPass &ps, int pass,
                                          uint32_t alarm_bin)
{
    int lane = threadIdx.x & 63;
    asm volatile("" : "+v"(lane));   // keeps the per-lane bin numbers out of the caller's loop-invariant registers
    const LrState st = *state;
    const uint32_t *mine = hist + kLrBins - 32 * (lane + 1);   // the lane's 32 bins, ascending
    uint32_t sum = 0;
    bool alarm = false;
#pragma clang loop unroll(disable)
    for (int q = 0; q < 8; ++q) {
        const u32x4 x = *reinterpret_cast<const u32x4 *>(mine + 4 * q);
        sum += x[0] + x[1] + x[2] + x[3];
        alarm |= (x[0] | x[1] | x[2] | x[3]) != 0 && (uint32_t)(kLrBins - 32 * (lane + 1) + 4 * q + 3) >= alarm_bin;
    }
    const uint32_t incl = wave_inclusive_scan(sum);
    uint32_t excl = incl - sum;
    uint32_t my_digit = 0xFFFFFFFFu, my_above = 0, my_inside = 0;
    if (excl < st.need && st.need <= incl) {   // one lane: walk its bins from the highest down
#pragma clang loop unroll(disable)
        for (int j = 31; j >= 0; --j) {
            const uint32_t h = mine[j];
            if (st.need <= excl + h) {
                my_digit = kLrBins - 32 * (lane + 1) + j;
                my_above = excl;
                my_inside = h;
                break;
            }
            excl += h;
        }
    }
    const uint64_t found = __ballot(my_digit != 0xFFFFFFFFu);   // exactly one lane: 1 <= need <= candidates
    const int src = found ? __ffsll((long long)found) - 1 : 0;
    const uint32_t digit = __shfl(my_digit, src, 64), above = __shfl(my_above, src, 64),
                   inside = __shfl(my_inside, src, 64);
    if (lane == 0) {
        LrState n = st;
        n.need = st.need - above;
        const uint32_t d = digit << ps.shift;
        if (ps.field == 0)
            n.a |= d;
        else if (ps.field == 1)
            n.b |= d;
        else
            n.c |= d;
        // every candidate left in the bin is wanted (always so after the last pass: composites are unique)
        if (n.need == inside || pass == kLrPasses - 1)
            n.open = 0;
        *state = n;
    }
    return __ballot(alarm) != 0;
}

enum { kLrDown = 0, kLrGate = 1 };

// LAYOUT kLrGate: lines are columns (stride ld).  The workgroup owns 8 consecutive columns,
//   VR = 8 / EPV vectors per row; thread t holds rows t, t + 1024, ...: its vector j is vector
//   j % VR of row t + (j / VR) 1024, and element e of it is on line (j % VR) EPV + e.
//   Workgroups are numbered so that the 8 that share 64 consecutive columns (the same 128-byte
//   pieces of every row) run on the same XCD at the same time and meet in its L2.
// LAYOUT kLrDown: lines are rows (contiguous).  The workgroup owns 8 >> vpl_log2 ... 8 consecutive
//   rows; a thread holds 1 << vpl_log2 vectors of each: its vector j is vector
//   t + (j & (vpl - 1)) 1024 of line j >> vpl_log2.
// FACTOR_ALONG: the factor varies along the line (the DaSS configuration, Eq. 4 / Eq. 5) and
//   the scaled factors of all positions are staged in LDS; otherwise there is one per line.
// The host guarantees 0 < n_keep < line length.
template <int DT, int LAYOUT, bool FACTOR_ALONG>
__global__ __launch_bounds__(kLrThreads) void unstructured_resident_kernel(
    void *__restrict__ Wv, int64_t rows, int64_t cols, int64_t ld, const float *__restrict__ norms,
    int fmode, uint32_t n_keep, uint8_t *__restrict__ mask, int vpl_log2, int lines_per_block,
    const uint32_t *__restrict__ gate, uint32_t gate_rows)
{
    constexpr int NT = kLrThreads, VPT = kLrVecs;
    // gate: the launches before this one set a word where they left work - one for the whole matrix
    // (gate_rows = 0) or one per block of gate_rows rows (row lines)
    if (gate && gate[gate_rows ? (uint32_t)(((int64_t)blockIdx.x * lines_per_block) / gate_rows) : 0u] == 0)
        return;   // uniform
    constexpr int EPV = DT == DASS_BF16 ? 8 : 4;
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    constexpr int VR = 8 / EPV;
    constexpr bool GATE = LAYOUT == kLrGate;
    extern __shared__ __attribute__((aligned(16))) char lr_smem[];
    uint32_t *hist = reinterpret_cast<uint32_t *>(lr_smem);                           // [lines_per_block][kLrBins]
    LrState *state = reinterpret_cast<LrState *>(lr_smem + (size_t)lines_per_block * kLrBins * 4);   // [kLrLines]
    uint32_t *flags = reinterpret_cast<uint32_t *>(state + kLrLines);                 // [0] a line is open, [1] f64 form wanted
    uint32_t *trash = flags + 4;                                                      // [64] counters nobody reads
    uint32_t *tie_count = trash + 64;                                                 // [kLrLines]
    uint2 *tie_list = reinterpret_cast<uint2 *>(tie_count + kLrLines);                // [kLrLines][kLrTies] fields (B, low bits of A : C)
    float *fl = reinterpret_cast<float *>(tie_list + kLrLines * kLrTies);             // scaled factors

    const int tid = threadIdx.x;
    const int64_t len = GATE ? rows : cols;
    char *W = static_cast<char *>(Wv);
    // Gate: blockIdx -> column octet (see above); the grid is padded to a multiple of 64
    const uint32_t slot = blockIdx.x / 8;
    const int64_t octet = GATE ? (int64_t)((slot / 8) * 8 + blockIdx.x % 8) * 8 + slot % 8 : 0;
    if (GATE && octet >= cols / 8)
        return;
    const int64_t c0 = octet * 8;
    const int64_t row0 = GATE ? 0 : (int64_t)blockIdx.x * lines_per_block;
    const int n_lines = GATE ? 8 : (int)(rows - row0 < lines_per_block ? rows - row0 : lines_per_block);
    const int64_t vec_per_line = cols / EPV;   // Down
    const int vpl_mask = (1 << vpl_log2) - 1;

    auto vec_line0 = [&](int j) { return GATE ? (j % VR) * EPV : j >> vpl_log2; };   // line of its element 0
    // A thread recomputes what depends on its number in every phase from a fresh copy of it
    // (t below), so that no per-vector address or flag occupies a register across the phases.
    auto fresh_tid = [&]() {
        uint32_t x = (uint32_t)tid;
        asm volatile("" : "+v"(x));
        return x;
    };
    // position of vector j along the lines: Gate: its row; Down: its index inside the line
    auto vec_pos = [&](int j, uint32_t t) -> uint32_t {
        return GATE ? t + (uint32_t)(j / VR) * NT : t + (uint32_t)(j & vpl_mask) * NT;
    };
    auto vec_valid = [&](int j, uint32_t t) {
        return GATE ? vec_pos(j, t) < (uint32_t)rows
                    : (vec_line0(j) < n_lines && vec_pos(j, t) < (uint32_t)vec_per_line);
    };
    // byte offsets fit 32 bits (checked by the host)
    const uint32_t ld32 = (uint32_t)ld, col_bytes = (uint32_t)c0 * EB, row0_32 = (uint32_t)row0;
    auto vec_addr = [&](int j, uint32_t t) -> char * {
        if (GATE)
            return W + (size_t)(vec_pos(j, t) * ld32 * EB + col_bytes + (uint32_t)((j % VR) * EPV * EB));
        return W + (size_t)((row0_32 + (uint32_t)vec_line0(j)) * ld32 * EB + vec_pos(j, t) * (EPV * EB));
    };

    u32x4 v[VPT];
    {
        const uint32_t t = fresh_tid();
#pragma unroll
        for (int j = 0; j < VPT; ++j)
            if (vec_valid(j, t))
                v[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(vec_addr(j, t)));
    }

    // ---- factors, scaled as select.h wants them
    bool fast_ok = true;
    if constexpr (FACTOR_ALONG) {
        for (int64_t i = tid; i < len; i += NT) {
            const float f = factor_of(norms[i], fmode);
            fast_ok &= factor_in_fast_range(f);
            fl[i] = f * kFactorScale;
        }
    } else {
        if (tid < n_lines) {   // one per line
            const float f = factor_of(norms[GATE ? c0 + tid : row0 + tid], fmode);
            fast_ok &= factor_in_fast_range(f);
            fl[tid] = f * kFactorScale;
        }
    }
    auto reset_state = [&]() {
        if (tid < kLrLines) {
            LrState st;
            st.a = st.b = st.c = 0;
            st.need = n_keep;
            st.open = tid < n_lines ? 1u : 0u;
            state[tid] = st;
            tie_count[tid] = 0;
        }
    };
    reset_state();
    if (tid == 0)
        flags[1] = 0;
    __syncthreads();
    if (!fast_ok)
        flags[1] = 1;
    __syncthreads();
    bool exact = flags[1] != 0;

    // Scaled factors of the EPV elements of vector j (line0: the line of element 0).
    auto vec_factors = [&](int j, uint32_t t, int line0, float *fs) __attribute__((always_inline)) {
        if constexpr (FACTOR_ALONG && GATE) {
            const float f = fl[vec_pos(j, t)];
#pragma unroll
            for (int e = 0; e < EPV; ++e)
                fs[e] = f;
        } else if constexpr (FACTOR_ALONG) {
#pragma unroll
            for (int q = 0; q < EPV / 4; ++q) {
                const u32x4 x = *reinterpret_cast<const u32x4 *>(fl + vec_pos(j, t) * EPV + 4 * q);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    fs[4 * q + i] = __uint_as_float(x[i]);
            }
        } else {
#pragma unroll
            for (int e = 0; e < EPV; ++e)
                fs[e] = fl[GATE ? line0 + e : line0];
        }
    };
    auto norm_index = [&](int j, uint32_t t, int e, int line) -> int64_t {
        if (FACTOR_ALONG)
            return GATE ? vec_pos(j, t) : vec_pos(j, t) * EPV + e;
        return GATE ? c0 + line : row0 + line;
    };

    // Counting pass on a digit of field A in the two-term form, every vector's code laid out
    // (the common passes): candidates are the elements whose bits under himask agree with the
    // decided ones.
    auto count_fast = [&](int shift, uint32_t wmask, uint32_t himask) __attribute__((always_inline)) {
        const uint32_t t = fresh_tid();
        // Straight-line code per element (a branch per element would make every LDS access wait
        // for the one before): an element that is no candidate adds to a per-lane dummy counter.
        // A closed line gets a pattern no score matches (scores have the sign bit clear).
        uint32_t *const dummy = trash + (t & 63u);
        uint32_t sa[kLrLines], hm[kLrLines];
        if constexpr (GATE) {
#pragma unroll
            for (int l = 0; l < kLrLines; ++l) {
                const bool open = lr_uniform(state[l].open) != 0;
                sa[l] = open ? lr_uniform(state[l].a) : 0xFFFFFFFFu;
                hm[l] = open ? himask : 0xFFFFFFFFu;
            }
        }
#pragma unroll
        for (int j = 0; j < VPT; ++j) {
            __builtin_amdgcn_sched_barrier(0);
            const int line0 = vec_line0(j);
            uint32_t da = 0;
            bool line_open = true;
            if constexpr (!GATE) {
                line_open = line0 < n_lines && lr_uniform(state[line0 & (kLrLines - 1)].open) != 0;
                da = lr_uniform(state[line0 & (kLrLines - 1)].a);
            }
            if (line_open && vec_valid(j, t)) {
                asm volatile("" : "+v"(v[j]));   // nothing derived from the data is carried from pass to pass
                float fs[EPV];
                vec_factors(j, t, line0, fs);
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    const int line = GATE ? line0 + e : line0;
                    const uint32_t a = __float_as_uint(fabsf(elem_of<DT>(v[j], e)) * fs[e]);
                    const bool cand = ((a ^ (GATE ? sa[line] : da)) & (GATE ? hm[line] : himask)) == 0;
                    atomicAdd(cand ? hist + line * kLrBins + ((a >> shift) & wmask) : dummy, 1u);
                }
            }
        }
    };

    // The scores of an open line that agree with the decided digits of A above bit `shift` go
    // into the line's list as (B, low 10 bits of A : C), and one wavefront ranks them directly.
    // shift 10, after two passes: the threshold's 22-bit bin, a handful of scores, so the third
    // counting pass is not needed; shift 0, after three: the scores that share the threshold's
    // A.  A list that overflows leaves the line to the next counting pass.
    auto collect_ties = [&](int shift) __attribute__((always_inline)) {
        const uint32_t t = fresh_tid();
        uint32_t sa[kLrLines];
        if constexpr (GATE) {
#pragma unroll
            for (int l = 0; l < kLrLines; ++l)   // a closed line gets a pattern no score has
                sa[l] = lr_uniform(state[l].open) != 0 ? lr_uniform(state[l].a) : 0xFFFFFFFFu;
        }
#pragma unroll
        for (int j = 0; j < VPT; ++j) {
            __builtin_amdgcn_sched_barrier(0);
            const int line0 = vec_line0(j);
            uint32_t da = 0;
            bool line_open = true;
            if constexpr (!GATE) {
                line_open = line0 < n_lines && lr_uniform(state[line0 & (kLrLines - 1)].open) != 0;
                da = lr_uniform(state[line0 & (kLrLines - 1)].a);
            }
            if (line_open && vec_valid(j, t)) {
                asm volatile("" : "+v"(v[j]));
                float fs[EPV];
                vec_factors(j, t, line0, fs);
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    const int line = GATE ? line0 + e : line0;
                    const float w = fabsf(elem_of<DT>(v[j], e));
                    const float p = w * fs[e];
                    if (((__float_as_uint(p) ^ (GATE ? sa[line] : da)) >> shift) == 0) {
                        const uint32_t slot = atomicAdd(tie_count + line, 1u);
                        if (slot < (uint32_t)kLrTies) {
                            const uint32_t idx = GATE ? vec_pos(j, t) : vec_pos(j, t) * EPV + e;
                            tie_list[line * kLrTies + slot] = make_uint2(
                                lr_mono(fmaf(w, fs[e], -p)), ((__float_as_uint(p) & 0x3ffu) << 16) | (0xFFFFu - idx));
                        }
                    }
                }
            }
        }
    };
    // Wavefront `line` ranks its line's list by (A, B, C) and closes the line on the entry of
    // the wanted rank.  The list holds every score of its bin, so an entry whose A no other
    // entry shares is a threshold on A alone (fields B and C stay 0: keep iff A >= threshold).
    auto rank_ties = [&](int line) {
        const uint32_t n = tie_count[line];
        if (n > (uint32_t)kLrTies)
            return;
        const uint32_t lane = tid & 63;
        const uint2 mine = tie_list[line * kLrTies + (lane < n ? lane : 0)];
        const uint32_t ma = mine.y >> 16, mc = mine.y & 0xFFFFu;
        uint32_t above = 0, same_a = 0;
        for (uint32_t k = 0; k < n; ++k) {
            const uint2 other = tie_list[line * kLrTies + k];
            const uint32_t oa = other.y >> 16, oc = other.y & 0xFFFFu;
            above += (oa > ma) | ((oa == ma) & ((other.x > mine.x) | ((other.x == mine.x) & (oc > mc))));
            same_a += oa == ma;
        }
        if (lane < n && above + 1 == state[line].need) {   // composites differ, so exactly one lane
            state[line].a |= ma;   // the undecided bits were 0 (all of them decided: the same bits again)
            if (same_a > 1) {
                state[line].b = mine.x;
                state[line].c = mc;
            }
            state[line].open = 0;
        }
    };

    // Fields A and B of one element, either form.
    auto fields = [&](float w, float fs, int64_t in, bool need_b, uint32_t &a, uint32_t &b) __attribute__((always_inline)) {
        w = fabsf(w);
        if (!exact) {
            const float p = w * fs;
            a = __float_as_uint(p);
            b = need_b ? lr_mono(fmaf(w, fs, -p)) : 0u;
        } else {   // f64 product with the unscaled factor, recomputed from the norm
            const uint64_t k = (uint64_t)__double_as_longlong((double)w * (double)factor_of(norms[in], fmode));
            a = (uint32_t)(k >> 32);
            b = (uint32_t)k;
        }
    };
    // The rare passes (fields B and C, f64 form) work from memory, where the weights are still
    // unmodified, in loops that are not laid out per vector: they cost the common passes neither
    // registers nor code.
    // Element e of a vector and its scaled factor, e known only at run time: the rare passes loop
    // over the elements too, so that they need few registers beside the 16 data vectors.
    auto word_at = [](const u32x4 &x, int k) { return k == 0 ? x[0] : k == 1 ? x[1] : k == 2 ? x[2] : x[3]; };
    auto elem_at = [&](const u32x4 &x, int e) {
        if constexpr (DT == DASS_BF16) {
            const uint32_t w = word_at(x, e >> 1);
            return __uint_as_float((e & 1) ? (w & 0xffff0000u) : (w << 16));
        } else {
            return __uint_as_float(word_at(x, e));
        }
    };
    auto zero_at_if = [](u32x4 &x, int e, bool drop) {
        const int k = DT == DASS_BF16 ? e >> 1 : e;
        const uint32_t m = !drop ? 0xffffffffu : DT == DASS_BF16 ? ((e & 1) ? 0x0000ffffu : 0xffff0000u) : 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            x[i] &= i == k ? m : 0xffffffffu;
    };
    auto factor_at = [&](int j, uint32_t t, int e, int line) {
        if (FACTOR_ALONG)
            return fl[GATE ? vec_pos(j, t) : vec_pos(j, t) * EPV + e];
        return fl[line];
    };
    auto count_any = [&](const LrPass ps, uint32_t wmask, uint32_t himask) __attribute__((always_inline)) {
        const uint32_t t = fresh_tid();
#pragma clang loop unroll(disable)
        for (int j = 0; j < VPT; ++j) {
            const int line0 = vec_line0(j);
            if (vec_valid(j, t)) {
                const u32x4 x = *reinterpret_cast<const u32x4 *>(vec_addr(j, t));   // still unmodified in memory
#pragma clang loop unroll(disable)
                for (int e = 0; e < EPV; ++e) {
                    const int line = GATE ? line0 + e : line0;
                    if (!state[line].open)
                        continue;
                    const uint32_t idx = GATE ? vec_pos(j, t) : vec_pos(j, t) * EPV + e;
                    uint32_t a, b;
                    fields(elem_at(x, e), factor_at(j, t, e, line), norm_index(j, t, e, line), true, a, b);
                    const uint32_t c = 0xFFFFu - idx;
                    const uint32_t ta = state[line].a, tb = state[line].b, tc = state[line].c;
                    bool cand;
                    uint32_t x;
                    if (ps.field == 0) {
                        cand = ((a ^ ta) & himask) == 0;
                        x = a;
                    } else if (ps.field == 1) {
                        cand = (a == ta) & (((b ^ tb) & himask) == 0);
                        x = b;
                    } else {
                        cand = (a == ta) & (b == tb) & (((c ^ tc) & himask) == 0);
                        x = c;
                    }
                    if (cand)
                        atomicAdd(hist + line * kLrBins + ((x >> ps.shift) & wmask), 1u);
                }
            }
        }
    };

    // One counting pass and its settling.  Wavefront l settles line l; a product that became
    // infinite shows in the first digit of p.  Leaves flags[0] = a line is still open.
    auto run_pass = [&](int pass, auto fast_tag) __attribute__((always_inline)) {
        for (int i = tid; i < lines_per_block * kLrBins / 4; i += NT)
            reinterpret_cast<u32x4 *>(hist)[i] = u32x4{0, 0, 0, 0};
        if (tid == 0)
            flags[0] = 0;
        __syncthreads();
        const LrPass ps = lr_pass(pass);
        const uint32_t wmask = (1u << ps.width) - 1u;
        const uint32_t himask = ps.shift + ps.width >= 32 ? 0u : ~0u << (ps.shift + ps.width);
        if constexpr (decltype(fast_tag)::value)
            count_fast(ps.shift, wmask, himask);
        else
            count_any(ps, wmask, himask);
        __syncthreads();
        const int wave = tid / 64;
        if (wave < n_lines && state[wave].open) {   // uniform inside the wavefront
            const uint32_t alarm_bin =
                (decltype(fast_tag)::value && pass == 0) ? (0x7f800000u >> 21) : (uint32_t)kLrBins;
            const bool alarm = lr_settle(hist + wave * kLrBins, state + wave, ps, pass, alarm_bin);
            if ((tid & 63) == 0) {
                if (state[wave].open)
                    flags[0] = 1;
                if (alarm)
                    flags[1] = 1;
            }
        }
        __syncthreads();
    };

    // Field A in the two-term form: two counting passes (22 bits), then the few scores left in
    // the threshold's bin are ranked directly.  Only a line whose bin holds more than kLrTies
    // scores (equal scores in number) takes the third counting pass and a second ranking, of the
    // scores that share the threshold's A.
    bool open_lines = true;
    // Ranking of the open lines' lists; leaves open_lines = a line is still open.
    auto ties_round = [&](int shift) __attribute__((always_inline)) {
        collect_ties(shift);
        __syncthreads();
        const int wave = tid / 64;
        if (wave < n_lines && state[wave].open)   // uniform inside the wavefront
            rank_ties(wave);
        if (tid == 0)
            flags[0] = 0;
        __syncthreads();
        if (tid < n_lines && state[tid].open)
            flags[0] = 1;
        __syncthreads();
        open_lines = flags[0] != 0;
        __syncthreads();
    };
    if (!exact) {
        for (int pass = 0; pass < 2; ++pass) {
            run_pass(pass, std::true_type{});
            if (flags[1]) {   // start again on f64 products (uniform)
                exact = true;
                reset_state();
                break;
            }
            open_lines = flags[0] != 0;
            if (!open_lines)
                break;   // uniform
            __syncthreads();   // flags[0] is cleared at the top of the next pass
        }
        __syncthreads();
        if (!exact && open_lines)
            ties_round(10);
        if (!exact && open_lines) {   // a bin with more than kLrTies scores
            if (tid < kLrLines)
                tie_count[tid] = 0;   // ordered before the next collection by the barriers of the pass
            run_pass(2, std::true_type{});
            open_lines = flags[0] != 0;
            __syncthreads();
            if (open_lines)
                ties_round(0);
        }
    }
    // What is left (a tie list that overflowed: from field B on; the f64 form: from the start)
    // goes digit by digit through the code that works from memory.
    if (exact || open_lines) {
        for (int pass = exact ? 0 : 3;; ++pass) {
            run_pass(pass, std::false_type{});
            if (!flags[0])
                break;   // uniform
            __syncthreads();
        }
    }

    // ---- apply: zero what ranks below the threshold, store, write the mask bits
    bool beyond_a = false;   // a threshold decided beyond field A
    for (int l = 0; l < n_lines; ++l)
        beyond_a |= state[l].b != 0 || state[l].c != 0;
    beyond_a = lr_uniform(beyond_a) != 0;

    auto write_mask = [&](int j, uint32_t t, int line0, uint32_t kept, uint32_t &row_bits) __attribute__((always_inline)) {
        if (!mask)
            return;
        if constexpr (GATE) {   // with f32 the first vector's keep bits wait for the second one's
            row_bits |= kept << ((j % VR) * EPV);
            if (j % VR == VR - 1) {
                mask[(int64_t)vec_pos(j, t) * (cols / 8) + octet] = (uint8_t)row_bits;
                row_bits = 0;
            }
        } else {
            const int64_t r = row0 + line0;
            if constexpr (EPV == 8)
                mask[r * (cols / 8) + vec_pos(j, t)] = (uint8_t)kept;
            else if ((tid & 1) == 0)   // see the caller: row_bits holds the neighbouring lane's half
                mask[r * (cols / 8) + vec_pos(j, t) / 2] = (uint8_t)(kept | (row_bits << 4));
        }
    };

    const uint32_t t = fresh_tid();
    // The common forms, every vector's code laid out: without fields B and C (keep iff A >= the
    // threshold's A) and with them.
    auto apply_fast = [&](auto with_bc_tag) __attribute__((always_inline)) {
        constexpr bool BC = decltype(with_bc_tag)::value;
        uint32_t sa[kLrLines], sb[kLrLines], sc[kLrLines];
        if constexpr (GATE) {
#pragma unroll
            for (int l = 0; l < kLrLines; ++l) {
                sa[l] = lr_uniform(state[l].a);
                sb[l] = BC ? lr_uniform(state[l].b) : 0u;
                sc[l] = BC ? lr_uniform(state[l].c) : 0u;
            }
        }
        uint32_t row_bits = 0;
#pragma unroll
        for (int j = 0; j < VPT; ++j) {
            __builtin_amdgcn_sched_barrier(0);
            const int line0 = vec_line0(j);
            const bool valid = vec_valid(j, t);
            uint32_t kept = 0;
            if (valid) {
                const int l0 = line0 & (kLrLines - 1);
                const uint32_t da = GATE ? 0u : lr_uniform(state[l0].a);
                const uint32_t db = GATE || !BC ? 0u : lr_uniform(state[l0].b);
                const uint32_t dc = GATE || !BC ? 0u : lr_uniform(state[l0].c);
                float fs[EPV];
                vec_factors(j, t, line0, fs);
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    const float w = fabsf(elem_of<DT>(v[j], e));
                    const float p = w * fs[e];
                    const uint32_t a = __float_as_uint(p);
                    const uint32_t ta = GATE ? sa[line0 + e] : da;
                    bool keep;
                    if constexpr (BC) {
                        const uint32_t tb = GATE ? sb[line0 + e] : db, tc = GATE ? sc[line0 + e] : dc;
                        const uint32_t b = lr_mono(fmaf(w, fs[e], -p));
                        const uint32_t c = 0xFFFFu - (GATE ? vec_pos(j, t) : vec_pos(j, t) * EPV + e);
                        keep = (a > ta) | ((a == ta) & ((b > tb) | ((b == tb) & (c >= tc))));
                    } else {
                        keep = a >= ta;
                    }
                    zero_lane_if<DT>(v[j], e, !keep);
                    kept |= (keep ? 1u : 0u) << e;
                }
                if constexpr (GATE)   // neighbouring workgroups write the other parts of the same 128 bytes: let L2 merge them
                    *reinterpret_cast<u32x4 *>(vec_addr(j, t)) = v[j];
                else
                    __builtin_nontemporal_store(v[j], reinterpret_cast<u32x4 *>(vec_addr(j, t)));
            }
            if (!GATE && EPV == 4)
                row_bits = __shfl_xor(kept, 1, 64);
            if (valid)
                write_mask(j, t, line0, kept, row_bits);
        }
    };
    if (!exact && !beyond_a) {
        apply_fast(std::false_type{});
    } else if (!exact) {
        apply_fast(std::true_type{});
    } else {
        uint32_t row_bits = 0;
#pragma clang loop unroll(disable)
        for (int j = 0; j < VPT; ++j) {
            const int line0 = vec_line0(j);
            const bool valid = vec_valid(j, t);
            uint32_t kept = 0;
            if (valid) {
                u32x4 x = *reinterpret_cast<const u32x4 *>(vec_addr(j, t));
#pragma clang loop unroll(disable)
                for (int e = 0; e < EPV; ++e) {
                    const int line = GATE ? line0 + e : line0;
                    const uint32_t idx = GATE ? vec_pos(j, t) : vec_pos(j, t) * EPV + e;
                    uint32_t a, b;
                    fields(elem_at(x, e), factor_at(j, t, e, line), norm_index(j, t, e, line), true, a, b);
                    const bool keep = lr_keep(state[line], a, b, 0xFFFFu - idx);
                    zero_at_if(x, e, !keep);
                    kept |= (keep ? 1u : 0u) << e;
                }
                *reinterpret_cast<u32x4 *>(vec_addr(j, t)) = x;
            }
            if (!GATE && EPV == 4)
                row_bits = __shfl_xor(kept, 1, 64);
            if (valid)
                write_mask(j, t, line0, kept, row_bits);
        }
    }
}

// ---------------------------------------------------------------- transpose --
// Column lines too long for one workgroup's registers (more than 16384 rows of bf16) are
// selected on a transposed copy, where they are row lines: dst[c, r] = src[r, c], 64 x 64
// element tiles through LDS, 16-byte accesses on both sides (8 consecutive lanes cover 128
// contiguous bytes of a row).  The LDS row stride in dwords is odd, so that the column gather of
// the second phase spreads over the banks.
template <int DT>
__global__ __launch_bounds__(256) void transpose_kernel(const void *__restrict__ srcv, int64_t rows, int64_t cols,
                                                        int64_t ld, void *__restrict__ dstv, int64_t ldd,
                                                        uint32_t tiles_c, const uint32_t *__restrict__ gate)
{
    if (gate && *gate == 0)
        return;   // the launches before this one have done the work (uniform)
    constexpr int EPV = DT == DASS_BF16 ? 8 : 4;
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    constexpr int TS = 64, VPR = TS / EPV;
    constexpr int ROW_DW = TS * EB / 4 + 1;
    __shared__ uint32_t tile[TS * ROW_DW];
    const int64_t r0 = (int64_t)(blockIdx.x / tiles_c) * TS, c0 = (int64_t)(blockIdx.x % tiles_c) * TS;
    const char *src = static_cast<const char *>(srcv);
    char *dst = static_cast<char *>(dstv);
    for (int v = threadIdx.x; v < TS * VPR; v += 256) {
        const int r = v / VPR, cv = v % VPR;
        if (r0 + r < rows && c0 + cv * EPV < cols) {   // rows and cols are multiples of EPV: whole vectors
            const u32x4 x = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4 *>(src + ((r0 + r) * ld + c0 + cv * EPV) * EB));
#pragma unroll
            for (int i = 0; i < 4; ++i)
                tile[r * ROW_DW + cv * 4 + i] = x[i];
        }
    }
    __syncthreads();
    for (int v = threadIdx.x; v < TS * VPR; v += 256) {
        const int rg = v % VPR, c = v / VPR;   // destination row c0 + c, its vector of source rows rg * EPV ..
        if (c0 + c < cols && r0 + rg * EPV < rows) {
            u32x4 x;
            if constexpr (DT == DASS_BF16) {
                const uint16_t *t16 = reinterpret_cast<const uint16_t *>(tile);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    x[i] = (uint32_t)t16[(rg * EPV + 2 * i) * ROW_DW * 2 + c] |
                           (uint32_t)t16[(rg * EPV + 2 * i + 1) * ROW_DW * 2 + c] << 16;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    x[i] = tile[(rg * EPV + i) * ROW_DW + c];
            }
            __builtin_nontemporal_store(x, reinterpret_cast<u32x4 *>(dst + ((c0 + c) * ldd + r0 + rg * EPV) * EB));
        }
    }
}

// Launch plan of the resident kernel for a matrix, or fits = false.
struct ResidentPlan {
    bool fits;
    int vpl_log2, lpb;
    int64_t grid;
    size_t smem;
};
static ResidentPlan plan_resident(int64_t rows, int64_t cols, int64_t ld, int dt, bool gate, bool along)
{
    ResidentPlan p{false, 0, kLrLines, 0, 0};
    const int epv = vec_elems(dt);
    const int64_t len = gate ? rows : cols;
    if (len > 0xFFFF)
        return p;
    if (gate) {   // a thread holds 8 / epv vectors of every 1024th row
        p.fits = (rows + kLrThreads - 1) / kLrThreads * (8 / epv) <= kLrVecs;
        p.grid = (cols / 8 + 63) / 64 * 64;
    } else {      // a thread holds 2^vpl_log2 vectors of each of its workgroup's lines
        const int64_t vpl = (cols / epv + kLrThreads - 1) / kLrThreads;
        while ((1 << p.vpl_log2) < vpl && p.vpl_log2 < 5)
            ++p.vpl_log2;
        p.fits = (1 << p.vpl_log2) <= kLrVecs;
        if (p.fits && kLrVecs >> p.vpl_log2 < p.lpb)
            p.lpb = kLrVecs >> p.vpl_log2;
        p.grid = (rows + p.lpb - 1) / p.lpb;
    }
    p.smem = (size_t)p.lpb * kLrBins * 4 + kLrLines * sizeof(LrState) + 16 + 256 + kLrLines * 4 +
             kLrLines * kLrTies * 8 + (along ? (size_t)len : (size_t)kLrLines) * sizeof(float);
    p.fits = p.fits && p.grid <= 0x7fffffffLL && p.smem <= 160 * 1024 &&
             rows * ld * elem_bytes(dt) < (1LL << 32);
    return p;
}

static dass_status launch_resident(const char *fn, const ResidentPlan &p, void *W, int64_t rows, int64_t cols,
                                   int64_t ld, int dt, const float *norms, bool col_lines, bool along, int fmode,
                                   uint32_t n_keep, uint8_t *mask_out, const uint32_t *gate, uint32_t gate_rows,
                                   hipStream_t stream)
{
    using k_t = void (*)(void *, int64_t, int64_t, int64_t, const float *, int, uint32_t, uint8_t *, int, int,
                         const uint32_t *, uint32_t);
    k_t k;
    if (dt == DASS_BF16)
        k = col_lines ? (along ? unstructured_resident_kernel<DASS_BF16, kLrGate, true>
                          : unstructured_resident_kernel<DASS_BF16, kLrGate, false>)
                 : (along ? unstructured_resident_kernel<DASS_BF16, kLrDown, true>
                          : unstructured_resident_kernel<DASS_BF16, kLrDown, false>);
    else
        k = col_lines ? (along ? unstructured_resident_kernel<DASS_F32, kLrGate, true>
                          : unstructured_resident_kernel<DASS_F32, kLrGate, false>)
                 : (along ? unstructured_resident_kernel<DASS_F32, kLrDown, true>
                          : unstructured_resident_kernel<DASS_F32, kLrDown, false>);
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)p.smem) != hipSuccess)
        return fail(DASS_ERR_HIP, "%s: cannot reserve %zu bytes of LDS", fn, p.smem);
    hipLaunchKernelGGL(k, dim3((unsigned)p.grid), dim3(kLrThreads), p.smem, stream, W, rows, cols, ld, norms, fmode,
                       n_keep, mask_out, p.vpl_log2, p.lpb, gate, gate_rows);
    return check_launch("unstructured kernel");
}

// Column lines that do not fit the resident kernel but would as row lines of the transposed
// matrix [cols, rows]: the plan for that matrix (leading dimension rows), or fits = false.
static ResidentPlan plan_transposed(int64_t rows, int64_t cols, int dt, bool along)
{
    if (rows % vec_elems(dt) != 0)
        return ResidentPlan{false, 0, 0, 0, 0};
    return plan_resident(cols, rows, rows, dt, false, along);
}

}  // namespace dass

extern "C" size_t dass_unstructured_workspace_bytes(int64_t rows, int64_t cols, dass_dtype dt,
                                                    dass_axis norm_axis, dass_axis group_axis)
{
    using namespace dass;
    const int64_t n = norm_axis == DASS_AXIS_ROWS ? rows : cols;
    if (n <= 0 || rows <= 0 || cols <= 0)
        return 0;
    // the factor vector, one flag word (in a block of its own), then room that the column-line paths share:
    size_t bytes = round_up((size_t)n * sizeof(float), 256) + kFlagBytes, extra = 0;
    if (valid_dtype(dt) && group_axis == DASS_AXIS_ROWS && cols % 8 == 0) {
        const bool along = norm_axis == group_axis;
        // long column lines are selected on a transposed copy of the matrix
        if (!plan_resident(rows, cols, cols, dt, true, along).fits && plan_transposed(rows, cols, dt, along).fits)
            extra = (size_t)rows * (size_t)cols * elem_bytes(dt);
        // the streaming passes over 64-column tiles keep their counts and lists there
        const TiledPlan tp = along ? plan_tiled(rows, cols, cols, dt) : TiledPlan{};
        if (tp.fits && tp.bytes > extra)
            extra = tp.bytes;
    }
    if (valid_dtype(dt) && group_axis == DASS_AXIS_COLS && norm_axis == DASS_AXIS_COLS && cols % 8 == 0) {
        const RowlinesPlan rp = plan_rowlines(rows, cols, cols, dt);   // one word per block of rows
        if (rp.fits)
            extra = rp.todo_bytes;
    }
    return bytes + extra;
}

namespace dass {

// The selection itself, shared by the two entry points.  `workspace_needed` is what the caller's
// contract asks for; a workspace that holds the factor vector but not the transposed copy sends
// long column lines to the multi-pass kernels.
static dass_status score_mask_unstructured_impl(const char *fn, void *W, int64_t rows, int64_t cols, int64_t ld,
                                                dass_dtype dt, const float *norms, dass_axis norm_axis,
                                                dass_axis group_axis, double alpha, int64_t n_prune,
                                                uint8_t *mask_out, void *workspace, size_t workspace_bytes,
                                                size_t workspace_needed, void *hip_stream)
{
    dass_status s = check_score_args(fn, W, rows, cols, ld, dt, norms, norm_axis, group_axis, alpha, workspace,
                                     workspace_bytes, workspace_needed);
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
    const uint32_t n_keep = (uint32_t)(len - n_prune);
    const bool bf16 = dt == DASS_BF16;
    const size_t f_bytes = round_up((size_t)(norm_axis == DASS_AXIS_ROWS ? rows : cols) * sizeof(float), 256);
    // room behind the factor vector and the flag word, if the caller's workspace has it
    char *const region = static_cast<char *>(workspace) + f_bytes + kFlagBytes;
    const size_t region_bytes = workspace_bytes > f_bytes + kFlagBytes ? workspace_bytes - f_bytes - kFlagBytes : 0;
    const uint32_t *gate = nullptr;   // set: the launches below run only where the word(s) it points to are nonzero
    uint32_t gate_rows = 0;           // 0: one word for the whole matrix; else one word per block of so many rows

    // Column lines in the DaSS configuration (the factor varies along the line, exponent 0.5 or 1):
    // streaming passes over 64-column tiles.  They decide every ordinary matrix; for what they do
    // not decide they leave W untouched and set the flag, and the launches below, which then run
    // behind that flag, redo the matrix.
    if ((alpha == 0.5 || alpha == 1.0) && group_axis == DASS_AXIS_ROWS && norm_axis == DASS_AXIS_ROWS && n_keep > 0 &&
        n_keep < (uint32_t)len) {
        const TiledPlan tp = plan_tiled(rows, cols, ld, dt, mask_out);
        if (tp.fits && region_bytes >= tp.bytes) {
            uint32_t *flag = reinterpret_cast<uint32_t *>(static_cast<char *>(workspace) + f_bytes);
            s = launch_tiled(fn, tp, W, rows, cols, ld, dt, norms, alpha == 1.0 ? kFactorNorm : kFactorSqrt, n_keep,
                             mask_out, flag, region, stream);
            if (s != DASS_OK)
                return s;
            gate = flag;
        }
    }
    // Row lines in the DaSS configuration: one launch in which a workgroup owns 8 whole rows; blocks of
    // rows it does not decide are marked and redone by the launches below.
    if ((alpha == 0.5 || alpha == 1.0) && group_axis == DASS_AXIS_COLS && norm_axis == DASS_AXIS_COLS && n_keep > 0 &&
        n_keep < (uint32_t)len) {
        const RowlinesPlan rp = plan_rowlines(rows, cols, ld, dt, mask_out);
        if (rp.fits && region_bytes >= rp.todo_bytes) {
            uint32_t *todo = reinterpret_cast<uint32_t *>(region);
            s = launch_rowlines(fn, rp, W, rows, cols, ld, dt, norms, alpha == 1.0 ? kFactorNorm : kFactorSqrt, n_keep,
                                mask_out, todo, stream);
            if (s != DASS_OK)
                return s;
            gate = todo;
            gate_rows = kRowlinesBlock;
        }
    }

    // Lines that fit the registers of one workgroup, exponent with an exact f32 factor: the
    // weights are read once.
    if ((alpha == 0.0 || alpha == 0.5 || alpha == 1.0) && len <= 0xFFFF && n_keep > 0 && n_keep < (uint32_t)len) {
        const int fmode = alpha == 0.0 ? kFactorOne : alpha == 1.0 ? kFactorNorm : kFactorSqrt;
        const bool along = norm_axis == group_axis;
        const bool col_lines = group_axis == DASS_AXIS_ROWS;
        const ResidentPlan p = plan_resident(rows, cols, ld, dt, col_lines, along);
        if (p.fits)
            return launch_resident(fn, p, W, rows, cols, ld, dt, norms, col_lines, along, fmode, n_keep, mask_out, gate,
                                   gate_rows, stream);
        // Longer column lines: transpose into the workspace, select there along the rows, transpose
        // back.  (No mask in this form: its bits would come out transposed.)
        const ResidentPlan pt =
            col_lines && !mask_out ? plan_transposed(rows, cols, dt, along) : ResidentPlan{false, 0, 0, 0, 0};
        if (pt.fits && region_bytes >= (size_t)rows * cols * elem_bytes(dt)) {
            void *Wt = region;
            const int64_t tiles_r = (rows + 63) / 64, tiles_c = (cols + 63) / 64;
            if (tiles_r * tiles_c > 0x7fffffffLL)
                return fail(DASS_ERR_SHAPE, "%s: too many tiles for one launch", fn);
            auto tk = bf16 ? transpose_kernel<DASS_BF16> : transpose_kernel<DASS_F32>;
            hipLaunchKernelGGL(tk, dim3((unsigned)(tiles_r * tiles_c)), dim3(256), 0, stream, (const void *)W, rows,
                               cols, ld, Wt, rows, (uint32_t)tiles_c, gate);
            s = check_launch("transpose kernel");
            if (s != DASS_OK)
                return s;
            s = launch_resident(fn, pt, Wt, cols, rows, rows, dt, norms, false, along, fmode, n_keep, nullptr, gate, 0, stream);
            if (s != DASS_OK)
                return s;
            hipLaunchKernelGGL(tk, dim3((unsigned)(tiles_r * tiles_c)), dim3(256), 0, stream, (const void *)Wt, cols,
                               rows, rows, W, ld, (uint32_t)tiles_r, gate);
            return check_launch("transpose kernel");
        }
    }

    float *f = static_cast<float *>(workspace);
    s = launch_factor(norms, norm_axis == DASS_AXIS_ROWS ? rows : cols, alpha, f, stream);
    if (s != DASS_OK)
        return s;

    const dim3 grid((unsigned)blocks), block(kUBlock);
    if (group_axis == DASS_AXIS_COLS) {
        auto k = bf16 ? (norm_axis == DASS_AXIS_COLS ? unstructured_cols_kernel<DASS_BF16, true>
                                                     : unstructured_cols_kernel<DASS_BF16, false>)
                      : (norm_axis == DASS_AXIS_COLS ? unstructured_cols_kernel<DASS_F32, true>
                                                     : unstructured_cols_kernel<DASS_F32, false>);
        hipLaunchKernelGGL(k, grid, block, 0, stream, W, rows, cols, ld, (const float *)f, n_keep,
                           mask_out, gate, gate_rows);
    } else {
        auto k = bf16 ? (norm_axis == DASS_AXIS_ROWS ? unstructured_rows_kernel<DASS_BF16, true>
                                                     : unstructured_rows_kernel<DASS_BF16, false>)
                      : (norm_axis == DASS_AXIS_ROWS ? unstructured_rows_kernel<DASS_F32, true>
                                                     : unstructured_rows_kernel<DASS_F32, false>);
        hipLaunchKernelGGL(k, grid, block, 0, stream, W, rows, cols, ld, (const float *)f, n_keep,
                           mask_out, gate);
    }
    return check_launch("unstructured kernel");
}

// ---- device memory of the library's own, for dass_score_mask_unstructured_static ----------
// The factor vector f = norms^alpha of one call: every GPU the library runs on holds this array
// until the process ends.  In host code the array's name is only a handle: its address on the
// current device comes from hipGetSymbolAddress, once per device, and is what kernels are given.
constexpr int64_t kStaticFactors = 65536;
static __device__ __align__(256) float scratch[kStaticFactors];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static float *scratch_ptr[kMaxDevices] = {nullptr};

// Address of `scratch` on the current device (looked up on the first call on that device).
static dass_status static_scratch(const char *fn, float **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return fail(DASS_ERR_HIP, "%s: hipGetDevice: %s", fn, hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(DASS_ERR_HIP, "%s: device ordinal %d outside 0..%d", fn, dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(DASS_ERR_HIP, "%s: hipGetSymbolAddress: %s", fn, hipGetErrorString(e));
        scratch_ptr[dev] = static_cast<float *>(p);
    }
    *out = scratch_ptr[dev];
    return DASS_OK;
}

}  // namespace dass

extern "C" dass_status dass_score_mask_unstructured(void *W, int64_t rows, int64_t cols, int64_t ld,
                                                    dass_dtype dt, const float *norms,
                                                    dass_axis norm_axis, dass_axis group_axis,
                                                    double alpha, int64_t n_prune,
                                                    uint8_t *mask_out, void *workspace,
                                                    size_t workspace_bytes, void *hip_stream)
{
    return dass::score_mask_unstructured_impl("dass_score_mask_unstructured", W, rows, cols, ld, dt, norms, norm_axis,
                                              group_axis, alpha, n_prune, mask_out, workspace, workspace_bytes,
                                              dass_unstructured_workspace_bytes(rows, cols, dt, norm_axis, group_axis),
                                              hip_stream);
}

extern "C" dass_status dass_score_mask_unstructured_static(void *W, int64_t rows, int64_t cols, int64_t ld,
                                                           dass_dtype dt, const float *norms,
                                                           dass_axis norm_axis, dass_axis group_axis,
                                                           double alpha, int64_t n_prune, uint8_t *mask_out,
                                                           void *hip_stream)
{
    using namespace dass;
    const char *fn = "dass_score_mask_unstructured_static";
    const int64_t n_norms = norm_axis == DASS_AXIS_ROWS ? rows : cols;
    if (n_norms > kStaticFactors)
        return fail(DASS_ERR_WORKSPACE, "%s: %lld norms exceed the %lld the library's own scratch holds; use "
                    "dass_score_mask_unstructured with a workspace", fn, (long long)n_norms, (long long)kStaticFactors);
    float *f = nullptr;
    const dass_status s = static_scratch(fn, &f);
    if (s != DASS_OK)
        return s;
    const size_t need = n_norms > 0 ? round_up((size_t)n_norms * sizeof(float), 256) : 0;
    return score_mask_unstructured_impl(fn, W, rows, cols, ld, dt, norms, norm_axis, group_axis, alpha, n_prune,
                                        mask_out, f, sizeof(float) * (size_t)kStaticFactors, need, hip_stream);
}
