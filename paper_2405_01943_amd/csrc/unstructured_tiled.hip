// Stage 2, unstructured, column lines (Sec. 3 "Pruning Granularity": the weights of Gate-Proj and
// Up-Proj that connect to one input form a comparison group, i.e. a column of the [d_int, d]
// matrix, stride ld), for the DaSS configuration: the factor norm^alpha varies along the line
// (Eq. 4), alpha = 0.5 or 1.
//
// A column is far longer than anything one lane can hold and 2 bytes wide in memory, so a
// workgroup that owns whole columns reads 16-byte pieces of 128-byte lines.  Here a workgroup
// owns a tile instead - 64 columns (whole 128-byte lines of bf16) x a slab of rows - and the
// selection is done by streaming passes over the matrix, which stays in the 256 MB memory-side
// cache between them:
//
//   window   per column, 128 sampled scores give two order statistics that bracket the wanted
//            quantile by six standard deviations of the sample rank: the window [lo, lo + 256 << sh)
//            on the bit pattern of the leading score term p (non-negative floats order like their
//            bits).  The same launch writes the scaled factor vector.
//   hist     every tile counts its scores into 256 window bins + "above" per column (LDS
//            atomics) and stores its counts; no global atomics, the result is reproducible.
//   scan     per column the slabs' counts are added and the bin that holds the n_keep-th largest
//            score is found: a range of p a few dozen scores wide, and the rank wanted inside it.
//   apply    second pass: every weight whose p lies below the threshold's bin becomes +0 and whole
//            128-byte lines are written once; the scores inside the bin stay for now and are
//            listed as (A, B, C) = (bits of p, the error term q in order-preserving form,
//            0xFFFF - row): lexicographic order of these triples is (exact score descending, row
//            ascending), as in unstructured.hip.
//   fix      one wavefront per column ranks its list; the entries below the wanted rank are
//            zeroed one by one (a few dozen 2-byte stores per column).
//
// The window is a statistical guess, the bins and the list have fixed sizes: a column whose
// threshold falls outside the window, whose bin holds more scores than the list (thousands of
// equal scores), or a factor or product outside the range in which p + q is the exact score
// sets one flag.  The apply pass then writes nothing and the caller's gated launches (the
// line-resident kernel or the multi-pass kernels) redo the matrix: the result is exact either
// way, only the time differs.  (A flag raised after the apply pass - a list that came out
// shorter than its count, which identical arithmetic in both passes rules out - finds a matrix
// in which only weights below every threshold are zero already: the redo selects the same set.)
#include "select.h"
#include "unstructured_tiled.h"

namespace dass {
namespace tiled {

constexpr int kCols = 64;               // columns of a tile
constexpr int kBins = 256;              // window bins
constexpr int kSlots = kBins + 2;       // [0] below the window, [1 .. 256] the bins ascending, [257] above
constexpr int kStride = kSlots + 1;     // LDS counters per column (odd: columns start on different banks)
constexpr int kSamples = 128;           // sampled rows per column
constexpr int kCap = 256;               // listed scores per column
constexpr int kThreads = 1024;          // hist, collect, apply
constexpr int kWinCols = 8;             // columns per workgroup of the window kernel: two per wavefront
constexpr uint32_t kInfBits = 0x7f800000u;
// Bits of the flag word: why the passes left the matrix to the caller's other kernels.
enum : uint32_t {
    kWhyRange = 1,      // a factor or a product outside the range of the two-term score
    kWhyWindow = 2,     // a column's threshold lies outside its sampled window
    kWhyBin = 4,        // the threshold's bin holds more scores than a list
    kWhyList = 8,       // a list overflowed
    kWhyCount = 16,     // a list is not as long as the counts said (never seen; checked all the same)
};

struct Window {   // per column
    uint32_t lo, sh;
};
struct Select {   // per column: the threshold's bin [lo, lo + width) of p and the rank wanted inside it
    uint32_t lo;       // weights with p below this are pruned
    uint32_t width;    // 0: every score of the bin is kept, nothing to list
    uint32_t need, inside;
};
struct Entry {    // a listed score; the threshold has the same form
    uint32_t a, b, c, pad;
};

__device__ __forceinline__ uint32_t mono(float q)   // unsigned integer that grows with q
{
    const uint32_t b = __float_as_uint(q);
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}

// Row sampled for slot k of kSamples: one per stratum of rows / kSamples rows, at an offset that
// changes from stratum to stratum (a fixed offset would alias with periodic row patterns).
__device__ __forceinline__ uint32_t sample_row(uint32_t k, uint32_t rows)
{
    const uint32_t stratum = rows / kSamples;
    const uint32_t base = (uint32_t)(((uint64_t)k * rows) / kSamples);
    const uint32_t r = base + (stratum ? ((k * 2654435761u) >> 8) % stratum : 0u);
    return r < rows ? r : rows - 1;
}

// ------------------------------------------------------------------ window --
// Blocks [0, win_blocks): 8 columns each, one wavefront per 2 columns.  Blocks after those: the
// scaled factor vector, 256 rows each.  Block 0 clears the flag and every window block the
// list counters of its columns.
template <int DT>
__global__ __launch_bounds__(256) void window_kernel(const void *__restrict__ Wv, uint32_t rows, uint32_t cols,
                                                     int64_t ld, const float *__restrict__ norms, int fmode,
                                                     uint32_t n_keep, uint32_t win_blocks, float *__restrict__ fs,
                                                     Window *__restrict__ win, uint32_t *__restrict__ cnt,
                                                     uint32_t *__restrict__ flag)
{
    constexpr int EPV = DT == DASS_BF16 ? 8 : 4;
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    constexpr int VPR = kWinCols / EPV;   // vectors per sampled row
    __shared__ uint32_t smp[kWinCols][kSamples + 1];
    const int tid = threadIdx.x;
    if (blockIdx.x >= win_blocks) {
        const uint32_t i = (blockIdx.x - win_blocks) * 256u + tid;
        if (i < rows)
            fs[i] = factor_of(norms[i], fmode) * kFactorScale;
        return;
    }
    if (blockIdx.x == 0 && tid == 0)
        *flag = 0;
    const uint32_t c0 = blockIdx.x * kWinCols;
    const char *W = static_cast<const char *>(Wv);
    for (int v = tid; v < kSamples * VPR; v += 256) {
        const uint32_t k = v / VPR, piece = v % VPR, c = c0 + piece * EPV;
        u32x4 x = u32x4{0, 0, 0, 0};
        const uint32_t r = sample_row(k, rows);
        if (c < cols)
            x = *reinterpret_cast<const u32x4 *>(W + ((int64_t)r * ld + c) * EB);
        const float f = factor_of(norms[r], fmode) * kFactorScale;
#pragma unroll
        for (int e = 0; e < EPV; ++e)
            smp[piece * EPV + e][k] = __float_as_uint(fabsf(elem_of<DT>(x, e)) * f);
    }
    __syncthreads();

    // Ranks (from the top) of the two order statistics: the wanted quantile of the sample, r_mid,
    // give or take six standard deviations of the number of sampled scores above the column's
    // threshold (a hypergeometric count, at most binomial in spread) and one more.
    const float phi = (float)n_keep / (float)rows;
    const float mid = phi * kSamples, dev = 6.0f * sqrtf(kSamples * phi * (1.0f - phi)) + 1.0f;
    const int r_hi = (int)floorf(mid - dev), r_lo = (int)ceilf(mid + dev);

    const int lane = tid & 63, wave = tid >> 6;
    for (int q = 0; q < kWinCols / 4; ++q) {
        const int cl = wave * (kWinCols / 4) + q;
        const uint32_t c = c0 + cl;
        if (c >= cols)
            break;   // uniform inside the wavefront
        const uint32_t s0 = smp[cl][lane], s1 = smp[cl][lane + 64];
        // the r-th largest sample, cut to its bits 30 .. 19 (a sixteenth of a binade): the largest T with r samples >= T
        auto order_stat = [&](int r) {
            uint32_t t = 0;
            for (int bit = 30; bit >= 19; --bit) {
                const uint32_t trial = t | (1u << bit);
                const int n = __popcll(__ballot(s0 >= trial)) + __popcll(__ballot(s1 >= trial));
                if (n >= r)
                    t = trial;
            }
            return t;
        };
        // An end beyond the sample: the sample's extreme serves if the chance that the threshold lies beyond
        // it, phi^128 or (1 - phi)^128, is below 1e-9; else the window is open at that end.
        const bool lo_open = r_lo > kSamples && phi > 0.85f, hi_open = r_hi < 1 && phi < 0.15f;
        const uint32_t lo = lo_open ? 0u : order_stat(r_lo <= kSamples ? r_lo : kSamples);
        const uint32_t hi = hi_open ? kInfBits - 1u : (order_stat(r_hi >= 1 ? r_hi : 1) | 0x7ffffu);
        const uint32_t span = hi - lo;   // lo <= hi: r_lo > r_hi
        const int width = 32 - __clz((int)span | 1);
        if (lane == 0) {
            win[c] = Window{lo, (uint32_t)(width > 8 ? width - 8 : 0)};
            cnt[c] = 0;
        }
    }
}

// Per-thread view of a tile: LPR lanes cover the 64 columns of a row with one 16-byte vector
// each, RPI rows per trip of the workgroup.
template <int DT>
struct Tile {
    static constexpr int EPV = DT == DASS_BF16 ? 8 : 4;
    static constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    static constexpr int LPR = kCols / EPV;
    static constexpr int RPI = kThreads / LPR;
    static constexpr int UNROLL = 4;
};

// -------------------------------------------------------------------- hist --
template <int DT>
__global__ __launch_bounds__(kThreads) void hist_kernel(const void *__restrict__ Wv, uint32_t rows, uint32_t cols,
                                                        int64_t ld, const float *__restrict__ fs,
                                                        const Window *__restrict__ win, uint32_t groups,
                                                        uint32_t slab_rows, uint32_t *__restrict__ part,
                                                        uint32_t *__restrict__ flag)
{
    using TL = Tile<DT>;
    constexpr int EPV = TL::EPV, EB = TL::EB, LPR = TL::LPR, RPI = TL::RPI, U = TL::UNROLL;
    extern __shared__ uint32_t hist[];   // [kCols][kStride]: more than a launch gets without asking
    const int tid = threadIdx.x;
    const uint32_t g = blockIdx.x % groups, slab = blockIdx.x / groups;
    const uint32_t piece = tid % LPR, r_in = tid / LPR;
    const uint32_t c0 = g * kCols + piece * EPV;
    const bool active = c0 < cols;
    for (int i = tid; i < kCols * kStride; i += kThreads)
        hist[i] = 0;

    uint32_t lo[EPV], sh[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) {
        const Window w = active ? win[c0 + e] : Window{0, 0};
        lo[e] = w.lo;
        sh[e] = w.sh;
    }
    __syncthreads();

    const uint32_t r_begin = slab * slab_rows, r_end = r_begin + slab_rows < rows ? r_begin + slab_rows : rows;
    const char *W = static_cast<const char *>(Wv) + (size_t)c0 * EB;
    uint32_t *const mine = hist + piece * EPV * kStride + 1;   // slot 1 of the thread's first column
    bool bad = false;
    uint32_t a_max = 0;
    if (active) {
        for (uint32_t r = r_begin + r_in; r < r_end; r += U * RPI) {
            u32x4 x[U];
            float f[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t ru = r + u * RPI;
                if (ru < r_end) {
                    x[u] = *reinterpret_cast<const u32x4 *>(W + (int64_t)ru * ld * EB);
                    f[u] = fs[ru];
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (r + u * RPI < r_end) {
                    // a factor outside the range of the two-term score: 0 < f' < 2^23, or f' infinite
                    bad |= !(f[u] == 0.0f || (f[u] >= kFactorMin * kFactorScale && f[u] < __uint_as_float(kInfBits)));
#pragma unroll
                    for (int e = 0; e < EPV; ++e) {
                        const uint32_t a = __float_as_uint(fabsf(elem_of<DT>(x[u], e)) * f[u]);
                        a_max = a > a_max ? a : a_max;
                        int bin = (int)(a - lo[e]) >> sh[e];            // negative below the window
                        bin = bin < -1 ? -1 : bin > kBins ? kBins : bin;   // -1: below, kBins: above
                        atomicAdd(mine + e * kStride + bin, 1u);
                    }
                }
            }
        }
    }
    if (bad || a_max >= kInfBits)   // a product that overflowed
        atomicOr(flag, kWhyRange);
    __syncthreads();
    // the tile's counts, two 16-bit counters a word (a slab has fewer than 65536 rows)
    uint32_t *out = part + ((size_t)slab * groups + g) * (kCols * kSlots / 2);
    for (int i = tid; i < kCols * kSlots / 2; i += kThreads) {
        const int c = i / (kSlots / 2), s = i % (kSlots / 2);
        out[i] = hist[c * kStride + 2 * s] | hist[c * kStride + 2 * s + 1] << 16;
    }
}

// -------------------------------------------------------------------- scan --
// One wavefront per column; lane l owns bins 255 - 4 l .. 252 - 4 l, so a prefix sum over the
// lanes counts from the top.
__global__ __launch_bounds__(256) void scan_kernel(const uint16_t *__restrict__ part, const Window *__restrict__ win,
                                                   uint32_t cols, uint32_t groups, uint32_t slabs, uint32_t n_keep,
                                                   Select *__restrict__ sel, uint32_t *__restrict__ flag)
{
    const int lane = threadIdx.x & 63;
    const uint32_t c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= cols)
        return;
    const size_t col_stride = kSlots, slab_stride = (size_t)groups * kCols * kSlots;
    const uint16_t *p = part + (size_t)c * col_stride;
    uint32_t h[4] = {0, 0, 0, 0}, above = 0;
    for (uint32_t s = 0; s < slabs; ++s) {
        const uint16_t *q = p + s * slab_stride;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            h[j] += q[1 + 255 - 4 * lane - j];
        above += q[kSlots - 1];
    }
    const uint32_t sum = h[0] + h[1] + h[2] + h[3];
    uint32_t incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t u = __shfl_up(incl, o, 64);
        if (lane >= o)
            incl += u;
    }
    uint32_t excl = incl - sum;
    const Window w = win[c];
    bool found = false;
    uint32_t bin = 0, need = 0, inside = 0;
    if (n_keep > above) {
        const uint32_t want = n_keep - above;
        if (excl < want && want <= incl) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (!found && want <= excl + h[j]) {
                    found = true;
                    bin = 255 - 4 * lane - j;
                    need = want - excl;
                    inside = h[j];
                }
                excl += h[j];
            }
        }
    }
    const uint64_t who = __ballot(found);
    if (who == 0 || __shfl(inside, __ffsll((long long)who) - 1, 64) > (uint32_t)kCap) {
        // the threshold is not inside the window, or its bin holds more than a list does
        if (lane == 0) {
            atomicOr(flag, who == 0 ? kWhyWindow : kWhyBin);
            sel[c] = Select{0, 0, 0, 0};
        }
        return;
    }
    if (found) {
        const uint32_t lo = w.lo + (bin << w.sh);
        if (need == inside)   // every score of the bin is wanted: its lower edge is the threshold
            sel[c] = Select{lo, 0, 0, 0};
        else
            sel[c] = Select{lo, 1u << w.sh, need, inside};
    }
}

// ------------------------------------------------------------------- apply --
// Nothing is shared between rows here, so the matrix is covered by many small workgroups whose
// threads make one trip each (streams faster than resident workgroups that loop): 256 threads take
// 4 row blocks of a tile, a thread one 16-byte vector of each (measured, a whole 7B model's 96
// matrices one after the other: 7.35 ms with 3 or 4 vectors per thread, 7.45 with 2, 7.5 with 6,
// 7.6 with 8).  A score inside its column's bin
// is rare (a few dozen per column): the workgroup gathers them in LDS (up to kLocal per column)
// and moves them to the columns' lists at the end, one global counter update per column; what
// does not fit goes to the list directly.
constexpr int kApplyThreads = 256, kApplyTrips = 4, kLocal = 8;

template <int DT, bool MASK>
__global__ __launch_bounds__(kApplyThreads) void apply_kernel(void *__restrict__ Wv, uint32_t rows, uint32_t cols,
                                                              int64_t ld, const float *__restrict__ fs,
                                                              const Select *__restrict__ sel, uint32_t groups,
                                                              uint32_t *__restrict__ cnt, Entry *__restrict__ list,
                                                              uint8_t *__restrict__ mask, uint32_t *__restrict__ flag)
{
    constexpr int EPV = DT == DASS_BF16 ? 8 : 4;
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    constexpr int LPR = kCols / EPV, RPI = kApplyThreads / LPR, U = kApplyTrips;
    __shared__ uint32_t found[kCols];
    __shared__ uint32_t base[kCols];
    __shared__ uint32_t held[kCols][kLocal][3];
    __shared__ uint2 bins[kCols];   // (lo, width) of the tile's columns
    __shared__ uint32_t stop;       // the flag as one thread read it: the same answer for the whole workgroup
    const int tid = threadIdx.x;
    const uint32_t g = blockIdx.x % groups, block = blockIdx.x / groups;
    if (tid < kCols) {
        const Select t = g * kCols + tid < cols ? sel[g * kCols + tid] : Select{0, 0, 0, 0};
        bins[tid] = make_uint2(t.lo, t.width);
        found[tid] = 0;
    }
    if (tid == kCols)
        stop = *flag;
    const uint32_t piece = tid % LPR, r0 = block * (U * RPI) + tid / LPR;
    const uint32_t c0 = g * kCols + piece * EPV;
    const bool active = c0 < cols;
    char *W = static_cast<char *>(Wv) + (size_t)c0 * EB;
    u32x4 x[U];
    float f[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t ru = r0 + u * RPI;
        if (active && ru < rows) {
            x[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(W + (int64_t)ru * ld * EB));
            f[u] = fs[ru];
        }
    }
    __syncthreads();
    if (stop)
        return;   // the matrix is left as it was for the gated launches that follow
    uint32_t lo[EPV], width[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) {
        const uint2 t = bins[piece * EPV + e];
        lo[e] = t.x;
        width[e] = t.y;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t ru = r0 + u * RPI;
        const bool live = active && ru < rows;
        uint32_t kept = 0;
        if (live) {
            // d = bits(p) - lo is negative (both are below 2^31) exactly for a pruned weight; its sign,
            // spread over the word, is the mask that clears the weight.  Whether any of the vector's scores
            // lies inside its column's bin is one flag per lane; which ones is asked only then.
            uint32_t d[EPV];
            int32_t gone[EPV];
            bool hit = false;
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                d[e] = __float_as_uint(fabsf(elem_of<DT>(x[u], e)) * f[u]) - lo[e];
                hit |= d[e] < width[e];
                gone[e] = (int32_t)d[e] >> 31;
                if constexpr (MASK)
                    kept |= (uint32_t)(~gone[e] & 1) << e;
            }
            if (hit) {   // rarely entered
                uint32_t hits = 0;
#pragma unroll
                for (int e = 0; e < EPV; ++e)
                    hits |= (d[e] < width[e] ? 1u : 0u) << e;
                while (hits) {
                    const int e = __ffs((int)hits) - 1;
                    hits &= hits - 1;
                    float w = 0.0f;
#pragma unroll
                    for (int k = 0; k < EPV; ++k)
                        w = k == e ? fabsf(elem_of<DT>(x[u], k)) : w;
                    const float p = w * f[u];
                    const uint32_t a = __float_as_uint(p), b = mono(fmaf(w, f[u], -p)), c = 0xFFFFu - ru;
                    const uint32_t col = piece * EPV + e;
                    const uint32_t slot = atomicAdd(&found[col], 1u);
                    if (slot < (uint32_t)kLocal) {
                        held[col][slot][0] = a;
                        held[col][slot][1] = b;
                        held[col][slot][2] = c;
                    } else {   // more of them in one workgroup than it holds: straight to the list
                        const uint32_t at = atomicAdd(cnt + g * kCols + col, 1u);
                        if (at < (uint32_t)kCap)
                            list[(size_t)(g * kCols + col) * kCap + at] = Entry{a, b, c, 0};
                        else
                            atomicOr(flag, kWhyList);
                    }
                }
            }
            if constexpr (DT == DASS_BF16) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t clear = ((uint32_t)gone[2 * k] & 0xffffu) | ((uint32_t)gone[2 * k + 1] & 0xffff0000u);
                    x[u][k] &= ~clear;
                }
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    x[u][k] &= ~(uint32_t)gone[k];
            }
            __builtin_nontemporal_store(x[u], reinterpret_cast<u32x4 *>(W + (int64_t)ru * ld * EB));
        }
        if constexpr (MASK) {
            if constexpr (EPV == 8) {
                if (live)
                    mask[(size_t)ru * (cols / 8) + c0 / 8] = (uint8_t)kept;
            } else {
                // f32: a mask byte covers two lanes' vectors of one row; the two share every branch up to here
                const uint32_t other = __shfl_xor(kept, 1, 64);
                if (live && (piece & 1) == 0)
                    mask[(size_t)ru * (cols / 8) + c0 / 8] = (uint8_t)(kept | other << 4);
            }
        }
    }
    __syncthreads();
    if (tid < kCols) {
        const uint32_t n = found[tid] < (uint32_t)kLocal ? found[tid] : (uint32_t)kLocal;
        base[tid] = n ? atomicAdd(cnt + g * kCols + tid, n) : 0u;
    }
    __syncthreads();
    for (int i = tid; i < kCols * kLocal; i += kApplyThreads) {
        const uint32_t col = i / kLocal, k = i % kLocal;
        const uint32_t n = found[col] < (uint32_t)kLocal ? found[col] : (uint32_t)kLocal;
        if (k < n) {
            const uint32_t at = base[col] + k;
            if (at < (uint32_t)kCap)
                list[(size_t)(g * kCols + col) * kCap + at] = Entry{held[col][k][0], held[col][k][1], held[col][k][2], 0};
            else
                atomicOr(flag, kWhyList);
        }
    }
}

// --------------------------------------------------------------------- fix --
// One wavefront per column ranks the column's list: an entry with `need` or more entries above
// it is pruned after all - its weight becomes +0 and its mask bit is cleared.  Lane l holds
// entries l, l + 64, ..; every entry in turn is read out of its lane's registers and compared by
// all lanes (no memory in the loop: it is a chain of dependent steps).
// The mask bit is cleared with a 32-bit atomic (entries of neighbouring columns share bytes): the
// host takes this path only for a mask that is made of whole aligned words.
template <int DT>
__global__ __launch_bounds__(256) void fix_kernel(void *__restrict__ Wv, uint32_t cols, int64_t ld,
                                                  const Select *__restrict__ sel, const uint32_t *__restrict__ cnt,
                                                  const Entry *__restrict__ list, uint8_t *__restrict__ mask,
                                                  uint32_t *__restrict__ flag)
{
    const int lane = threadIdx.x & 63;
    const uint32_t c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= cols)
        return;
    // four loads that do not wait for one another (each is a trip to memory another kernel wrote)
    const uint32_t stop = *flag;
    Select s = sel[c];
    uint32_t n = cnt[c];
    Entry mine[kCap / 64];
    mine[0] = list[(size_t)c * kCap + lane];   // past the list's end: stale or never written, not used
    // the same for every lane of the wavefront: say so, the loops below then run on the scalar unit
    n = __builtin_amdgcn_readfirstlane(n);
    s.width = __builtin_amdgcn_readfirstlane(s.width);
    s.need = __builtin_amdgcn_readfirstlane(s.need);
    s.inside = __builtin_amdgcn_readfirstlane(s.inside);
    if (stop || s.width == 0)
        return;   // the passes have given up, or every score of the bin is kept
    if (n != s.inside) {   // ruled out by identical arithmetic in hist and apply; never trust it silently
        if (lane == 0)
            atomicOr(flag, kWhyCount);
        return;
    }
#pragma unroll
    for (int j = 1; j < kCap / 64; ++j) {
        const uint32_t k = lane + 64 * j;
        mine[j] = k < n ? list[(size_t)c * kCap + k] : Entry{0, 0, 0, 0};
    }
    // Ranking on (A, B) as one 64-bit number; C (the row) is looked at only where two entries agree in
    // both, which a second sweep settles if it happens at all.
    uint64_t key[kCap / 64];
#pragma unroll
    for (int j = 0; j < kCap / 64; ++j)
        key[j] = (uint64_t)mine[j].a << 32 | mine[j].b;
    uint32_t above[kCap / 64] = {0, 0, 0, 0}, same[kCap / 64] = {0, 0, 0, 0};
    const int slots = (int)((n + 63) / 64);   // uniform: 1 for an ordinary column
#pragma unroll
    for (int src = 0; src < kCap / 64; ++src) {
        if (src >= slots)
            break;
        const int in_slot = (int)n - 64 * src < 64 ? (int)n - 64 * src : 64;
        for (int k = 0; k < in_slot; ++k) {
            const uint64_t o = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)mine[src].a, k) << 32 |
                               (uint32_t)__builtin_amdgcn_readlane((int)mine[src].b, k);
#pragma unroll
            for (int j = 0; j < kCap / 64; ++j)
                if (j < slots) {
                    above[j] += o > key[j];
                    same[j] += o == key[j];
                }
        }
    }
    bool tied = false;   // an entry counts itself once
#pragma unroll
    for (int j = 0; j < kCap / 64; ++j)
        tied |= lane + 64 * j < n && same[j] > 1;
    if (__ballot(tied)) {
#pragma unroll
        for (int src = 0; src < kCap / 64; ++src) {
            if (src >= slots)
                break;
            const int in_slot = (int)n - 64 * src < 64 ? (int)n - 64 * src : 64;
            for (int k = 0; k < in_slot; ++k) {
                const uint64_t o = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)mine[src].a, k) << 32 |
                                   (uint32_t)__builtin_amdgcn_readlane((int)mine[src].b, k);
                const uint32_t oc = (uint32_t)__builtin_amdgcn_readlane((int)mine[src].c, k);
#pragma unroll
                for (int j = 0; j < kCap / 64; ++j)
                    if (j < slots)
                        above[j] += (o == key[j]) & (oc > mine[j].c);
            }
        }
    }
    char *W = static_cast<char *>(Wv);
#pragma unroll
    for (int j = 0; j < kCap / 64; ++j) {
        if (lane + 64 * j < n && above[j] >= s.need) {   // ranks need + 1 and below
            const uint32_t row = 0xFFFFu - mine[j].c;
            if constexpr (DT == DASS_BF16)
                *reinterpret_cast<uint16_t *>(W + ((int64_t)row * ld + c) * 2) = 0;
            else
                *reinterpret_cast<uint32_t *>(W + ((int64_t)row * ld + c) * 4) = 0;
            if (mask) {
                const size_t byte = (size_t)row * (cols / 8) + c / 8;
                atomicAnd(reinterpret_cast<uint32_t *>(mask) + byte / 4, ~(1u << ((byte % 4) * 8 + c % 8)));
            }
        }
    }
}

}  // namespace tiled

TiledPlan plan_tiled(int64_t rows, int64_t cols, int64_t ld, int dt, const uint8_t *mask_out)
{
    using namespace tiled;
    TiledPlan p{};
    p.fits = false;
    if (mask_out && ((reinterpret_cast<uintptr_t>(mask_out) & 3u) != 0 || (rows * (cols / 8)) % 4 != 0))
        return p;
    // column lines long enough for a 128-row sample to say something, matrices large enough for six launches to pay
    if (rows < 1024 || rows > 0xFFFF || cols % 8 != 0 || cols > (1 << 24) || rows * cols < (1LL << 21) ||
        rows * ld * elem_bytes(dt) >= (1LL << 40))
        return p;
    p.groups = (cols + kCols - 1) / kCols;
    // One workgroup per compute unit (256 of them) and never a few left over for a second round; two
    // per compute unit where a workgroup would otherwise stream more than 8192 rows (measured: 7B
    // 87 -> 83 us, Gemma-7B 167 -> 155 us with one, the 70B layer 425 -> 415 us with two).  Fewer slabs
    // also mean fewer counts to write and to add up.  Slabs of at least 256 rows.
    int64_t slabs = 256 / p.groups;
    if (slabs < 1)
        slabs = 1;
    if (rows / slabs > 8192 && 512 / p.groups > slabs)
        slabs = 512 / p.groups;
    if (slabs > rows / 256)
        slabs = rows / 256;
    if (slabs < 1)
        slabs = 1;
    p.slab_rows = (rows + slabs - 1) / slabs;
    p.slabs = (int)((rows + p.slab_rows - 1) / p.slab_rows);
    if (p.groups * p.slabs > 0x7fffffffLL)
        return p;
    const size_t padded_cols = (size_t)p.groups * kCols;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += round_up(bytes, 256);
        return at;
    };
    p.off_fs = take((size_t)rows * sizeof(float));
    p.off_win = take(padded_cols * sizeof(Window));
    p.off_part = take((size_t)p.slabs * padded_cols * kSlots * sizeof(uint16_t));
    p.off_sel = take(padded_cols * sizeof(Select));
    p.off_cnt = take(padded_cols * sizeof(uint32_t));
    p.off_list = take(padded_cols * kCap * sizeof(Entry));
    p.bytes = off;
    p.fits = true;
    return p;
}

dass_status launch_tiled(const char *fn, const TiledPlan &p, void *W, int64_t rows, int64_t cols, int64_t ld, int dt,
                         const float *norms, int fmode, uint32_t n_keep, uint8_t *mask_out, uint32_t *flag,
                         void *region, hipStream_t stream)
{
    using namespace tiled;
    char *base = static_cast<char *>(region);
    float *fs = reinterpret_cast<float *>(base + p.off_fs);
    Window *win = reinterpret_cast<Window *>(base + p.off_win);
    uint32_t *part = reinterpret_cast<uint32_t *>(base + p.off_part);
    Select *sel = reinterpret_cast<Select *>(base + p.off_sel);
    uint32_t *cnt = reinterpret_cast<uint32_t *>(base + p.off_cnt);
    Entry *list = reinterpret_cast<Entry *>(base + p.off_list);
    const bool bf16 = dt == DASS_BF16;
    const uint32_t r32 = (uint32_t)rows, c32 = (uint32_t)cols, groups = (uint32_t)p.groups,
                   slab_rows = (uint32_t)p.slab_rows, slabs = (uint32_t)p.slabs;
    const uint32_t win_blocks = (c32 + kWinCols - 1) / kWinCols, fs_blocks = (r32 + 255) / 256;
    const dim3 tiles(groups * slabs), per_col((c32 + 3) / 4);

    hipLaunchKernelGGL(bf16 ? window_kernel<DASS_BF16> : window_kernel<DASS_F32>, dim3(win_blocks + fs_blocks), dim3(256),
                       0, stream, (const void *)W, r32, c32, ld, norms, fmode, n_keep, win_blocks, fs, win, cnt, flag);
    constexpr size_t hist_lds = (size_t)kCols * kStride * sizeof(uint32_t);
    auto hk = bf16 ? hist_kernel<DASS_BF16> : hist_kernel<DASS_F32>;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(hk), hipFuncAttributeMaxDynamicSharedMemorySize, (int)hist_lds) !=
        hipSuccess)
        return fail(DASS_ERR_HIP, "%s: cannot reserve %zu bytes of LDS", fn, hist_lds);
    hipLaunchKernelGGL(hk, tiles, dim3(kThreads), hist_lds, stream,
                       (const void *)W, r32, c32, ld, (const float *)fs, (const Window *)win, groups, slab_rows, part, flag);
    hipLaunchKernelGGL(scan_kernel, per_col, dim3(256), 0, stream, (const uint16_t *)part, (const Window *)win, c32, groups,
                       slabs, n_keep, sel, flag);
    const uint32_t rows_per_block = kApplyTrips * kApplyThreads / (bf16 ? 8 : 16);
    auto ak = bf16 ? (mask_out ? apply_kernel<DASS_BF16, true> : apply_kernel<DASS_BF16, false>)
                   : (mask_out ? apply_kernel<DASS_F32, true> : apply_kernel<DASS_F32, false>);
    hipLaunchKernelGGL(ak, dim3(groups * ((r32 + rows_per_block - 1) / rows_per_block)), dim3(kApplyThreads), 0, stream, W,
                       r32, c32, ld, (const float *)fs, (const Select *)sel, groups, cnt, list, mask_out, flag);
    hipLaunchKernelGGL(bf16 ? fix_kernel<DASS_BF16> : fix_kernel<DASS_F32>, per_col, dim3(256), 0, stream, W, c32, ld,
                       (const Select *)sel, (const uint32_t *)cnt, (const Entry *)list, mask_out, flag);
    return check_launch("tiled unstructured kernels");
}

}  // namespace dass
