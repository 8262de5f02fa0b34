// Stage 2, unstructured, row lines (Sec. 3 "Pruning Granularity": the weights of Down-Proj that
// feed one output form a comparison group, a row of the [d, d_int] matrix), for the DaSS
// configuration: the factor varies along the line (Eq. 5: the norms of the intermediate
// activations run along the row), alpha = 0.5 or 1.
//
// The scheme of unstructured_tiled.hip - a sampled window on the bit pattern of the leading score
// term p, 256 bins inside it, the threshold's bin, an apply pass that lists the few scores inside
// that bin, a ranking of the list - with whole lines owned by one workgroup: nothing is merged
// between workgroups, so all of it is ONE launch.  A workgroup of 1024 threads takes 8 rows and
//   0  clears its counters,
//   A  samples 128 positions of each row (one wavefront per row): the row's window,
//   B  streams its rows (read 1) and counts into 8 x 256 LDS bins (+ side counters); the scaled
//      factors of the columns are computed into LDS first - all of them if 44 KB hold them,
//      else chunk by chunk of columns, each chunk ahead of the part of the rows that needs it,
//      so that two workgroups fit a compute unit's LDS whatever the line length,
//   C  finds each row's bin (one wavefront per row),
//   D  streams its rows again (read 2, out of the memory-side cache), zeroes what lies below the
//      bin, writes whole lines once, and lists the scores inside the bin in LDS,
//   E  ranks each row's list (one wavefront per row) and zeroes the entries below the wanted rank.
// What this does not decide for one of the 8 rows (a factor or product outside the range of the
// two-term score, a threshold outside the window, more scores in the bin than the list holds)
// leaves all 8 rows untouched and marks the block in `todo`; the caller's next launch, gated
// per block, redoes those rows.
#include "select.h"
#include "unstructured_tiled.h"

namespace dass {
namespace rowl {

constexpr int kRows = kRowlinesBlock;   // rows per workgroup
constexpr int kThreads = 1024;
constexpr int kBins = 256;
// Counters of a row: [0 .. 255] the bins ascending, then 64 counters for scores above the window and 64
// for scores below it, one per lane: a fifth of a row's scores lies on either side, and 64 lanes
// adding to one LDS word take turns.
constexpr int kAbove = kBins, kBelow = kBins + 64;
constexpr int kStride = kBins + 128;
constexpr int kSamples = 128;
constexpr int kCap = 256;               // listed scores per row
constexpr int kU = 4;                   // vectors a thread has in flight while counting
constexpr int kUD = 2;                  // and in the apply pass (two workgroups share a compute unit only
                                        // if a thread takes at most 64 registers; four vectors there take 72)
constexpr uint32_t kInfBits = 0x7f800000u;

struct Window {
    uint32_t lo, sh;
};
// The columns are taken in `count` chunks of `vecs` 16-byte vectors (the last one `last_vecs`); the
// magic numbers are ceil(2^32 / vecs) and ceil(2^32 / last_vecs) for the division by multiply-high.
struct Chunks {
    uint32_t count, vecs, last_vecs, magic, last_magic;
};
struct Select {
    uint32_t lo, width, need, inside;
};

__device__ __forceinline__ uint32_t mono(float q)   // unsigned integer that grows with q
{
    const uint32_t b = __float_as_uint(q);
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}

// The 128 sampled positions of a row are 16 runs of 8 consecutive columns (a sample spread one by one
// would touch 128 of the row's 172 memory lines: most of the matrix, just to sample it): run k
// lies in the k-th sixteenth of the row, at an offset that changes from run to run.  Returns the
// run's first column, a multiple of 8.
constexpr int kRuns = kSamples / 8;
__device__ __forceinline__ uint32_t sample_run(uint32_t k, uint32_t cols)
{
    const uint32_t octets = cols / 8, stratum = octets / kRuns;   // cols >= 1024: stratum >= 8
    const uint32_t o = (uint32_t)(((uint64_t)k * octets) / kRuns) + ((k * 2654435761u) >> 8) % stratum;
    return (o < octets ? o : octets - 1) * 8;
}

// Layout of the dynamic LDS, in bytes from its start.
struct Smem {
    size_t fs, hist, list, cnt, win, sel, fail, bytes;
};
__host__ __device__ inline Smem smem_layout(uint32_t chunk_cols)
{
    Smem m;
    size_t off = 0;
    m.fs = off;
    off += ((size_t)chunk_cols * 4 + 15) / 16 * 16;
    // the counters are dead once the bins are found (phase C), the lists are filled after that: one place for both
    m.hist = m.list = off;
    off += (size_t)kRows * (kCap * 12 > kStride * 4 ? kCap * 12 : kStride * 4);
    m.cnt = off;
    off += kRows * 4;
    m.win = off;
    off += kRows * sizeof(Window);
    m.sel = off;
    off += kRows * sizeof(Select);
    m.fail = off;
    off += 16;
    m.bytes = off;
    return m;
}

// (two workgroups of 1024 threads share a compute unit when a thread takes at most 64 registers)
template <int DT, bool MASK>
__global__ __launch_bounds__(kThreads) void rowlines_kernel(void *__restrict__ Wv, uint32_t rows, uint32_t cols,
                                                            int64_t ld, const float *__restrict__ norms, int fmode,
                                                            uint32_t n_keep, const Chunks ck,
                                                            uint8_t *__restrict__ mask, uint32_t *__restrict__ todo)
{
    constexpr int EPV = DT == DASS_BF16 ? 8 : 4;
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const Smem m = smem_layout(ck.vecs * EPV);
    float *fs = reinterpret_cast<float *>(smem + m.fs);
    uint32_t *hist = reinterpret_cast<uint32_t *>(smem + m.hist);
    uint32_t *list = reinterpret_cast<uint32_t *>(smem + m.list);   // [kRows][kCap][3]
    uint32_t *cnt = reinterpret_cast<uint32_t *>(smem + m.cnt);
    Window *win = reinterpret_cast<Window *>(smem + m.win);
    Select *sel = reinterpret_cast<Select *>(smem + m.sel);
    uint32_t *fail = reinterpret_cast<uint32_t *>(smem + m.fail);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t row0 = blockIdx.x * kRows;
    const uint32_t n_rows = rows - row0 < (uint32_t)kRows ? rows - row0 : (uint32_t)kRows;
    char *W = static_cast<char *>(Wv) + (size_t)row0 * ld * EB;
    const uint32_t row_bytes = (uint32_t)ld * EB;   // the block's 8 rows span less than 4 GB (host check)

    // the rows' samples (phase A, one wavefront per row) are fetched first: they are on their way
    // while phase 0 runs.  Their factors come straight from the norms.
    float smp_w[2] = {0.0f, 0.0f}, smp_n[2] = {0.0f, 0.0f};
    if ((uint32_t)wave < n_rows) {   // lane l: columns 2 (l % 4), + 1 of run l / 4
        const uint32_t c = sample_run(lane / 4, cols) + 2 * (lane % 4);
        if constexpr (DT == DASS_BF16) {
            const uint32_t two = *reinterpret_cast<const uint32_t *>(W + wave * row_bytes + c * 2);
            smp_w[0] = __uint_as_float(two << 16);
            smp_w[1] = __uint_as_float(two & 0xffff0000u);
        } else {
            const float2 two = *reinterpret_cast<const float2 *>(W + wave * row_bytes + c * 4);
            smp_w[0] = two.x;
            smp_w[1] = two.y;
        }
        const float2 n2 = *reinterpret_cast<const float2 *>(norms + c);
        smp_n[0] = n2.x;
        smp_n[1] = n2.y;
    }

    // ---- 0: counters cleared
    for (int i = tid; i < kRows * kStride; i += kThreads)
        hist[i] = 0;
    if (tid < kRows)
        cnt[tid] = 0;
    if (tid == 0)
        *fail = 0;
    __syncthreads();

    // ---- A: the rows' windows, one wavefront per row
    if ((uint32_t)wave < n_rows) {
        uint32_t s[2];
#pragma unroll
        for (int q = 0; q < 2; ++q)
            s[q] = __float_as_uint(fabsf(smp_w[q]) * (factor_of(smp_n[q], fmode) * kFactorScale));
        // Ranks (from the top) of the two order statistics: the wanted quantile of the sample give or
        // take six standard deviations of the sampled count above the threshold, and one more.
        const float phi = (float)n_keep / (float)cols;
        const float mid = phi * kSamples, dev = 6.0f * sqrtf(kSamples * phi * (1.0f - phi)) + 1.0f;
        const int r_hi = (int)floorf(mid - dev), r_lo = (int)ceilf(mid + dev);
        // the r-th largest sample, cut to its bits 30 .. 19: the largest T with r samples >= T
        auto order_stat = [&](int r) {
            uint32_t t = 0;
            for (int bit = 30; bit >= 19; --bit) {
                const uint32_t trial = t | (1u << bit);
                const int n = __popcll(__ballot(s[0] >= trial)) + __popcll(__ballot(s[1] >= trial));
                if (n >= r)
                    t = trial;
            }
            return t;
        };
        // an end beyond the sample: the sample's extreme serves if the chance that the threshold lies
        // beyond it, phi^128 or (1 - phi)^128, is below 1e-9; else the window is open at that end
        const bool lo_open = r_lo > kSamples && phi > 0.85f, hi_open = r_hi < 1 && phi < 0.15f;
        const uint32_t lo = lo_open ? 0u : order_stat(r_lo <= kSamples ? r_lo : kSamples);
        const uint32_t hi = hi_open ? kInfBits - 1u : (order_stat(r_hi >= 1 ? r_hi : 1) | 0x7ffffu);
        const int width = 32 - __clz((int)(hi - lo) | 1);
        if (lane == 0)
            win[wave] = Window{lo, (uint32_t)(width > 8 ? width - 8 : 0)};
    }
    __syncthreads();

    // Scaled factors of chunk ch into LDS (cols is a multiple of 8, norms are 16-byte aligned).  The
    // barriers around it are the caller's.
    bool bad = false;
    auto stage = [&](uint32_t ch) {
        const uint32_t c_begin = ch * ck.vecs * EPV, n = (ch == ck.count - 1 ? ck.last_vecs : ck.vecs) * EPV;
        for (uint32_t j = 4 * tid; j < n; j += 4 * kThreads) {
            const u32x4 n4 = *reinterpret_cast<const u32x4 *>(norms + c_begin + j);
            u32x4 f4;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float f = factor_of(__uint_as_float(n4[i]), fmode);
                bad |= !factor_in_fast_range(f);
                f4[i] = __float_as_uint(f * kFactorScale);
            }
            *reinterpret_cast<u32x4 *>(fs + j) = f4;
        }
    };
    // Vector v of a chunk's flat list (the block's rows x the chunk's vectors) -> (row, vector inside the
    // chunk); v < 2^17 and the divisor < 2^14, so the multiply-high by ceil(2^32 / divisor) is the exact quotient.
    auto split = [&](uint32_t v, uint32_t n_vecs, uint32_t magic, uint32_t &row, uint32_t &cv) {
        row = __umulhi(v, magic);
        cv = v - row * n_vecs;
    };
    auto factors = [&](uint32_t cv, float *f) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < EPV / 4; ++q) {
            const u32x4 x = *reinterpret_cast<const u32x4 *>(fs + cv * EPV + 4 * q);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                f[4 * q + i] = __uint_as_float(x[i]);
        }
    };

    // ---- B: counts
    uint32_t a_max = 0;
    for (uint32_t ch = 0; ch < ck.count; ++ch) {
    const uint32_t n_vecs = ch == ck.count - 1 ? ck.last_vecs : ck.vecs, magic = ch == ck.count - 1 ? ck.last_magic : ck.magic;
    const uint32_t total = n_rows * n_vecs, chunk_bytes = ch * ck.vecs * 16;
    if (ch > 0)
        __syncthreads();   // the previous chunk's factors are no longer read
    stage(ch);
    __syncthreads();
    for (uint32_t v0 = tid; v0 < total; v0 += kU * kThreads) {
        u32x4 x[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const uint32_t v = v0 + u * kThreads;
            if (v < total) {
                uint32_t row, cv;
                split(v, n_vecs, magic, row, cv);
                x[u] = *reinterpret_cast<const u32x4 *>(W + row * row_bytes + chunk_bytes + cv * 16);
            }
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            asm volatile("" ::: "memory");       // one vector's factors in registers at a time: no LDS read
            __builtin_amdgcn_sched_barrier(0);   // moves up past this line
            if (v0 + u * kThreads < total) {
                uint32_t row, cv;   // again, rather than kept in registers across the loads
                split(v0 + u * kThreads, n_vecs, magic, row, cv);
                float f[EPV];
                factors(cv, f);
                const Window w = win[row];
                uint32_t *const mine = hist + row * kStride;
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    const uint32_t a = __float_as_uint(fabsf(elem_of<DT>(x[u], e)) * f[e]);
                    a_max = a > a_max ? a : a_max;
                    int bin = (int)(a - w.lo) >> w.sh;   // negative below the window, 256 or more above it
                    bin = bin < 0 ? kBelow + lane : bin >= kBins ? kAbove + lane : bin;
                    atomicAdd(mine + bin, 1u);
                }
            }
        }
    }
    }
    if (bad || a_max >= kInfBits)   // a factor outside the range of the two-term score, a product that overflowed
        *fail = 1;
    __syncthreads();

    // ---- C: each row's bin; lane l owns bins 255 - 4 l .. 252 - 4 l, a prefix sum over the lanes counts from the top
    if ((uint32_t)wave < n_rows) {
        const uint32_t *h_row = hist + wave * kStride;
        uint32_t h[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            h[j] = h_row[255 - 4 * lane - j];
        uint32_t above = h_row[kAbove + lane];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1)
            above += __shfl_xor(above, o, 64);
        const uint32_t sum = h[0] + h[1] + h[2] + h[3];
        uint32_t incl = sum;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t t = __shfl_up(incl, o, 64);
            if (lane >= o)
                incl += t;
        }
        uint32_t excl = incl - sum;
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
            if (lane == 0)
                *fail = 1;   // threshold outside the window, or more scores in its bin than the list holds
        } else if (found) {
            const Window w = win[wave];
            const uint32_t lo = w.lo + (bin << w.sh);
            sel[wave] = need == inside ? Select{lo, 0, 0, 0} : Select{lo, 1u << w.sh, need, inside};
        }
    }
    __syncthreads();
    if (*fail) {   // uniform: the rows stay as they are for the launch that follows
        if (tid == 0)
            todo[blockIdx.x] = 1;
        return;
    }

    // ---- D: apply and list
    for (uint32_t ch = 0; ch < ck.count; ++ch) {
    const uint32_t n_vecs = ch == ck.count - 1 ? ck.last_vecs : ck.vecs, magic = ch == ck.count - 1 ? ck.last_magic : ck.magic;
    const uint32_t total = n_rows * n_vecs, chunk_bytes = ch * ck.vecs * 16, chunk_vec0 = ch * ck.vecs;
    if (ck.count > 1) {   // one chunk: the factors are still there
        __syncthreads();
        stage(ch);
        __syncthreads();
    }
    for (uint32_t v0 = tid; v0 < total; v0 += kUD * kThreads) {
        u32x4 x[kUD];
#pragma unroll
        for (int u = 0; u < kUD; ++u) {
            const uint32_t v = v0 + u * kThreads;
            if (v < total) {
                uint32_t row, cv;
                split(v, n_vecs, magic, row, cv);
                x[u] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4 *>(W + row * row_bytes + chunk_bytes + cv * 16));
            }
        }
#pragma unroll
        for (int u = 0; u < kUD; ++u) {
            const bool live = v0 + u * kThreads < total;
            asm volatile("" ::: "memory");       // one vector's factors in registers at a time: no LDS read
            __builtin_amdgcn_sched_barrier(0);   // moves up past this line
            uint32_t kept = 0, row = 0, cv = 0;
            if (live)
                split(v0 + u * kThreads, n_vecs, magic, row, cv);
            if (live) {
                float f[EPV];
                factors(cv, f);
                const Select t = sel[row];
                uint32_t hits = 0;
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    const uint32_t d = __float_as_uint(fabsf(elem_of<DT>(x[u], e)) * f[e]) - t.lo;   // negative: pruned
                    hits |= (d < t.width ? 1u : 0u) << e;
                    kept |= ((int32_t)d >= 0 ? 1u : 0u) << e;
                }
                while (hits) {   // rarely entered: a few dozen scores per row
                    const int e = __ffs((int)hits) - 1;
                    hits &= hits - 1;
                    float w = 0.0f, fe = 0.0f;
#pragma unroll
                    for (int k = 0; k < EPV; ++k) {
                        w = k == e ? fabsf(elem_of<DT>(x[u], k)) : w;
                        fe = k == e ? f[k] : fe;
                    }
                    const float p = w * fe;
                    const uint32_t slot = atomicAdd(&cnt[row], 1u);
                    if (slot < (uint32_t)kCap) {
                        uint32_t *entry = list + (row * kCap + slot) * 3;
                        entry[0] = __float_as_uint(p);
                        entry[1] = mono(fmaf(w, fe, -p));
                        entry[2] = 0xFFFFu - ((chunk_vec0 + cv) * EPV + e);
                    }
                }
#pragma unroll
                for (int e = 0; e < EPV; ++e)
                    zero_lane_if<DT>(x[u], e, ((kept >> e) & 1u) == 0);
                __builtin_nontemporal_store(x[u], reinterpret_cast<u32x4 *>(W + row * row_bytes + chunk_bytes + cv * 16));
            }
            if constexpr (MASK) {
                if constexpr (EPV == 8) {
                    if (live)
                        mask[(size_t)(row0 + row) * (cols / 8) + chunk_vec0 + cv] = (uint8_t)kept;
                } else {
                    // f32: a mask byte covers two neighbouring lanes' vectors (vpl is even, the two share every branch)
                    const uint32_t other = __shfl_xor(kept, 1, 64);
                    if (live && (cv & 1) == 0)
                        mask[(size_t)(row0 + row) * (cols / 8) + (chunk_vec0 + cv) / 2] = (uint8_t)(kept | other << 4);
                }
            }
        }
    }
    }
    // The 2-byte stores of E go to lines written just above by other wavefronts of this workgroup.  The
    // barrier orders them: it carries a workgroup-scope release (every store above has been accepted by
    // L2, where stores to one address stay in order).  A device-scope fence here would write back and
    // invalidate the XCD's whole L2 once per workgroup (measured: 170 us per matrix).
    __syncthreads();

    // ---- E: rank each row's list; an entry with `need` or more entries above it is pruned after all
    bool short_list = false;
    if ((uint32_t)wave < n_rows && sel[wave].width != 0) {
        const uint32_t n = __builtin_amdgcn_readfirstlane(cnt[wave] < (uint32_t)kCap ? cnt[wave] : (uint32_t)kCap);
        const uint32_t need = __builtin_amdgcn_readfirstlane(sel[wave].need);
        short_list = cnt[wave] != sel[wave].inside;   // ruled out by identical arithmetic in B and D; checked all the same
        const uint32_t *mine_list = list + wave * kCap * 3;
        uint32_t ma[kCap / 64], mb[kCap / 64], mc[kCap / 64];
        uint64_t key[kCap / 64];
#pragma unroll
        for (int j = 0; j < kCap / 64; ++j) {
            const uint32_t k = lane + 64 * j;
            ma[j] = k < n ? mine_list[k * 3] : 0u;
            mb[j] = k < n ? mine_list[k * 3 + 1] : 0u;
            mc[j] = k < n ? mine_list[k * 3 + 2] : 0u;
            key[j] = (uint64_t)ma[j] << 32 | mb[j];
        }
        uint32_t above[kCap / 64] = {0, 0, 0, 0};
        const int slots = (int)((n + 63) / 64);
#pragma unroll
        for (int src = 0; src < kCap / 64; ++src) {
            if (src >= slots)
                break;
            const int in_slot = (int)n - 64 * src < 64 ? (int)n - 64 * src : 64;
            for (int k = 0; k < in_slot; ++k) {
                const uint64_t o = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)ma[src], k) << 32 |
                                   (uint32_t)__builtin_amdgcn_readlane((int)mb[src], k);
                const uint32_t oc = (uint32_t)__builtin_amdgcn_readlane((int)mc[src], k);
#pragma unroll
                for (int j = 0; j < kCap / 64; ++j)
                    if (j < slots)
                        above[j] += (o > key[j]) | ((o == key[j]) & (oc > mc[j]));
            }
        }
#pragma unroll
        for (int j = 0; j < kCap / 64; ++j) {
            if (lane + 64 * j < n && above[j] >= need) {
                const uint32_t c = 0xFFFFu - mc[j];
                if constexpr (DT == DASS_BF16)
                    *reinterpret_cast<uint16_t *>(W + wave * row_bytes + c * 2) = 0;
                else
                    *reinterpret_cast<uint32_t *>(W + wave * row_bytes + c * 4) = 0;
                if constexpr (MASK) {
                    const size_t byte = (size_t)(row0 + wave) * (cols / 8) + c / 8;
                    atomicAnd(reinterpret_cast<uint32_t *>(mask) + byte / 4, ~(1u << ((byte % 4) * 8 + c % 8)));
                }
            }
        }
    }
    // A short list leaves only weights below the threshold zeroed: redoing the rows selects the same set.
    if (__syncthreads_or(short_list) && tid == 0)
        todo[blockIdx.x] = 1;
    else if (tid == 0)
        todo[blockIdx.x] = 0;
}

}  // namespace rowl

RowlinesPlan plan_rowlines(int64_t rows, int64_t cols, int64_t ld, int dt, const uint8_t *mask_out)
{
    using namespace rowl;
    RowlinesPlan p{};
    p.fits = false;
    if (mask_out && ((reinterpret_cast<uintptr_t>(mask_out) & 3u) != 0 || (rows * (cols / 8)) % 4 != 0))
        return p;   // mask bits are corrected with 32-bit atomics
    // row lines long enough for a 128-position sample to say something, matrices large enough to fill the chip
    if (cols < 1024 || cols > 0xFFFF || cols % 8 != 0 || rows * cols < (1LL << 21) ||
        (int64_t)kRows * ld * elem_bytes(dt) >= (1LL << 32))
        return p;
    // columns in chunks of at most 11264 (44 KB of factors: with the lists, two workgroups per compute unit)
    p.chunks = (int)((cols + 11263) / 11264);
    p.chunk_cols = (cols / 8 + p.chunks - 1) / p.chunks * 8;
    p.smem = smem_layout((uint32_t)p.chunk_cols).bytes;
    p.blocks = (rows + kRows - 1) / kRows;
    if (p.blocks > 0x7fffffffLL)
        return p;
    p.todo_bytes = round_up((size_t)p.blocks * sizeof(uint32_t), 256);
    p.fits = true;
    return p;
}

dass_status launch_rowlines(const char *fn, const RowlinesPlan &p, void *W, int64_t rows, int64_t cols, int64_t ld, int dt,
                            const float *norms, int fmode, uint32_t n_keep, uint8_t *mask_out, uint32_t *todo,
                            hipStream_t stream)
{
    using namespace rowl;
    const bool bf16 = dt == DASS_BF16;
    auto k = bf16 ? (mask_out ? rowlines_kernel<DASS_BF16, true> : rowlines_kernel<DASS_BF16, false>)
                  : (mask_out ? rowlines_kernel<DASS_F32, true> : rowlines_kernel<DASS_F32, false>);
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.smem) !=
        hipSuccess)
        return fail(DASS_ERR_HIP, "%s: cannot reserve %zu bytes of LDS", fn, p.smem);
    const uint32_t vpl = (uint32_t)(cols / vec_elems(dt));
    Chunks ck;
    ck.count = (uint32_t)p.chunks;
    ck.vecs = (uint32_t)(p.chunk_cols / vec_elems(dt));
    ck.last_vecs = vpl - (ck.count - 1) * ck.vecs;
    ck.magic = (uint32_t)(((1ULL << 32) + ck.vecs - 1) / ck.vecs);
    ck.last_magic = (uint32_t)(((1ULL << 32) + ck.last_vecs - 1) / ck.last_vecs);
    hipLaunchKernelGGL(k, dim3((unsigned)p.blocks), dim3(kThreads), p.smem, stream, W, (uint32_t)rows, (uint32_t)cols, ld,
                       norms, fmode, n_keep, ck, mask_out, todo);
    return check_launch("row-line unstructured kernel");
}

}  // namespace dass
