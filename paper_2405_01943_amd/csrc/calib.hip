// Stage 1: calibration statistics.  For every intermediate neuron i
//     sumsq[i] (+)= sum_t ( act(x_t . Wgate_i) * (x_t . Wup_i) )^2
// i.e. the GLU product of Sec. 2.2 Eq. 2 reduced to the squared L2 norm that
// Sec. 3 uses as the group-importance indicator, over all calibration tokens.
// The two projections are dense contractions; y lives only in accumulators.
//
// bf16: MFMA kernels.  A workgroup owns a 256-token x 128-neuron tile and keeps
// a gate and an up accumulator for it (all 256 accumulator registers of its four
// wavefronts); X, Wgate and Wup slabs of BK columns are staged through LDS in
// 16-byte chunks, XOR-swizzled so that the 16-byte fragment reads of a wavefront
// spread over all banks.  Tokens are the MFMA "M" index and neurons the "N"
// index, so the 16 accumulator registers a lane holds for one 32x32 block belong
// to ONE neuron and 16 tokens: the sum over tokens starts as plain register
// adds, then one cross-lane add, then one f32 atomic per neuron and wavefront.
//   calib_pipe64_kernel  d a multiple of 64 (every model shape): slabs of 64
//                      columns go from global memory straight into a ring of
//                      five 32 KB LDS units (no register staging), whole
//                      128-byte lines per request; loads, fragment reads and
//                      MFMAs of consecutive slabs are interleaved by hand.  The
//                      same main loop also serves Eq. 2 + Eq. 3 themselves
//                      (dass_mlp_forward) through two storing epilogues.
//   calib_mfma_kernel  any other d (a multiple of 8): register-staged,
//                      double-buffered; the K tail is masked.
//
// f32: a plain LDS-tiled FMA kernel (small shapes).
#include "dass_internal.h"

#include <type_traits>

namespace dass {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // one 16-byte chunk = 8 bf16

// ------------------------------------------------------------- activations --
template <int ACT>
__device__ __forceinline__ float glu_act_fast(float g)
{
    // exp2 and the reciprocal are the hardware's 1-ulp instructions; a true division costs a
    // dozen instructions per element and the bf16 path is good to 1e-6 without it.
    if constexpr (ACT == DASS_ACT_SILU) {
        return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
    } else if constexpr (ACT == DASS_ACT_GELU_TANH) {
        // 0.5 g (1 + tanh z) = g / (1 + exp(-2 z)),  z = sqrt(2/pi) (g + 0.044715 g^3)
        // exp(-2 z) = exp2(g (c0 + c1 g^2)),  c0 = -2 sqrt(2/pi) log2(e),  c1 = 0.044715 c0
        const float e = g * fmaf(-0.10294324f, g * g, -2.3022082f);
        return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(e));
    } else if constexpr (ACT == DASS_ACT_GELU_ERF) {
        // erf by the classical five-term rational form in t = 1 / (1 + p z) times exp(-z^2)
        // (Abramowitz & Stegun 7.1.26, absolute error of erf below 1.5e-7), written on z = |g| / sqrt(2)
        // so that neither branch cancels: with h = (1 - erf z) / 2 = P(t) exp(-g^2 / 2) / 2,
        // GELU(g) = g (1 - h) for g >= 0 and g h for g < 0.  The library's erff is several times the
        // instructions; the norms are good to 1e-6 either way.
        const float t = __builtin_amdgcn_rcpf(fmaf(fabsf(g), 0.3275911f * 0.70710678f, 1.0f));
        float P = fmaf(t, 1.061405429f, -1.453152027f);
        P = fmaf(t, P, 1.421413741f);
        P = fmaf(t, P, -0.284496736f);
        P = fmaf(t, P, 0.254829592f);
        const float h = 0.5f * t * P * __builtin_amdgcn_exp2f(g * g * -0.72134752f);   // exp(-g^2 / 2)
        return g * (g >= 0.0f ? 1.0f - h : h);
    } else {
        return fmaxf(g, 0.0f);
    }
}

__device__ __forceinline__ float glu_act_precise(float g, int act)
{
    switch (act) {
    case DASS_ACT_SILU:
        return g / (1.0f + expf(-g));
    case DASS_ACT_GELU_TANH: {
        const float z2 = 1.5957691216057308f * g * (1.0f + 0.044715f * g * g);
        return g / (1.0f + expf(-z2));
    }
    case DASS_ACT_GELU_ERF:
        return 0.5f * g * (1.0f + erff(g * 0.7071067811865476f));
    default:
        return fmaxf(g, 0.0f);
    }
}

// ------------------------------------------------------- small helper kernels --
__global__ void fill_zero_kernel(float *p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        p[i] = 0.0f;
}

__global__ void sqrt_kernel(const float *__restrict__ sumsq, float *__restrict__ norms, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        norms[i] = (float)sqrt((double)sumsq[i]);
}

// ------------------------------------------------------------------ bf16 MFMA --
// Slot (in 16-byte units) of K-chunk c of tile row r inside the row's CHUNKS
// slots.  A 16-byte fragment read is served for 16 lanes = 16 consecutive rows
// at a time; 16 / CHUNKS rows share one 256-byte line of the 64 banks, so the
// XOR term changes every 16 / CHUNKS rows and the 16 reads land on 16 distinct
// (line half, slot) places.
template <int CHUNKS>
__device__ __forceinline__ int swizzle(int r, int c)
{
    return c ^ ((r / (16 / CHUNKS)) & (CHUNKS - 1));
}

template <int BM, int BN, int BK, int WM, int WN, int MINB, int ACT>
__global__ __launch_bounds__(64 * WM * WN, MINB) void calib_mfma_kernel(
    const uint16_t *__restrict__ X, int64_t T, int64_t ldx, const uint16_t *__restrict__ Wg,
    const uint16_t *__restrict__ Wu, int64_t ldw, int64_t d, int64_t d_int,
    float *__restrict__ sumsq, int64_t tiles_t, int64_t tiles_n)
{
    constexpr int NT = 64 * WM * WN;       // threads
    constexpr int CH = BK / 8;             // 16-byte chunks per tile row
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int A_CHUNKS = BM * CH / NT;  // chunks per thread per slab
    constexpr int B_CHUNKS = BN * CH / NT;  // per matrix
    constexpr int ROWS_PER_PASS = NT / CH;
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    constexpr int STAGE = A_BYTES + 2 * B_BYTES;
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0 && BK % 16 == 0, "tile shape");
    static_assert((BM * CH) % NT == 0 && (BN * CH) % NT == 0, "staging split");
    static_assert(CH == 4 || CH == 8, "swizzle assumes 4 or 8 chunks per row");

    __shared__ __attribute__((aligned(16))) char lds[2 * STAGE];

    // ---- tile assignment: consecutive workgroup ids go to different XCDs (8 of
    // them, each with its own L2); give each XCD a contiguous run of a tile order
    // in which any 32 consecutive tiles form a 4-token-tile x 8-neuron-tile patch.
    const int64_t n_tiles = tiles_t * tiles_n;
    const int64_t per_xcd = (n_tiles + 7) / 8;
    const int64_t lin = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (lin >= n_tiles)
        return;
    constexpr int BAND = 8;
    const int64_t full_bands = tiles_n / BAND;
    int64_t tile_t, tile_n;
    if (lin < full_bands * BAND * tiles_t) {
        const int64_t band = lin / (BAND * tiles_t), rem = lin % (BAND * tiles_t);
        tile_t = rem / BAND;
        tile_n = band * BAND + rem % BAND;
    } else {
        const int64_t rem = lin - full_bands * BAND * tiles_t;
        const int64_t bw = tiles_n - full_bands * BAND;
        tile_t = rem / bw;
        tile_n = full_bands * BAND + rem % bw;
    }
    const int64_t t0 = tile_t * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- global -> register staging: thread owns chunk column (tid % CH) of rows
    // tid / CH + p * ROWS_PER_PASS.  Out-of-range rows are clamped to the last
    // valid row: their products are discarded in the epilogue.
    const int ld_c = tid % CH, ld_r = tid / CH;
    const uint16_t *a_ptr[A_CHUNKS];
    const uint16_t *g_ptr[B_CHUNKS];
    const uint16_t *u_ptr[B_CHUNKS];
#pragma unroll
    for (int p = 0; p < A_CHUNKS; ++p) {
        int64_t r = t0 + ld_r + p * ROWS_PER_PASS;
        r = r < T ? r : T - 1;
        a_ptr[p] = X + r * ldx + ld_c * 8;
    }
#pragma unroll
    for (int p = 0; p < B_CHUNKS; ++p) {
        int64_t r = n0 + ld_r + p * ROWS_PER_PASS;
        r = r < d_int ? r : d_int - 1;
        g_ptr[p] = Wg + r * ldw + ld_c * 8;
        u_ptr[p] = Wu + r * ldw + ld_c * 8;
    }
    u32x4 a_st[A_CHUNKS], g_st[B_CHUNKS], u_st[B_CHUNKS];

    auto load_slab = [&](int64_t k0) {
#pragma unroll
        for (int p = 0; p < A_CHUNKS; ++p)
            a_st[p] = *reinterpret_cast<const u32x4 *>(a_ptr[p] + k0);
#pragma unroll
        for (int p = 0; p < B_CHUNKS; ++p) {
            g_st[p] = *reinterpret_cast<const u32x4 *>(g_ptr[p] + k0);
            u_st[p] = *reinterpret_cast<const u32x4 *>(u_ptr[p] + k0);
        }
    };
    // Last slab when d is not a multiple of BK: chunks past d are read from the
    // row's first chunk instead (always in range) and cleared.
    auto load_slab_tail = [&](int64_t k0) {
        const bool k_ok = k0 + ld_c * 8 < d;
        const int64_t off = k_ok ? k0 : -(int64_t)(ld_c * 8);
        const uint32_t keep = k_ok ? 0xffffffffu : 0u;
#pragma unroll
        for (int p = 0; p < A_CHUNKS; ++p)
            a_st[p] = *reinterpret_cast<const u32x4 *>(a_ptr[p] + off) & keep;
#pragma unroll
        for (int p = 0; p < B_CHUNKS; ++p) {
            g_st[p] = *reinterpret_cast<const u32x4 *>(g_ptr[p] + off) & keep;
            u_st[p] = *reinterpret_cast<const u32x4 *>(u_ptr[p] + off) & keep;
        }
    };
    auto store_slab = [&](int buf) {
        char *base = lds + buf * STAGE;
#pragma unroll
        for (int p = 0; p < A_CHUNKS; ++p) {
            const int r = ld_r + p * ROWS_PER_PASS;
            *reinterpret_cast<u32x4 *>(base + (r * CH + swizzle<CH>(r, ld_c)) * 16) = a_st[p];
        }
#pragma unroll
        for (int p = 0; p < B_CHUNKS; ++p) {
            const int r = ld_r + p * ROWS_PER_PASS;
            const int off = (r * CH + swizzle<CH>(r, ld_c)) * 16;
            *reinterpret_cast<u32x4 *>(base + A_BYTES + off) = g_st[p];
            *reinterpret_cast<u32x4 *>(base + A_BYTES + B_BYTES + off) = u_st[p];
        }
    };

    f32x16 acc_g[MI][NI], acc_u[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc_g[i][j][r] = 0.0f;
                acc_u[i][j][r] = 0.0f;
            }

    // fragment read positions: lane holds tile row (lane % 32) and the
    // (lane / 32)-th 8-element K chunk of each 16-wide K step
    const int fr = lane & 31, fc = lane >> 5;

    const int64_t n_slabs = (d + BK - 1) / BK;
    const bool ragged_k = d % BK != 0;
    auto fetch = [&](int64_t slab) {
        if (ragged_k && slab == n_slabs - 1)
            load_slab_tail(slab * BK);
        else
            load_slab(slab * BK);
    };
    fetch(0);
    store_slab(0);
    __syncthreads();

    for (int64_t ks = 0; ks < n_slabs; ++ks) {
        const int cur = (int)(ks & 1);
        const bool more = ks + 1 < n_slabs;
        if (more)
            fetch(ks + 1);

        const char *base = lds + cur * STAGE;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[MI], gf[NI], uf[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const int r = wm * TM + i * 32 + fr;
                af[i] = *reinterpret_cast<const bf16x8 *>(
                    base + (r * CH + swizzle<CH>(r, kk * 2 + fc)) * 16);
            }
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int r = wn * TN + j * 32 + fr;
                const int off = (r * CH + swizzle<CH>(r, kk * 2 + fc)) * 16;
                gf[j] = *reinterpret_cast<const bf16x8 *>(base + A_BYTES + off);
                uf[j] = *reinterpret_cast<const bf16x8 *>(base + A_BYTES + B_BYTES + off);
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    acc_g[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], gf[j],
                                                                          acc_g[i][j], 0, 0, 0);
                    acc_u[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], uf[j],
                                                                          acc_u[i][j], 0, 0, 0);
                }
        }
        if (more)
            store_slab(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: y = act(g) * u, squared and summed over the tile's tokens.
    // Accumulator register r of lane l in a 32x32 block is token row
    // 8 * (r / 4) + 4 * (l / 32) + r % 4 and neuron column l % 32.
    const bool full_t = t0 + BM <= T;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        float part = 0.0f;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float y = glu_act_fast<ACT>(acc_g[i][j][r]) * acc_u[i][j][r];
                const int64_t t = t0 + wm * TM + i * 32 + 8 * (r / 4) + 4 * fc + (r % 4);
                part += (full_t || t < T) ? y * y : 0.0f;
            }
        }
        part += __shfl_xor(part, 32, 64);
        const int64_t n = n0 + wn * TN + j * 32 + fr;
        if (fc == 0 && n < d_int)
            atomicAdd(sumsq + n, part);
    }
}

// ------------------------------------------------------- bf16 MFMA, pipelined --
typedef __attribute__((address_space(3))) void *lds_ptr_t;

// s_waitcnt that only constrains the vector-memory counter (6 bits, split field).
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

// Workgroup barrier that the compiler may not move LDS traffic across (the
// direct-to-LDS loads are invisible to its alias analysis).
__device__ __forceinline__ void block_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Workgroup tile of calib_pipe64_kernel, shared with the host-side checks.
constexpr int P_BM = 256, P_BN = 128;

// ------------------------------------------------- bf16 MFMA, 128-byte rows --
// The workgroup tile and wavefront tiles of calib_mfma_kernel (256 tokens x 128 neurons x {gate,
// up}; a wavefront 128 x 64 x 2), fed by direct global -> LDS loads instead of register staging.
// K slabs are 64 columns: a wave-load covers 8 tile rows x 128 bytes, so every request to L2 is a
// whole 128-byte line (half as many requests as with 64-byte row pieces, measured +9 % at the
// same board power), and there is one barrier per 64 columns.
//
// 64 KB per slab leaves room for 2.5 slabs in the 160 KB of LDS, so the A part (X: 256 rows x
// 128 B) and the B part (Wgate and Wup: 2 x 128 rows x 128 B) of a slab are ring units of their
// own, five units of 32 KB: slab s keeps its A part in unit 2 s mod 5 and its B part in unit
// (2 s + 1) mod 5.  Both are free once every wavefront holds its last fragments of slab s, i.e.
// after the barrier that follows K step 2 of 4; what goes into them is the B part of slab s + 2
// (due one slab later) and the A part of slab s + 3 (due two slabs later), one wave-load every
// second MFMA pair, the B part first.
//
// What happens to the finished tile is a template parameter:
//   kEpiNorms  the calibration statistic: y = act(g) u squared and summed over the tokens
//   kEpiGlu    Eq. 2 itself: y rounded to bf16 and stored, [T, d_int] row-major
//   kEpiGemm   no activation: a plain product X W^T stored as bf16 (Eq. 3 with X = y, W = Wdown).
//              The "gate" rows of a tile are W rows n0 .. n0 + 127, its "up" rows the next 128,
//              so a tile is 256 x 256 outputs and Wu is not used.
// The two storing forms go through LDS (free after the last barrier of the main loop): lanes
// pair neighbouring columns into 32-bit words, the workgroup then writes whole 16-byte chunks
// of output rows.
constexpr int P64_LDS = 5 * 32768;
enum { kEpiNorms = 0, kEpiGlu = 1, kEpiGemm = 2 };

// float -> bf16 bits, round to nearest even (finite inputs)
// Two f32 rounded to bf16 (nearest even), `lo` in the low half of the word: one v_cvt_pk_bf16_f32.
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ uint32_t bf16_pair(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}

template <int ACT, int EPI>
__global__ __launch_bounds__(256) void calib_pipe64_kernel(
    const uint16_t *__restrict__ X, int64_t T, int64_t ldx, const uint16_t *__restrict__ Wg,
    const uint16_t *__restrict__ Wu, int64_t ldw, int64_t d, int64_t d_int,
    float *__restrict__ sumsq, uint16_t *__restrict__ out, int64_t ldo, int64_t tiles_t, int64_t tiles_n,
    int super_rows)
{
    constexpr int BM = P_BM, BN = P_BN, BK = 64, WN = 2;
    constexpr int BN_TILE = EPI == kEpiGemm ? 2 * BN : BN;   // rows of W (output columns) per tile
    constexpr int TM = 128, TN = 64, MI = 8, NI = 4;   // wavefront tile in 16 x 16 MFMA blocks
    constexpr int CH = BK / 8;               // 16-byte chunks per tile row
    constexpr int UNIT = 32768;              // A part, or gate half + up half of the B part
    constexpr int B_HALF = BN * BK * 2;      // 16 KB
    constexpr int A_WL = 8, B_WL = 4;        // wave-loads (8 rows x 128 B) per wavefront per slab: 8 + 4 + 4

    extern __shared__ __attribute__((aligned(1024))) char lds64[];   // P64_LDS bytes

    // ---- tile assignment.  Consecutive workgroup ids go to different XCDs (8 of them, each
    // with its own L2).  The tile grid is cut into patches of 4 token tiles x 8 neuron tiles; an
    // XCD's 32 concurrent workgroups take one patch, so its L2 serves all but 3/16 of their reads.
    // Patches are dealt round-robin to the XCDs from a list ordered so that the 8 patches in
    // flight share data through the memory-side cache:
    //   super_rows = 1: token-major.  The 8 patches lie in one row of patches: X is fetched
    //     from HBM by one XCD and found in the cache by the others, and the weights stay
    //     cached from one row to the next as long as both matrices fit (measured: +5 % over
    //     giving each XCD its own band of neurons).
    //   super_rows = R > 1, for weights too large to stay cached: rows of patches are taken R
    //     at a time, and inside such a super-row the patch columns are outermost.  The 8 patches
    //     share one patch column of the weights, fetched once per super-row, and the super-row's
    //     X (R x 8 MB at d = 4096) stays cached while the columns sweep past.
    constexpr int PT = 4, PN = 8;
    const int64_t np_n = (tiles_n + PN - 1) / PN;
    const int64_t idx = blockIdx.x / 8, within = idx % (PT * PN);
    const int64_t patch = (idx / (PT * PN)) * 8 + blockIdx.x % 8;
    const int64_t sr = patch / (np_n * super_rows), rem = patch % (np_n * super_rows);
    const int64_t prow = sr * super_rows + rem % super_rows, pcol = rem / super_rows;
    const int64_t tile_t = prow * PT + within / PN, tile_n = pcol * PN + within % PN;
    if (tile_t >= tiles_t || tile_n >= tiles_n)
        return;
    const int64_t t0 = tile_t * BM, n0 = tile_n * BN_TILE;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // ---- global -> LDS.  Lane l of a wave-load fills slot (l % 8) of row (l / 8) of an 8-row
    // block, i.e. it fetches K chunk (l % 8) ^ swizzle of that row.  Rows past the end of the
    // matrix are clamped.  Each operand is addressed as a raw buffer that starts at the tile's
    // first row and ends with its last valid element: the per-lane byte offset is a 32-bit
    // register, the K offset a scalar, and a read outside the buffer returns 0 instead of faulting.
    const int wl_row = lane >> 3, wl_slot = lane & 7;
    const int64_t rows_x = T - t0 < BM ? T - t0 : BM, rows_w = d_int - n0 < BN ? d_int - n0 : BN;
    // kEpiGemm: the second 128 rows of the tile may be fewer, or none (then an empty buffer:
    // its reads fetch nothing and return 0; clamped rows beyond its end do the same)
    const int64_t left_u = d_int - n0 - BN;
    const int64_t rows_u = EPI != kEpiGemm ? rows_w : left_u < 0 ? 0 : left_u < BN ? left_u : BN;
    uint32_t a_off[A_WL], b_off[B_WL];
#pragma unroll
    for (int p = 0; p < A_WL; ++p) {
        // rows past T are not clamped: they lie beyond the end of the buffer and read as 0, which
        // the epilogues rely on (act(0) * 0 adds nothing to a norm; stores are bounded by T)
        const int r = (wave * A_WL + p) * 8 + wl_row;
        a_off[p] = (uint32_t)((int64_t)r * ldx * 2 + (wl_slot ^ swizzle<CH>(r, 0)) * 16);
    }
#pragma unroll
    for (int p = 0; p < B_WL; ++p) {
        const int r = (wave * B_WL + p) * 8 + wl_row;
        const int64_t rr = r < rows_w ? r : rows_w - 1;
        b_off[p] = (uint32_t)(rr * ldw * 2 + (wl_slot ^ swizzle<CH>(r, 0)) * 16);
    }
    constexpr int kRawBuffer = 0x00020000;
    const int span_x = (int)((rows_x - 1) * ldx * 2 + d * 2), span_w = (int)((rows_w - 1) * ldw * 2 + d * 2);
    const int span_u = rows_u > 0 ? (int)((rows_u - 1) * ldw * 2 + d * 2) : 0;
    const uint16_t *up_rows = EPI == kEpiGemm ? Wg + (n0 + BN) * ldw : Wu + n0 * ldw;
    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(X + t0 * ldx), 0, span_x, kRawBuffer);
    const __amdgpu_buffer_rsrc_t rg =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(Wg + n0 * ldw), 0, span_w, kRawBuffer);
    const __amdgpu_buffer_rsrc_t ru =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(up_rows), 0, span_u, kRawBuffer);

    // q-th of this wavefront's 8 loads of an A part (slab at byte offset kb) into ring unit `unit`
    auto issue_a = [&](int unit, int kb, int q) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr_t)(lds64 + unit * UNIT + (wave * A_WL + q) * 1024), 16,
                                                 a_off[q], kb, 0, 0);
    };
    // q-th of its 8 loads of a B part: 4 of Wgate, then 4 of Wup
    auto issue_b = [&](int unit, int kb, int q) {
        if (q < B_WL)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rg, (lds_ptr_t)(lds64 + unit * UNIT + (wave * B_WL + q) * 1024), 16,
                                                     b_off[q], kb, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                ru, (lds_ptr_t)(lds64 + unit * UNIT + B_HALF + (wave * B_WL + q - B_WL) * 1024), 16, b_off[q - B_WL], kb, 0, 0);
    };

    f32x4 acc_g[MI][NI], acc_u[MI][NI];

    // ---- LDS -> registers.  The MFMA is v_mfma_f32_16x16x32_bf16: a lane holds tile row
    // (lane % 16) of a 16-row block and K chunk kk * 4 + lane / 16 of K step kk (0, 1: 32 columns
    // each); kk * 4 and lane / 16 occupy different bits, so the byte offset inside a unit is that
    // of K step 0 XOR kk * 64.  Blocks of 16 rows are 2048 bytes apart and swizzled alike.
    int a_frag0, b_frag0;
    {
        const int fr = lane & 15, fc = lane >> 4;
        const int ra = wm * TM + fr, rb = wn * TN + fr;
        a_frag0 = (ra * CH + swizzle<CH>(ra, fc)) * 16;
        b_frag0 = (rb * CH + swizzle<CH>(rb, fc)) * 16;
    }
    struct Frags {
        bf16x8 a[MI], g[NI], u[NI];
    };
    constexpr int N_READS = MI + 2 * NI;   // 16 fragment reads per K step
    // q-th fragment of K step kk of the slab in units (ua, ub), in the order the MFMAs need them:
    // a0 a1 g0 u0 g1 u1 g2 u2 g3 u3 a2 .. a7
    auto read_one = [&](Frags &f, int ua, int ub, int kk, int q) {
        const char *pa = lds64 + ua * UNIT + (a_frag0 ^ (kk * 64)), *pb = lds64 + ub * UNIT + (b_frag0 ^ (kk * 64));
        if (q < 2) {
            f.a[q] = *reinterpret_cast<const bf16x8 *>(pa + q * 2048);
        } else if (q < 2 + 2 * NI) {
            const int j = (q - 2) >> 1;
            if ((q - 2) & 1)
                f.u[j] = *reinterpret_cast<const bf16x8 *>(pb + B_HALF + j * 2048);
            else
                f.g[j] = *reinterpret_cast<const bf16x8 *>(pb + j * 2048);
        } else {
            const int i = q - 2 * NI;
            f.a[i] = *reinterpret_cast<const bf16x8 *>(pa + i * 2048);
        }
    };
    constexpr int N_PAIRS = MI * NI;   // 32 pairs of MFMAs per K step
    // Pair q of a K step.  The order is a Gray code over the operands: every MFMA shares one operand
    // with the one before, (a0, g) (a1, g) (a1, u) (a0, u) for g = g_0 .. g_3 with its u, then the next
    // two A blocks.  Measured against A-block-major order (a_i with g_0 u_0 g_1 u_1 ..): +1.5 %.
    auto mfma_pair = [&](const Frags &f, int q) {
        const int ip = q / (2 * NI), r = q % (2 * NI), j = r / 2;
        const int i0 = 2 * ip, i1 = 2 * ip + 1;
        if (r % 2 == 0) {
            acc_g[i0][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.a[i0], f.g[j], acc_g[i0][j], 0, 0, 0);
            acc_g[i1][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.a[i1], f.g[j], acc_g[i1][j], 0, 0, 0);
        } else {
            acc_u[i1][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.a[i1], f.u[j], acc_u[i1][j], 0, 0, 0);
            acc_u[i0][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.a[i0], f.u[j], acc_u[i0][j], 0, 0, 0);
        }
    };

    // ---- prologue: A0 B0 A1 B1 A2 fill the five units
    const int S = (int)(d / BK);   // slabs; the host guarantees d % 64 == 0
#pragma unroll
    for (int q = 0; q < 8; ++q)
        issue_a(0, 0, q);
#pragma unroll
    for (int q = 0; q < 8; ++q)
        issue_b(1, 0, q);
    if (S > 1) {
#pragma unroll
        for (int q = 0; q < 8; ++q)
            issue_a(2, BK * 2, q);
#pragma unroll
        for (int q = 0; q < 8; ++q)
            issue_b(3, BK * 2, q);
    }
    if (S > 2) {
#pragma unroll
        for (int q = 0; q < 8; ++q)
            issue_a(4, 2 * BK * 2, q);
    }
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                acc_g[i][j][r] = 0.0f;
                acc_u[i][j][r] = 0.0f;
            }
    if (S > 2)
        wait_vmcnt<24>();   // slab 0 has landed
    else if (S > 1)
        wait_vmcnt<16>();
    else
        wait_vmcnt<0>();
    block_barrier();
    Frags f0, f1;
#pragma unroll
    for (int q = 0; q < N_READS; ++q)
        read_one(f0, 0, 1, 0, q);

    // ---- main loop.  One slab = 2 K steps of 32 gate/up MFMA pairs, the first on f0, the second
    // on f1.  During K step 0 a wavefront reads the fragments of K step 1 (one read every second
    // pair); during the second half of K step 1, after the slab's one barrier, those of K step 0
    // of the next slab (one read a pair).  One global->LDS wave-load goes out every fourth pair:
    // the rest of the B part of slab s + 1 (first half of K step 0), then the A part of slab s + 2
    // (up to the barrier), then the first half of the B part of slab s + 2 into the A unit of
    // slab s, which is free once every wavefront holds its last fragments of slab s.  B1, A2, B2:
    // whether these parts exist and were not issued by the prologue; NEXT: whether a slab follows.
    // All four are compile-time, so the steady state has no branch between its MFMAs.
    int ua = 0, ub = 1;   // ring units of slab s
    auto slab_body = [&](int s, auto b1_tag, auto a2_tag, auto b2_tag, auto next_tag) {
        constexpr bool B1 = decltype(b1_tag)::value, A2 = decltype(a2_tag)::value, B2 = decltype(b2_tag)::value,
                       NEXT = decltype(next_tag)::value;
        const int ua1 = ua + 2 >= 5 ? ua - 3 : ua + 2, ub1 = ub + 2 >= 5 ? ub - 3 : ub + 2;   // units of slab s + 1
        const int uam = ua >= 2 ? ua - 2 : ua + 3, ubm = ub >= 2 ? ub - 2 : ub + 3;           // units of slab s - 1
        const int k1 = (s + 1) * BK * 2, k2 = (s + 2) * BK * 2;
#pragma unroll
        for (int q = 0; q < N_PAIRS; ++q) {   // K step 0
            if (B1 && q < N_PAIRS / 2 && (q & 3) == 0)
                issue_b(uam, k1, 4 + (q >> 2));
            if (A2 && q >= N_PAIRS / 2 && (q & 3) == 0)
                issue_a(ubm, k2, (q - N_PAIRS / 2) >> 2);
            if ((q & 1) == 0)
                read_one(f1, ua, ub, 1, q >> 1);
            mfma_pair(f0, q);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int q = 0; q < N_PAIRS / 2; ++q) {   // K step 1, first half
            if (A2 && (q & 3) == 0)
                issue_a(ubm, k2, 4 + (q >> 2));
            mfma_pair(f1, q);
            __builtin_amdgcn_sched_barrier(0);
        }
        // Slab s + 1 has landed (only the A part of slab s + 2, the last 8 loads, may be in
        // flight) and this wavefront holds its last fragments of slab s: vmcnt(8 or 0), lgkmcnt(0).
        if (A2)
            __builtin_amdgcn_s_waitcnt(0x0078);
        else
            __builtin_amdgcn_s_waitcnt(0x0070);
        block_barrier();
#pragma unroll
        for (int q = N_PAIRS / 2; q < N_PAIRS; ++q) {   // K step 1, second half; the units of slab s are free
            if (B2 && (q & 3) == 0)
                issue_b(ua, k2, (q - N_PAIRS / 2) >> 2);
            if (NEXT)
                read_one(f0, ua1, ub1, 0, q - N_PAIRS / 2);
            mfma_pair(f1, q);
            __builtin_amdgcn_sched_barrier(0);
        }
        ua = ua1;
        ub = ub1;
    };
    using Yes = std::true_type;
    using No = std::false_type;
    if (S >= 3) {
        slab_body(0, No{}, No{}, Yes{}, Yes{});   // B1 and A2 went out in the prologue
        int s = 1;
        for (; s + 2 < S; ++s)
            slab_body(s, Yes{}, Yes{}, Yes{}, Yes{});
        slab_body(s, Yes{}, No{}, No{}, Yes{});       // slab S - 2
        slab_body(s + 1, No{}, No{}, No{}, No{});     // slab S - 1
    } else if (S == 2) {
        slab_body(0, No{}, No{}, No{}, Yes{});
        slab_body(1, No{}, No{}, No{}, No{});
    } else {
        slab_body(0, No{}, No{}, No{}, No{});
    }

    if constexpr (EPI == kEpiNorms) {
        // ---- epilogue: y = act(g) * u, squared and summed over the tile's tokens (tokens are the
        // MFMA's M index: the 4 registers a lane holds of a 16 x 16 block are rows 4 (lane / 16) ..
        // + 3 of column lane % 16, i.e. 4 tokens of one neuron).  Tokens past T were read as zeros, so
        // their y is 0 and no test is needed.  The lane's neuron index is derived here from the lane
        // number afresh: nothing per-lane has to survive the main loop for it (a spill would give
        // the kernel a scratch segment).
        uint32_t lane_e = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        asm volatile("" : "+v"(lane_e));
        const int fr_e = lane_e & 15, fc_e = lane_e >> 4;
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            float part = 0.0f;
#pragma unroll
            for (int i = 0; i < MI; ++i) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float y = glu_act_fast<ACT>(acc_g[i][j][r]) * acc_u[i][j][r];
                    part = fmaf(y, y, part);
                }
            }
            part += __shfl_xor(part, 16, 64);
            part += __shfl_xor(part, 32, 64);
            const int64_t n = n0 + wn * TN + j * 16 + fr_e;
            if (fc_e == 0 && n < d_int)
                atomicAdd(sumsq + n, part);
        }
    } else {
        // ---- storing epilogues.  Every wavefront is past the last barrier and the last LDS read
        // of the main loop, so the ring is free: the tile goes there as bf16, row stride SROW (16
        // bytes of padding), and leaves it in whole 16-byte chunks of output rows.
        constexpr int COLS = BN_TILE;                // output columns of the tile
        constexpr int SROW = COLS * 2 + 16;
        static_assert(BM * SROW <= P64_LDS, "the tile fits in the ring");
        // A lane holds rows r and r + 1 (registers 2 k, 2 k + 1) of column fr; with its neighbour
        // fr ^ 1 it trades one of them, so that even lanes own row 2 k and odd lanes row 2 k + 1
        // of the column pair: one 32-bit LDS write each.
        uint32_t lane_s = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));   // afresh, as above
        asm volatile("" : "+v"(lane_s));
        const int fr = lane_s & 15, fc = lane_s >> 4;
        auto put_pair = [&](float v0, float v1, int row_even, int col_base) {
            const bool odd = fr & 1;
            const float mine = odd ? v1 : v0, send = odd ? v0 : v1;
            const float got = __shfl_xor(send, 1, 64);
            const uint32_t word = odd ? bf16_pair(got, mine) : bf16_pair(mine, got);
            const int row = row_even + (odd ? 1 : 0), col = col_base + (fr & ~1);
            *reinterpret_cast<uint32_t *>(lds64 + row * SROW + col * 2) = word;
        };
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const int row_even = wm * TM + i * 16 + 4 * fc + 2 * k;
                    const int col_base = wn * TN + j * 16;
                    if constexpr (EPI == kEpiGlu) {
                        put_pair(glu_act_fast<ACT>(acc_g[i][j][2 * k]) * acc_u[i][j][2 * k],
                                 glu_act_fast<ACT>(acc_g[i][j][2 * k + 1]) * acc_u[i][j][2 * k + 1], row_even, col_base);
                    } else {
                        put_pair(acc_g[i][j][2 * k], acc_g[i][j][2 * k + 1], row_even, col_base);
                        put_pair(acc_u[i][j][2 * k], acc_u[i][j][2 * k + 1], row_even, BN + col_base);
                    }
                }
        __syncthreads();
        constexpr int CPR = COLS / 8;   // 16-byte chunks per tile row
        for (int c = tid; c < BM * CPR; c += 256) {
            const int row = c / CPR, cc = c % CPR;
            const int64_t t = t0 + row, n = n0 + cc * 8;
            if (t < T && n < d_int)   // d_int is a multiple of 8: a chunk is inside or outside
                __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(lds64 + row * SROW + cc * 16),
                                            reinterpret_cast<u32x4 *>(out + t * ldo + n));   // streamed: not read again from L2
        }
    }
}

// ------------------------------------------------------------------ f32 tiled --
constexpr int F_BM = 64, F_BN = 64, F_BK = 16, F_PAD = 4;

__global__ __launch_bounds__(256) void calib_f32_kernel(
    const float *__restrict__ X, int64_t T, int64_t ldx, const float *__restrict__ Wg,
    const float *__restrict__ Wu, int64_t ldw, int64_t d, int64_t d_int, int act,
    float *__restrict__ sumsq, int64_t tiles_n)
{
    __shared__ float xs[F_BK][F_BM + F_PAD];
    __shared__ float gs[F_BK][F_BN + F_PAD];
    __shared__ float us[F_BK][F_BN + F_PAD];
    __shared__ float red[16][F_BN];

    const int64_t tile_t = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
    const int64_t t0 = tile_t * F_BM, n0 = tile_n * F_BN;
    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    const int lr = tid / 4, lk = (tid % 4) * 4;  // staging: row lr, columns lk..lk+3

    float ag[4][4], au[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            ag[i][j] = au[i][j] = 0.0f;

    for (int64_t k0 = 0; k0 < d; k0 += F_BK) {
        const bool k_ok = k0 + lk < d;  // d is a multiple of 4
        float4 xv = make_float4(0.f, 0.f, 0.f, 0.f), gv = xv, uv = xv;
        if (k_ok && t0 + lr < T)
            xv = *reinterpret_cast<const float4 *>(X + (t0 + lr) * ldx + k0 + lk);
        if (k_ok && n0 + lr < d_int) {
            gv = *reinterpret_cast<const float4 *>(Wg + (n0 + lr) * ldw + k0 + lk);
            uv = *reinterpret_cast<const float4 *>(Wu + (n0 + lr) * ldw + k0 + lk);
        }
        __syncthreads();  // previous slab fully consumed
        xs[lk + 0][lr] = xv.x; xs[lk + 1][lr] = xv.y; xs[lk + 2][lr] = xv.z; xs[lk + 3][lr] = xv.w;
        gs[lk + 0][lr] = gv.x; gs[lk + 1][lr] = gv.y; gs[lk + 2][lr] = gv.z; gs[lk + 3][lr] = gv.w;
        us[lk + 0][lr] = uv.x; us[lk + 1][lr] = uv.y; us[lk + 2][lr] = uv.z; us[lk + 3][lr] = uv.w;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < F_BK; ++k) {
            float a[4], g[4], u[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = xs[k][ty * 4 + i];
                g[i] = gs[k][tx * 4 + i];
                u[i] = us[k][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    ag[i][j] = fmaf(a[i], g[j], ag[i][j]);
                    au[i][j] = fmaf(a[i], u[j], au[i][j]);
                }
        }
    }
    // tokens past T were staged as zero rows: g = u = 0 gives y = 0
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float y = glu_act_precise(ag[i][j], act) * au[i][j];
            s = fmaf(y, y, s);
        }
        red[ty][tx * 4 + j] = s;
    }
    __syncthreads();
    if (tid < F_BN) {
        float s = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s += red[r][tid];
        if (n0 + tid < d_int)
            atomicAdd(sumsq + n0 + tid, s);
    }
}

// ------------------------------------------------------------------ host side --
template <int BM, int BN, int BK, int WM, int WN, int MINB>
static void launch_mfma(int act, dim3 grid, hipStream_t stream, const uint16_t *X, int64_t T,
                        int64_t ldx, const uint16_t *Wg, const uint16_t *Wu, int64_t ldw, int64_t d,
                        int64_t d_int, float *sumsq, int64_t tiles_t, int64_t tiles_n)
{
    const dim3 block(64 * WM * WN);
    switch (act) {
    case DASS_ACT_SILU:
        hipLaunchKernelGGL((calib_mfma_kernel<BM, BN, BK, WM, WN, MINB, DASS_ACT_SILU>), grid, block, 0,
                           stream, X, T, ldx, Wg, Wu, ldw, d, d_int, sumsq, tiles_t, tiles_n);
        break;
    case DASS_ACT_GELU_TANH:
        hipLaunchKernelGGL((calib_mfma_kernel<BM, BN, BK, WM, WN, MINB, DASS_ACT_GELU_TANH>), grid, block,
                           0, stream, X, T, ldx, Wg, Wu, ldw, d, d_int, sumsq, tiles_t, tiles_n);
        break;
    case DASS_ACT_GELU_ERF:
        hipLaunchKernelGGL((calib_mfma_kernel<BM, BN, BK, WM, WN, MINB, DASS_ACT_GELU_ERF>), grid, block,
                           0, stream, X, T, ldx, Wg, Wu, ldw, d, d_int, sumsq, tiles_t, tiles_n);
        break;
    default:
        hipLaunchKernelGGL((calib_mfma_kernel<BM, BN, BK, WM, WN, MINB, DASS_ACT_RELU>), grid, block, 0,
                           stream, X, T, ldx, Wg, Wu, ldw, d, d_int, sumsq, tiles_t, tiles_n);
        break;
    }
}

template <int ACT, int EPI>
static hipError_t launch_pipe64_act(dim3 grid, hipStream_t stream, const uint16_t *X, int64_t T, int64_t ldx,
                                    const uint16_t *Wg, const uint16_t *Wu, int64_t ldw, int64_t d, int64_t d_int,
                                    float *sumsq, uint16_t *out, int64_t ldo, int64_t tiles_t, int64_t tiles_n,
                                    int super_rows)
{
    // the kernel's ring takes all 160 KB of LDS, more than a launch gets without asking
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(calib_pipe64_kernel<ACT, EPI>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, P64_LDS);
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL((calib_pipe64_kernel<ACT, EPI>), grid, dim3(256), P64_LDS, stream, X, T, ldx, Wg, Wu, ldw, d,
                       d_int, sumsq, out, ldo, tiles_t, tiles_n, super_rows);
    return hipSuccess;
}

template <int EPI>
static hipError_t launch_pipe64(int act, dim3 grid, hipStream_t stream, const uint16_t *X, int64_t T, int64_t ldx,
                                const uint16_t *Wg, const uint16_t *Wu, int64_t ldw, int64_t d, int64_t d_int,
                                float *sumsq, uint16_t *out, int64_t ldo, int64_t tiles_t, int64_t tiles_n,
                                int super_rows)
{
    switch (act) {
    case DASS_ACT_SILU:
        return launch_pipe64_act<DASS_ACT_SILU, EPI>(grid, stream, X, T, ldx, Wg, Wu, ldw, d, d_int, sumsq, out, ldo,
                                                     tiles_t, tiles_n, super_rows);
    case DASS_ACT_GELU_TANH:
        return launch_pipe64_act<DASS_ACT_GELU_TANH, EPI>(grid, stream, X, T, ldx, Wg, Wu, ldw, d, d_int, sumsq, out,
                                                          ldo, tiles_t, tiles_n, super_rows);
    case DASS_ACT_GELU_ERF:
        return launch_pipe64_act<DASS_ACT_GELU_ERF, EPI>(grid, stream, X, T, ldx, Wg, Wu, ldw, d, d_int, sumsq, out,
                                                         ldo, tiles_t, tiles_n, super_rows);
    default:
        return launch_pipe64_act<DASS_ACT_RELU, EPI>(grid, stream, X, T, ldx, Wg, Wu, ldw, d, d_int, sumsq, out, ldo,
                                                     tiles_t, tiles_n, super_rows);
    }
}

// Grid of the pipelined kernels: whole 4 x 8 patches of tiles dealt to the 8 XCDs, rows of
// patches in groups of `super_rows`.  Returns 0 when one launch cannot hold it.
static int64_t pipe_grid(int64_t tiles_t, int64_t tiles_n, int super_rows)
{
    const int64_t patches = ((tiles_t + 3) / 4 + super_rows - 1) / super_rows * super_rows * ((tiles_n + 7) / 8);
    const int64_t blocks = (patches + 7) / 8 * 8 * 32;
    return blocks > 0x7fffffffLL ? 0 : blocks;
}

}  // namespace dass

extern "C" size_t dass_calib_workspace_bytes(int64_t T, int64_t d, int64_t d_int, dass_dtype dt)
{
    (void)T; (void)d; (void)d_int; (void)dt;
    return 0;  // the accumulation goes straight into sumsq
}

extern "C" dass_status dass_calib_norms(const void *X, int64_t T, int64_t ldx, const void *Wgate,
                                        const void *Wup, int64_t ldw, int64_t d, int64_t d_int,
                                        dass_dtype dt, dass_act act, float *sumsq, int accumulate,
                                        float *norms_out, void *workspace, size_t workspace_bytes,
                                        void *hip_stream)
{
    using namespace dass;
    const char *fn = "dass_calib_norms";
    (void)workspace;
    (void)workspace_bytes;
    if (!X || !Wgate || !Wup || !sumsq)
        return fail(DASS_ERR_NULL, "%s: X, Wgate, Wup and sumsq must not be NULL", fn);
    if (!valid_dtype(dt))
        return fail(DASS_ERR_DTYPE, "%s: unknown dtype %d", fn, (int)dt);
    if ((int)act < DASS_ACT_SILU || (int)act > DASS_ACT_RELU)
        return fail(DASS_ERR_DTYPE, "%s: unknown activation %d", fn, (int)act);
    if (T <= 0 || d <= 0 || d_int <= 0)
        return fail(DASS_ERR_SHAPE, "%s: T=%lld d=%lld d_int=%lld must be positive", fn,
                    (long long)T, (long long)d, (long long)d_int);
    if (ldx < d || ldw < d)
        return fail(DASS_ERR_SHAPE, "%s: ldx=%lld, ldw=%lld must be >= d=%lld", fn, (long long)ldx,
                    (long long)ldw, (long long)d);
    const int vec = vec_elems(dt);
    if (d % vec != 0)
        return fail(DASS_ERR_SHAPE, "%s: d=%lld must be a multiple of %d", fn, (long long)d, vec);
    if (!aligned16(X) || !aligned16(Wgate) || !aligned16(Wup) ||
        (reinterpret_cast<uintptr_t>(sumsq) & 3u) ||
        (norms_out && (reinterpret_cast<uintptr_t>(norms_out) & 3u)))
        return fail(DASS_ERR_ALIGN, "%s: X, Wgate, Wup must be 16-byte aligned", fn);
    if (ldx % vec != 0 || ldw % vec != 0)
        return fail(DASS_ERR_ALIGN, "%s: ldx, ldw must be multiples of %d elements", fn, vec);

    // ---- launch plan; every size check comes before the first launch
    constexpr int BM = P_BM, BN = P_BN, BK = 64;
    const bool bf16 = dt == DASS_BF16;
    const int64_t tiles_t = bf16 ? (T + BM - 1) / BM : (T + F_BM - 1) / F_BM;
    const int64_t tiles_n = bf16 ? (d_int + BN - 1) / BN : (d_int + F_BN - 1) / F_BN;
    // calib_pipe64_kernel: d a multiple of its 64-column slab, and 32-bit byte offsets inside a
    // tile's rows.  Its grid is whole 4 x 8 patches of tiles dealt to the 8 XCDs, rows of patches in
    // groups of 8 when Wgate + Wup exceed the 256 MB memory-side cache (see the kernel).
    const bool pipe64 = bf16 && d % 64 == 0 && (int64_t)BM * ldx * 2 < 0x7fffffffLL &&
                        (int64_t)BN * ldw * 2 < 0x7fffffffLL;
    const int super_rows = 2 * d_int * d * 2 > (256LL << 20) ? 8 : 1;
    const int64_t blocks = pipe64 ? pipe_grid(tiles_t, tiles_n, super_rows)
                           : bf16 ? (tiles_t * tiles_n + 7) / 8 * 8
                                  : tiles_t * tiles_n;
    if (blocks <= 0 || blocks > 0x7fffffffLL)
        return fail(DASS_ERR_SHAPE, "%s: too many tiles for one launch; split the tokens", fn);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const unsigned vgrid = (unsigned)((d_int + 255) / 256);
    if (!accumulate) {
        hipLaunchKernelGGL(fill_zero_kernel, dim3(vgrid), dim3(256), 0, stream, sumsq, d_int);
        dass_status s = check_launch("fill kernel");
        if (s != DASS_OK)
            return s;
    }
    if (pipe64) {
        const hipError_t e = launch_pipe64<kEpiNorms>((int)act, dim3((unsigned)blocks), stream,
                                                      static_cast<const uint16_t *>(X), T, ldx,
                                                      static_cast<const uint16_t *>(Wgate),
                                                      static_cast<const uint16_t *>(Wup), ldw, d, d_int, sumsq,
                                                      nullptr, 0, tiles_t, tiles_n, super_rows);
        if (e != hipSuccess)
            return fail(DASS_ERR_HIP, "%s: cannot reserve %d bytes of LDS: %s", fn, P64_LDS, hipGetErrorString(e));
    } else if (bf16) {
        launch_mfma<BM, BN, BK, 4, 2, 1>((int)act, dim3((unsigned)blocks), stream, static_cast<const uint16_t *>(X),
                                         T, ldx, static_cast<const uint16_t *>(Wgate),
                                         static_cast<const uint16_t *>(Wup), ldw, d, d_int, sumsq, tiles_t, tiles_n);
    } else {
        hipLaunchKernelGGL(calib_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                           static_cast<const float *>(X), T, ldx, static_cast<const float *>(Wgate),
                           static_cast<const float *>(Wup), ldw, d, d_int, (int)act, sumsq, tiles_n);
    }
    dass_status s = check_launch("calibration kernel");
    if (s != DASS_OK)
        return s;
    if (norms_out) {
        hipLaunchKernelGGL(sqrt_kernel, dim3(vgrid), dim3(256), 0, stream, (const float *)sumsq,
                           norms_out, d_int);
        s = check_launch("sqrt kernel");
    }
    return s;
}

// ------------------------------------------------------------- MLP output --
extern "C" size_t dass_mlp_forward_workspace_bytes(int64_t T, int64_t d, int64_t d_int, dass_dtype dt)
{
    (void)d;
    if (T <= 0 || d_int <= 0 || dt != DASS_BF16)
        return 0;
    return (size_t)T * (size_t)d_int * 2;   // y of Eq. 2 as bf16, [T, d_int]
}

extern "C" dass_status dass_mlp_forward(const void *X, int64_t T, int64_t ldx, const void *Wgate, const void *Wup,
                                        int64_t ldw, const void *Wdown, int64_t ldd, int64_t d, int64_t d_int,
                                        dass_dtype dt, dass_act act, void *out, int64_t ldo, void *workspace,
                                        size_t workspace_bytes, void *hip_stream)
{
    using namespace dass;
    const char *fn = "dass_mlp_forward";
    const bool eq2_only = Wdown == nullptr;   // y stays in the workspace; out and ldd, ldo are not used
    if (!X || !Wgate || !Wup || !workspace || (!eq2_only && !out))
        return fail(DASS_ERR_NULL, "%s: X, Wgate, Wup, workspace (and out, unless Wdown is NULL) must not be NULL", fn);
    if (!valid_dtype(dt))
        return fail(DASS_ERR_DTYPE, "%s: unknown dtype %d", fn, (int)dt);
    if (dt != DASS_BF16)
        return fail(DASS_ERR_DTYPE, "%s: only bf16 is implemented", fn);
    if ((int)act < DASS_ACT_SILU || (int)act > DASS_ACT_RELU)
        return fail(DASS_ERR_DTYPE, "%s: unknown activation %d", fn, (int)act);
    if (T <= 0 || d <= 0 || d_int <= 0)
        return fail(DASS_ERR_SHAPE, "%s: T=%lld d=%lld d_int=%lld must be positive", fn, (long long)T,
                    (long long)d, (long long)d_int);
    if (d % 64 != 0 || d_int % 64 != 0)
        return fail(DASS_ERR_SHAPE, "%s: d=%lld and d_int=%lld must be multiples of 64", fn, (long long)d,
                    (long long)d_int);
    if (ldx < d || ldw < d || (!eq2_only && (ldd < d_int || ldo < d)))
        return fail(DASS_ERR_SHAPE, "%s: a leading dimension is shorter than its row", fn);
    if (!aligned16(X) || !aligned16(Wgate) || !aligned16(Wup) || !aligned16(workspace) ||
        (!eq2_only && (!aligned16(Wdown) || !aligned16(out))))
        return fail(DASS_ERR_ALIGN, "%s: every pointer must be 16-byte aligned", fn);
    if (ldx % 8 != 0 || ldw % 8 != 0 || (!eq2_only && (ldd % 8 != 0 || ldo % 8 != 0)))
        return fail(DASS_ERR_ALIGN, "%s: leading dimensions must be multiples of 8 elements", fn);
    if (workspace_bytes < dass_mlp_forward_workspace_bytes(T, d, d_int, dt))
        return fail(DASS_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed", fn, workspace_bytes,
                    dass_mlp_forward_workspace_bytes(T, d, d_int, dt));
    // 32-bit byte offsets inside a tile's rows, as in dass_calib_norms
    if ((int64_t)P_BM * ldx * 2 >= 0x7fffffffLL || (int64_t)P_BN * ldw * 2 >= 0x7fffffffLL ||
        (int64_t)P_BM * d_int * 2 >= 0x7fffffffLL || (!eq2_only && (int64_t)P_BN * ldd * 2 >= 0x7fffffffLL))
        return fail(DASS_ERR_SHAPE, "%s: rows too long for the tile addressing", fn);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint16_t *Y = static_cast<uint16_t *>(workspace);
    const int64_t tiles_t = (T + P_BM - 1) / P_BM;
    // Eq. 2: y = act(X Wgate^T) * (X Wup^T), tiles of 256 tokens x 128 neurons
    {
        const int64_t tiles_n = (d_int + P_BN - 1) / P_BN;
        const int super_rows = 2 * d_int * d * 2 > (256LL << 20) ? 8 : 1;
        const int64_t blocks = pipe_grid(tiles_t, tiles_n, super_rows);
        if (blocks == 0)
            return fail(DASS_ERR_SHAPE, "%s: too many tiles for one launch; split the tokens", fn);
        const hipError_t e = launch_pipe64<kEpiGlu>((int)act, dim3((unsigned)blocks), stream,
                                                    static_cast<const uint16_t *>(X), T, ldx,
                                                    static_cast<const uint16_t *>(Wgate),
                                                    static_cast<const uint16_t *>(Wup), ldw, d, d_int, nullptr, Y,
                                                    d_int, tiles_t, tiles_n, super_rows);
        if (e != hipSuccess)
            return fail(DASS_ERR_HIP, "%s: cannot reserve %d bytes of LDS: %s", fn, P64_LDS, hipGetErrorString(e));
        const dass_status s = check_launch("GLU kernel");
        if (s != DASS_OK || eq2_only)
            return s;
    }
    // Eq. 3: out = y Wdown^T, tiles of 256 tokens x 256 output features, K = d_int
    {
        const int64_t tiles_n = (d + 2 * P_BN - 1) / (2 * P_BN);
        const int super_rows = d * d_int * 2 > (256LL << 20) ? 8 : 1;
        const int64_t blocks = pipe_grid(tiles_t, tiles_n, super_rows);
        if (blocks == 0)
            return fail(DASS_ERR_SHAPE, "%s: too many tiles for one launch; split the tokens", fn);
        const hipError_t e = launch_pipe64_act<DASS_ACT_RELU, kEpiGemm>(
            dim3((unsigned)blocks), stream, Y, T, d_int, static_cast<const uint16_t *>(Wdown), nullptr, ldd, d_int, d,
            nullptr, static_cast<uint16_t *>(out), ldo, tiles_t, tiles_n, super_rows);
        if (e != hipSuccess)
            return fail(DASS_ERR_HIP, "%s: cannot reserve %d bytes of LDS: %s", fn, P64_LDS, hipGetErrorString(e));
        return check_launch("down-projection kernel");
    }
}
