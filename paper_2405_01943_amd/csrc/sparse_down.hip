// Eq. 3 (Sec. 2.2) from the 2:4 compressed Down-Proj: out = y Wdown^T on the sparse matrix cores
// (v_smfmac_f32_32x32x32_bf16), the hardware use of N:M sparsity that Sec. 2.2 points to.
//
// The sparse operand of that instruction is its first one, so Wdown's output features are the
// MFMA "M" index and tokens the "N" index: a workgroup owns 256 features x 256 tokens, its four
// wavefronts 128 x 128 each (16 accumulator blocks = all 256 accumulation registers).
// Operand layout (checked on the GPU against a host product): a lane (row, half c) takes 8
// consecutive stored values of its row = the dense K range 16 c .. 16 c + 15 of the instruction's
// 32, the 16 bits of those four groups' position codes as its index operand, and from the dense
// side K 8 c .. 8 c + 7 and 16 + 8 c .. 16 + 8 c + 7.  The compressed form of dass_compress_24
// (groups along the columns) is exactly that: no shuffling, only addresses.
//
// K slabs of 64 dense columns go from global memory straight into a ring of three LDS stages
// (buffer_load ... lds): 256 rows x 64 B of values and 256 tokens x 128 B of y = 48 KB a stage;
// the codes come two slabs at a time (256 rows x 16 B, two 4 KB blocks behind the ring), so that
// a lane fetches 16 bytes of them, not 4.  Rows are XOR-swizzled in 16-byte chunks so that the fragment reads spread
// over the banks.  One barrier per slab; the loads of slab s + 2 are issued right after it.
#include "dass_internal.h"

#include <type_traits>

namespace dass {
namespace sp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) __bf16 bf16x16;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((address_space(3))) void *lds_ptr_t;

constexpr int kFM = 256, kTN = 256, kBK = 64;          // features, tokens per tile; dense K per slab
constexpr int kABytes = kFM * (kBK / 2) * 2;           // 16 KB of values
constexpr int kBBytes = kTN * kBK * 2;                 // 32 KB of y
constexpr int kStage = kABytes + kBBytes;              // 48 KB
constexpr int kStages = 3;
constexpr int kMBlock = kFM * 16;                      // codes of two slabs (128 dense K): 16 B a row, 4 KB
constexpr int kMBase = kStages * kStage;               // two such blocks behind the ring
constexpr int kLds = kMBase + 2 * kMBlock;             // 152 KB
// wave-loads a wavefront issues for slab s: 4 of values, 8 of y, and with every even slab the
// codes of that slab and the next
constexpr int kLoadsOdd = 12, kLoadsEven = 13;

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}
__device__ __forceinline__ void block_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}
// Two f32 rounded to bf16 (nearest even), `lo` in the low half of the word: one v_cvt_pk_bf16_f32.
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ uint32_t bf16_pair(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}

__global__ __launch_bounds__(256) void down_sparse24_kernel(
    const uint16_t *__restrict__ Y, int64_t T, int64_t ldy, const uint16_t *__restrict__ values, int64_t ldv,
    const uint8_t *__restrict__ meta, int64_t ldm, int64_t d, int64_t d_int, uint16_t *__restrict__ out,
    int64_t ldo, int64_t tiles_t, int64_t tiles_f)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];   // kLds bytes

    // ---- tile assignment: patches of 4 token tiles x 8 feature tiles, dealt to the 8 XCDs
    // (workgroup b runs on XCD b % 8), as in the calibration kernel
    constexpr int PT = 4, PF = 8;
    const int64_t np_f = (tiles_f + PF - 1) / PF;
    const int64_t idx = blockIdx.x / 8, within = idx % (PT * PF);
    const int64_t patch = (idx / (PT * PF)) * 8 + blockIdx.x % 8;
    const int64_t tile_t = (patch / np_f) * PT + within / PF, tile_f = (patch % np_f) * PF + within % PF;
    if (tile_t >= tiles_t || tile_f >= tiles_f)
        return;
    const int64_t t0 = tile_t * kTN, f0 = tile_f * kFM;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;   // feature half, token half of the tile
    const int fr = lane & 31, fc = lane >> 5;

    // ---- global -> LDS.  Rows past the end of a matrix lie beyond the end of its buffer
    // descriptor and read as zeros.
    const int64_t rows_f = d - f0 < kFM ? d - f0 : kFM, rows_t = T - t0 < kTN ? T - t0 : kTN;
    constexpr int kRawBuffer = 0x00020000;
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(values + f0 * ldv), 0, (int)((rows_f - 1) * ldv * 2 + d_int), kRawBuffer);
    const __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(meta + f0 * ldm), 0, (int)((rows_f - 1) * ldm + d_int / 8), kRawBuffer);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(Y + t0 * ldy), 0, (int)((rows_t - 1) * ldy * 2 + d_int * 2), kRawBuffer);
    // values: a wave-load is 16 rows x 64 B; lane l fills slot l % 4 of row l / 4 with chunk slot ^ (row / 4 & 3)
    uint32_t a_off[4], m_off, b_off[8];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int r = (wave * 4 + q) * 16 + (lane >> 2);
        a_off[q] = (uint32_t)((int64_t)r * ldv * 2 + (((lane & 3) ^ ((r >> 2) & 3)) * 16));
    }
    // codes: a wave-load is 64 rows x 16 B (two slabs), one row a lane
    m_off = (uint32_t)((int64_t)(wave * 64 + lane) * ldm);
    // y: a wave-load is 8 rows x 128 B; lane l fills slot l % 8 of row l / 8 with chunk slot ^ (row / 2 & 7)
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int r = (wave * 8 + q) * 8 + (lane >> 3);
        b_off[q] = (uint32_t)((int64_t)r * ldy * 2 + (((lane & 7) ^ ((r >> 1) & 7)) * 16));
    }
    // q-th wave-load of slab s: 0..3 values, 4..11 y, 12 (even slabs only) the codes of slabs s, s + 1
    auto load_one = [&](int s, int q) {
        char *st = lds + (s % kStages) * kStage;
        if (q < 4)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, (lds_ptr_t)(st + (wave * 4 + q) * 1024), 16, a_off[q], s * kBK, 0,
                                                     0);
        else if (q < 12)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ry, (lds_ptr_t)(st + kABytes + (wave * 8 + q - 4) * 1024), 16,
                                                     b_off[q - 4], s * kBK * 2, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rm, (lds_ptr_t)(lds + kMBase + ((s >> 1) & 1) * kMBlock + wave * 1024),
                                                     16, m_off, (s >> 1) * 16, 0, 0);
    };
    auto issue_slab = [&](int s) {   // prologue only
#pragma unroll
        for (int q = 0; q < kLoadsOdd; ++q)
            load_one(s, q);
        if ((s & 1) == 0)
            load_one(s, kLoadsOdd);
    };

    // ---- LDS -> registers
    int a_row[4], b_row[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        a_row[i] = wm * 128 + i * 32 + fr;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        b_row[j] = wn * 128 + j * 32 + fr;
    struct Frags {
        bf16x8 a[4], lo[4], hi[4];   // the dense operand of block j is lo[j] followed by hi[j]
    };
    // q-th of the 12 fragment reads of K step kk of the slab in stage st: 4 sparse, 8 dense halves
    auto read_one = [&](Frags &f, const char *st, int kk, int q) {
        if (q < 4) {
            const int r = a_row[q];
            f.a[q] = *reinterpret_cast<const bf16x8 *>(st + (r * 4 + ((2 * kk + fc) ^ ((r >> 2) & 3))) * 16);
        } else {
            const int j = (q - 4) >> 1, r = b_row[j];
            const char *row = st + kABytes + r * 128;
            const int sw = (r >> 1) & 7;
            if ((q & 1) == 0)
                f.lo[j] = *reinterpret_cast<const bf16x8 *>(row + (((4 * kk + fc) ^ sw) * 16));
            else
                f.hi[j] = *reinterpret_cast<const bf16x8 *>(row + (((4 * kk + 2 + fc) ^ sw) * 16));
        }
    };
    u32x2 codes[4], codes_next[4];   // the 16 nibbles of a slab of each of this lane's four rows
    auto read_codes = [&](u32x2 *c, int s, int i) {   // slab s: half s % 2 of the row's 16 bytes in block s / 2
        c[i] = *reinterpret_cast<const u32x2 *>(lds + kMBase + ((s >> 1) & 1) * kMBlock + a_row[i] * 16 + (s & 1) * 8);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0.0f;
    auto mfma = [&](const Frags &f, const u32x2 *c, int kk, int q) {
        const int i = q >> 2, j = q & 3;
        const bf16x16 b = __builtin_shufflevector(f.lo[j], f.hi[j], 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
        acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(f.a[i], b, acc[i][j], (int)(c[i][kk] >> (16 * fc)), 0, 0);
    };

    // ---- main loop.  A slab is two K steps of 16 sparse MFMAs.  Under the MFMAs of K step 0 go
    // the fragment reads of K step 1; then one barrier - slab s + 1 has landed, nobody reads slab
    // s from LDS any more, so its stage takes slab s + 3 - and under the MFMAs of K step 1 go those
    // 14 loads and the fragment reads of K step 0 of slab s + 1.
    const int S = (int)(d_int / kBK);   // the host guarantees d_int % 64 == 0
    issue_slab(0);
    if (S > 1)
        issue_slab(1);
    if (S > 2)
        issue_slab(2);
    if (S > 2)
        wait_vmcnt<kLoadsOdd + kLoadsEven>();   // slabs 1 and 2 may be in flight
    else if (S > 1)
        wait_vmcnt<kLoadsOdd>();
    else
        wait_vmcnt<0>();
    block_barrier();
    Frags fa, fb;
#pragma unroll
    for (int q = 0; q < 12; ++q)
        read_one(fa, lds, 0, q);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        read_codes(codes, 0, i);
    // MORE: a slab follows; LOAD: slab s + 3 exists; AHEAD: slab s + 2 exists (it may be in flight
    // at the barrier).  All three are compile-time: the steady state has no branch between MFMAs.
    // PAR: the parity of s (0, 1), which says how many loads slabs s + 2 and s + 3 are, or 2 when it
    // is only known at run time (the last slabs): then the barrier waits as if slab s + 2 were the
    // shorter kind (one load more has to land, harmless) and the codes' load is a run-time test.
    auto slab_body = [&](int s, auto more_tag, auto load_tag, auto ahead_tag, auto par_tag) {
        constexpr bool MORE = decltype(more_tag)::value, LOAD = decltype(load_tag)::value,
                       AHEAD = decltype(ahead_tag)::value;
        constexpr int PAR = decltype(par_tag)::value;
        constexpr int kAhead = PAR == 0 ? kLoadsEven : kLoadsOdd;                    // loads of slab s + 2
        constexpr int kIssue = PAR == 1 ? kLoadsEven : kLoadsOdd;                    // loads of slab s + 3
        const char *st = lds + (s % kStages) * kStage, *st_next = lds + ((s + 1) % kStages) * kStage;
#pragma unroll
        for (int q = 0; q < 16; ++q) {   // K step 0
            if (q < 12)
                read_one(fb, st, 1, q);
            mfma(fa, codes, 0, q);
            __builtin_amdgcn_sched_barrier(0);
        }
        // slab s + 1 has landed (only slab s + 2 may be in flight) and this wavefront holds its last
        // fragments of slab s: vmcnt(14 or 0), lgkmcnt(0)
        if (AHEAD)
            __builtin_amdgcn_s_waitcnt(0x0070 | kAhead);
        else
            __builtin_amdgcn_s_waitcnt(0x0070);
        block_barrier();
#pragma unroll
        for (int q = 0; q < 16; ++q) {   // K step 1
            if (LOAD && q < kIssue)
                load_one(s + 3, q);
            if (LOAD && PAR == 2 && q == kLoadsOdd && ((s + 3) & 1) == 0)   // uniform
                load_one(s + 3, kLoadsOdd);
            if (MORE) {
                if (q < 12)
                    read_one(fa, st_next, 0, q);
                else
                    read_codes(codes_next, s + 1, q - 12);
            }
            mfma(fb, codes, 1, q);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (MORE) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                codes[i] = codes_next[i];
        }
    };
    using Yes = std::true_type;
    using No = std::false_type;
    using Even = std::integral_constant<int, 0>;
    using Odd = std::integral_constant<int, 1>;
    using Any = std::integral_constant<int, 2>;
    int s = 0;
    for (; s + 4 < S; s += 2) {   // s is even here
        slab_body(s, Yes{}, Yes{}, Yes{}, Even{});
        slab_body(s + 1, Yes{}, Yes{}, Yes{}, Odd{});
    }
    if (s + 3 < S)
        slab_body(s++, Yes{}, Yes{}, Yes{}, Any{});   // slab S - 4 when the loop left it
    if (s + 2 < S)
        slab_body(s++, Yes{}, No{}, Yes{}, Any{});    // slab S - 3
    if (s + 1 < S)
        slab_body(s++, Yes{}, No{}, No{}, Any{});     // slab S - 2
    slab_body(s, No{}, No{}, No{}, Any{});            // slab S - 1

    // ---- epilogue: the tile goes to LDS as bf16 [token][feature] (row stride 528 B) and leaves it
    // in whole 16-byte chunks of output rows.  A lane holds, per block, 4 x 4 consecutive features
    // of one token: 8-byte writes.
    block_barrier();   // every wavefront is done with the last slab
    constexpr int SROW = kFM * 2 + 16;
    static_assert(kTN * SROW <= kLds, "the tile fits in the ring");
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int token = wn * 128 + j * 32 + fr, feature = wm * 128 + i * 32 + 8 * g + 4 * fc;
                u32x2 w;
                w[0] = bf16_pair(acc[i][j][4 * g], acc[i][j][4 * g + 1]);
                w[1] = bf16_pair(acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
                *reinterpret_cast<u32x2 *>(lds + token * SROW + feature * 2) = w;
            }
    __syncthreads();
    constexpr int CPR = kFM / 8;   // 16-byte chunks per tile row
    for (int c = tid; c < kTN * CPR; c += 256) {
        const int row = c / CPR, cc = c % CPR;
        const int64_t t = t0 + row, f = f0 + cc * 8;
        if (t < T && f < d)   // d is a multiple of 8: a chunk is inside or outside
            __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(lds + row * SROW + cc * 16),
                                        reinterpret_cast<u32x4 *>(out + t * ldo + f));   // streamed: not read again from L2
    }
}

}  // namespace sp
}  // namespace dass

extern "C" dass_status dass_down_proj_sparse24(const void *Y, int64_t T, int64_t ldy, const void *values, int64_t ldv,
                                               const uint8_t *meta, int64_t ldm, int64_t d, int64_t d_int,
                                               dass_dtype dt, void *out, int64_t ldo, void *hip_stream)
{
    using namespace dass;
    const char *fn = "dass_down_proj_sparse24";
    if (!Y || !values || !meta || !out)
        return fail(DASS_ERR_NULL, "%s: Y, values, meta and out must not be NULL", fn);
    if (!valid_dtype(dt))
        return fail(DASS_ERR_DTYPE, "%s: unknown dtype %d", fn, (int)dt);
    if (dt != DASS_BF16)
        return fail(DASS_ERR_DTYPE, "%s: only bf16 is implemented", fn);
    if (T <= 0 || d <= 0 || d_int <= 0)
        return fail(DASS_ERR_SHAPE, "%s: T=%lld d=%lld d_int=%lld must be positive", fn, (long long)T, (long long)d,
                    (long long)d_int);
    if (d_int % 64 != 0 || d % 8 != 0)
        return fail(DASS_ERR_SHAPE, "%s: d_int=%lld must be a multiple of 64 and d=%lld of 8", fn, (long long)d_int,
                    (long long)d);
    if (ldy < d_int || ldv < d_int / 2 || ldm < d_int / 8 || ldo < d)
        return fail(DASS_ERR_SHAPE, "%s: a leading dimension is shorter than its row", fn);
    if (!aligned16(Y) || !aligned16(values) || !aligned16(out) || (reinterpret_cast<uintptr_t>(meta) & 3u))
        return fail(DASS_ERR_ALIGN, "%s: Y, values and out must be 16-byte aligned, meta 4-byte", fn);
    if (ldy % 8 != 0 || ldv % 8 != 0 || ldo % 8 != 0 || ldm % 4 != 0)
        return fail(DASS_ERR_ALIGN, "%s: ldy, ldv, ldo must be multiples of 8 elements, ldm of 4 bytes", fn);
    // 32-bit byte offsets inside a tile's rows
    if ((int64_t)sp::kTN * ldy * 2 >= 0x7fffffffLL || (int64_t)sp::kFM * ldv * 2 >= 0x7fffffffLL ||
        (int64_t)sp::kFM * ldm >= 0x7fffffffLL)
        return fail(DASS_ERR_SHAPE, "%s: rows too long for the tile addressing", fn);
    const int64_t tiles_t = (T + sp::kTN - 1) / sp::kTN, tiles_f = (d + sp::kFM - 1) / sp::kFM;
    const int64_t patches = (tiles_t + 3) / 4 * ((tiles_f + 7) / 8);
    const int64_t blocks = (patches + 7) / 8 * 8 * 32;
    if (blocks > 0x7fffffffLL)
        return fail(DASS_ERR_SHAPE, "%s: too many tiles for one launch; split the tokens", fn);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(sp::down_sparse24_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, sp::kLds);
    if (e != hipSuccess)
        return fail(DASS_ERR_HIP, "%s: cannot reserve %d bytes of LDS: %s", fn, sp::kLds, hipGetErrorString(e));
    hipLaunchKernelGGL(sp::down_sparse24_kernel, dim3((unsigned)blocks), dim3(256), sp::kLds, stream,
                       static_cast<const uint16_t *>(Y), T, ldy, static_cast<const uint16_t *>(values), ldv, meta, ldm,
                       d, d_int, static_cast<uint16_t *>(out), ldo, tiles_t, tiles_f);
    return check_launch("sparse down-projection kernel");
}
