// 2:4 compressed form of a pruned matrix (the N:M pattern of Sec. 2.2 with N = 2, M = 4): for
// every group of 4 consecutive positions along the group axis, two values and the nibble
// p0 | p1 << 2 of their positions, p0 < p1.  The stored positions are the first two of
// (nonzero positions ascending) ++ (zero positions ascending): a group with at most two nonzeros
// is kept exactly, a denser one loses its surplus and is counted.
//
// One pass, bound by reading W once and writing half of it (HBM).  A thread owns one unit:
//   groups along the columns: 8 consecutive elements of a row (2 groups) -> 4 values, 1 byte
//   groups along the rows:    4 rows of one 16-byte column slot (8 bf16 / 4 f32 columns)
//                             -> 2 rows of the slot, 4 / 2 bytes
#include "select.h"

namespace dass {

constexpr int kCmpBlock = 256;
constexpr int kCmpUnits = 4;   // most units per thread, a block apart (loads in flight)

// code of a group from its 4-bit nonzero mask: 16 nibbles in one constant
constexpr uint64_t code_table()
{
    uint64_t t = 0;
    for (int mask = 0; mask < 16; ++mask) {
        int order[4] = {0, 0, 0, 0}, n = 0;
        for (int a = 0; a < 4; ++a)
            if (mask >> a & 1)
                order[n++] = a;
        for (int a = 0; a < 4; ++a)
            if (!(mask >> a & 1))
                order[n++] = a;
        const int p0 = order[0] < order[1] ? order[0] : order[1];
        const int p1 = order[0] < order[1] ? order[1] : order[0];
        t |= (uint64_t)(p0 | p1 << 2) << (4 * mask);
    }
    return t;
}
constexpr uint64_t kCodeOfMask = code_table();

__device__ __forceinline__ uint32_t code_of(uint32_t mask) { return (uint32_t)(kCodeOfMask >> (4 * mask)) & 15u; }

// bits of element e of a 16-byte vector, in the low bits
template <int DT>
__device__ __forceinline__ uint32_t bits_of(const u32x4 &v, int e)
{
    if constexpr (DT == DASS_BF16)
        return (v[e >> 1] >> (16 * (e & 1))) & 0xffffu;
    else
        return v[e];
}
template <int DT>
__device__ __forceinline__ bool nonzero_bits(uint32_t b)
{
    return (b & (DT == DASS_BF16 ? 0x7fffu : 0x7fffffffu)) != 0;   // -0 is a zero
}

__device__ __forceinline__ void add_surplus(long long *surplus_out, int mine)
{
    if (!surplus_out)
        return;
    int total = mine;
#pragma unroll
    for (int s = 32; s > 0; s >>= 1)
        total += __shfl_xor(total, s, 64);
    if ((threadIdx.x & 63) == 0 && total)
        atomicAdd(reinterpret_cast<unsigned long long *>(surplus_out), (unsigned long long)total);
}

// ---- groups along the columns.  Unit u of row r: elements 8 u .. 8 u + 7.
template <int DT, int UPT>
__global__ __launch_bounds__(kCmpBlock) void compress_cols_kernel(
    const void *__restrict__ Wv, int64_t rows, int64_t cols, int64_t ld, void *__restrict__ values,
    int64_t ldv, uint8_t *__restrict__ meta, int64_t ldm, long long *surplus_out, uint32_t blocks_per_row)
{
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    constexpr int VPU = DT == DASS_BF16 ? 1 : 2;   // 16-byte vectors per unit
    const int64_t r = blockIdx.x / blocks_per_row;
    const uint32_t bx = blockIdx.x % blocks_per_row;
    const int64_t units = cols / 8;
    const char *W = static_cast<const char *>(Wv) + r * ld * EB;
    char *V = static_cast<char *>(values) + r * ldv * EB;
    uint8_t *M = meta + r * ldm;

    u32x4 v[UPT][VPU];
    int64_t unit[UPT];
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
        unit[k] = ((int64_t)bx * UPT + k) * kCmpBlock + threadIdx.x;
        if (unit[k] < units) {
#pragma unroll
            for (int h = 0; h < VPU; ++h)
                v[k][h] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(W + (unit[k] * VPU + h) * 16));
        }
    }
    int surplus = 0;
    uint32_t outv[UPT][4], outb[UPT];
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
        outv[k][0] = outv[k][1] = outv[k][2] = outv[k][3] = outb[k] = 0;
        if (unit[k] >= units)
            continue;
        uint32_t kept[4], byte = 0;
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            uint32_t b[4], mask = 0;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int e = 4 * g + a;   // element of the unit
                if constexpr (DT == DASS_BF16)
                    b[a] = bits_of<DT>(v[k][0], e);
                else
                    b[a] = bits_of<DT>(v[k][g], a);   // an f32 vector is one group
                mask |= nonzero_bits<DT>(b[a]) ? 1u << a : 0u;
            }
            surplus += __popc(mask) > 2;
            const uint32_t code = code_of(mask), p0 = code & 3u, p1 = code >> 2;
            kept[2 * g] = p0 == 0 ? b[0] : p0 == 1 ? b[1] : b[2];        // p0 <= 2
            kept[2 * g + 1] = p1 == 1 ? b[1] : p1 == 2 ? b[2] : b[3];    // p1 >= 1
            byte |= code << (4 * g);
        }
        outv[k][0] = DT == DASS_BF16 ? kept[0] | kept[1] << 16 : kept[0];
        outv[k][1] = DT == DASS_BF16 ? kept[2] | kept[3] << 16 : kept[1];
        outv[k][2] = kept[2];
        outv[k][3] = kept[3];
        outb[k] = byte;
    }
    // Stores.  Neighbouring lanes hold neighbouring units (a thread's unit index has the parity
    // of its lane), so two lanes' bf16 values make one 16-byte store and four lanes' codes one
    // 32-bit store where the row's alignment allows; the ragged end of a row and unaligned rows
    // store piecewise.  Every lane takes part in the exchanges.
    const int lane = threadIdx.x & 63;
    const bool wide_v = ((reinterpret_cast<uintptr_t>(V)) & 15u) == 0;
    const bool wide_m = ((reinterpret_cast<uintptr_t>(M)) & 3u) == 0;
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
        const bool have = unit[k] < units;
        if constexpr (DT == DASS_BF16) {
            const uint32_t nx = __shfl_down(outv[k][0], 1, 64), ny = __shfl_down(outv[k][1], 1, 64);
            const bool pair = wide_v && unit[k] + 1 < units;   // uniform over a lane pair
            if (have && pair && (lane & 1) == 0) {
                u32x4 o = {outv[k][0], outv[k][1], nx, ny};
                *reinterpret_cast<u32x4 *>(V + unit[k] * 8) = o;
            } else if (have && !(wide_v && (lane & 1) && unit[k] < units)) {
                uint2 o;
                o.x = outv[k][0];
                o.y = outv[k][1];
                *reinterpret_cast<uint2 *>(V + unit[k] * 8) = o;
            }
        } else if (have) {
            u32x4 o = {outv[k][0], outv[k][1], outv[k][2], outv[k][3]};
            *reinterpret_cast<u32x4 *>(V + unit[k] * 16) = o;
        }
        const uint32_t b1 = __shfl_down(outb[k], 1, 64), b2 = __shfl_down(outb[k], 2, 64),
                       b3 = __shfl_down(outb[k], 3, 64);
        const int64_t quad = unit[k] & ~(int64_t)3;   // first unit of this lane's group of four
        const bool whole = wide_m && quad + 3 < units;   // uniform over the four lanes
        if (have && whole) {
            if ((lane & 3) == 0)
                *reinterpret_cast<uint32_t *>(M + unit[k]) = outb[k] | b1 << 8 | b2 << 16 | b3 << 24;
        } else if (have) {
            M[unit[k]] = (uint8_t)outb[k];
        }
    }
    add_surplus(surplus_out, surplus);
}

// ---- groups along the rows.  Unit: group g (rows 4 g .. 4 g + 3) of column slot s.
template <int DT, int UPT>
__global__ __launch_bounds__(kCmpBlock) void compress_rows_kernel(
    const void *__restrict__ Wv, int64_t rows, int64_t cols, int64_t ld, void *__restrict__ values,
    int64_t ldv, uint8_t *__restrict__ meta, int64_t ldm, long long *surplus_out, uint32_t blocks_per_row)
{
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    constexpr int EPV = DT == DASS_BF16 ? 8 : 4;
    const int64_t g = blockIdx.x / blocks_per_row;   // group row
    const uint32_t bx = blockIdx.x % blocks_per_row;
    const int64_t slots = cols / EPV;
    const char *W = static_cast<const char *>(Wv) + 4 * g * ld * EB;
    char *V = static_cast<char *>(values) + 2 * g * ldv * EB;
    uint8_t *M = meta + g * ldm;

    u32x4 v[UPT][4];
    int64_t slot[UPT];
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
        slot[k] = ((int64_t)bx * UPT + k) * kCmpBlock + threadIdx.x;
        if (slot[k] < slots) {
#pragma unroll
            for (int a = 0; a < 4; ++a)
                v[k][a] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(W + a * ld * EB + slot[k] * 16));
        }
    }
    int surplus = 0;
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
        if (slot[k] >= slots)
            continue;
        uint32_t lo[EPV], hi[EPV], codes = 0;
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            uint32_t b[4], mask = 0;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                b[a] = bits_of<DT>(v[k][a], e);
                mask |= nonzero_bits<DT>(b[a]) ? 1u << a : 0u;
            }
            surplus += __popc(mask) > 2;
            const uint32_t code = code_of(mask), p0 = code & 3u, p1 = code >> 2;
            lo[e] = p0 == 0 ? b[0] : p0 == 1 ? b[1] : b[2];
            hi[e] = p1 == 1 ? b[1] : p1 == 2 ? b[2] : b[3];
            codes |= code << (4 * e);
        }
        u32x4 o0, o1;
        if constexpr (DT == DASS_BF16) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                o0[w] = lo[2 * w] | lo[2 * w + 1] << 16;
                o1[w] = hi[2 * w] | hi[2 * w + 1] << 16;
            }
            *reinterpret_cast<uint32_t *>(M + slot[k] * 4) = codes;
        } else {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                o0[w] = lo[w];
                o1[w] = hi[w];
            }
            *reinterpret_cast<uint16_t *>(M + slot[k] * 2) = (uint16_t)codes;
        }
        *reinterpret_cast<u32x4 *>(V + slot[k] * 16) = o0;
        *reinterpret_cast<u32x4 *>(V + ldv * EB + slot[k] * 16) = o1;
    }
    add_surplus(surplus_out, surplus);
}

}  // namespace dass

extern "C" dass_status dass_compress_24(const void *W, int64_t rows, int64_t cols, int64_t ld, dass_dtype dt,
                                        dass_axis group_axis, void *values_out, int64_t ldv, uint8_t *meta_out,
                                        int64_t ldm, long long *surplus_out, void *hip_stream)
{
    using namespace dass;
    const char *fn = "dass_compress_24";
    if (!W || !values_out || !meta_out)
        return fail(DASS_ERR_NULL, "%s: W, values_out and meta_out must not be NULL", fn);
    if (!valid_dtype(dt))
        return fail(DASS_ERR_DTYPE, "%s: unknown dtype %d", fn, (int)dt);
    if (group_axis != DASS_AXIS_ROWS && group_axis != DASS_AXIS_COLS)
        return fail(DASS_ERR_ARG, "%s: unknown axis %d", fn, (int)group_axis);
    if (rows <= 0 || cols <= 0)
        return fail(DASS_ERR_SHAPE, "%s: rows=%lld cols=%lld must be positive", fn, (long long)rows, (long long)cols);
    const int vec = vec_elems(dt);
    const bool along_rows = group_axis == DASS_AXIS_ROWS;
    if (cols % 8 != 0 || (along_rows && rows % 4 != 0))
        return fail(DASS_ERR_SHAPE, "%s: cols must be a multiple of 8%s", fn,
                    along_rows ? " and rows a multiple of 4" : "");
    const int64_t vcols = along_rows ? cols : cols / 2, mcols = along_rows ? cols / 2 : cols / 8;
    if (ld < cols || ldv < vcols || ldm < mcols)
        return fail(DASS_ERR_SHAPE, "%s: a leading dimension is shorter than its row", fn);
    // along the rows a thread writes whole 16-byte vectors of values and 2 or 4 bytes of codes at
    // once; along the columns 4 values (8 or 16 bytes) and single bytes
    if (!aligned16(W) || !aligned16(values_out) || (along_rows && (reinterpret_cast<uintptr_t>(meta_out) & 3u)) ||
        (surplus_out && (reinterpret_cast<uintptr_t>(surplus_out) & 7u)))
        return fail(DASS_ERR_ALIGN, "%s: W and values_out must be 16-byte, meta_out 4-byte, surplus_out 8-byte aligned",
                    fn);
    if (ld % vec != 0 || ldv % (along_rows ? vec : 4) != 0 || (along_rows && ldm % 4 != 0))
        return fail(DASS_ERR_ALIGN, "%s: ld must be a multiple of %d elements, ldv of %d, ldm of %d bytes", fn, vec,
                    along_rows ? vec : 4, along_rows ? 4 : 1);
    // the outputs may not overlap the input: a unit is read by one thread, written by another's range
    const uintptr_t w0 = reinterpret_cast<uintptr_t>(W), w1 = w0 + (uintptr_t)rows * ld * elem_bytes(dt);
    const uintptr_t v0 = reinterpret_cast<uintptr_t>(values_out),
                    v1 = v0 + (uintptr_t)(along_rows ? rows / 2 : rows) * ldv * elem_bytes(dt);
    if (v0 < w1 && w0 < v1)
        return fail(DASS_ERR_ARG, "%s: values_out overlaps W", fn);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int64_t per_line = along_rows ? cols / vec : cols / 8;      // units of one (group) row
    const int64_t lines = along_rows ? rows / 4 : rows;
    // Units per thread (4, 2 or 1, a block apart): the count that wastes the fewest lanes on the
    // ragged last block of a line; more units per thread on a tie (more loads in flight).
    int upt = kCmpUnits;
    int64_t bpr = 0;
    for (int u = kCmpUnits, best = -1; u >= 1; u /= 2) {
        const int64_t span = (int64_t)kCmpBlock * u, b = (per_line + span - 1) / span;
        const int fill = (int)(per_line * 1024 / (b * span));
        if (fill > best) {
            best = fill;
            upt = u;
            bpr = b;
        }
    }
    if (bpr * lines > 0x7fffffffLL)
        return fail(DASS_ERR_SHAPE, "%s: too many blocks for one launch; split the rows", fn);
    const dim3 grid((unsigned)(bpr * lines)), block(kCmpBlock);
    using k_t = void (*)(const void *, int64_t, int64_t, int64_t, void *, int64_t, uint8_t *, int64_t, long long *,
                         uint32_t);
    k_t k;
    if (along_rows) {
        if (dt == DASS_BF16)
            k = upt == 4 ? compress_rows_kernel<DASS_BF16, 4> : upt == 2 ? compress_rows_kernel<DASS_BF16, 2>
                                                                          : compress_rows_kernel<DASS_BF16, 1>;
        else
            k = upt == 4 ? compress_rows_kernel<DASS_F32, 4> : upt == 2 ? compress_rows_kernel<DASS_F32, 2>
                                                                         : compress_rows_kernel<DASS_F32, 1>;
    } else {
        if (dt == DASS_BF16)
            k = upt == 4 ? compress_cols_kernel<DASS_BF16, 4> : upt == 2 ? compress_cols_kernel<DASS_BF16, 2>
                                                                          : compress_cols_kernel<DASS_BF16, 1>;
        else
            k = upt == 4 ? compress_cols_kernel<DASS_F32, 4> : upt == 2 ? compress_cols_kernel<DASS_F32, 2>
                                                                         : compress_cols_kernel<DASS_F32, 1>;
    }
    hipLaunchKernelGGL(k, grid, block, 0, stream, W, rows, cols, ld, values_out, ldv, meta_out, ldm, surplus_out,
                       (uint32_t)bpr);
    return check_launch("compress kernel");
}
