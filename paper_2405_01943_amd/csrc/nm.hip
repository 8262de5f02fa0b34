// Stage 2, N:M: score every weight as |W| * f (Sec. 3 Eq. 4 / Eq. 5), keep the
// n_keep best of every m consecutive positions along the group axis (Sec. 3
// "Extension to N:M Sparsity"), write +0 over the rest in place.
//
// One streaming pass: every weight is read once and written once with 16-byte
// accesses; selection happens in registers on the exact f64 product.
#include "select.h"

#include <mutex>

namespace dass {

constexpr int kBlock = 256;

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

}  // namespace dass

extern "C" size_t dass_nm_workspace_bytes(int64_t rows, int64_t cols, dass_axis norm_axis)
{
    const int64_t n = norm_axis == DASS_AXIS_ROWS ? rows : cols;
    return n > 0 ? dass::round_up((size_t)n * sizeof(float), 256) : 0;
}

extern "C" dass_status dass_score_mask_nm(void *W, int64_t rows, int64_t cols, int64_t ld,
                                          dass_dtype dt, const float *norms, dass_axis norm_axis,
                                          dass_axis group_axis, double alpha, int n_keep, int m,
                                          uint8_t *mask_out, void *workspace,
                                          size_t workspace_bytes, void *hip_stream)
{
    using namespace dass;
    const char *fn = "dass_score_mask_nm";
    dass_status st = check_score_args(fn, W, rows, cols, ld, dt, norms, norm_axis, group_axis, alpha,
                                      workspace, workspace_bytes,
                                      dass_nm_workspace_bytes(rows, cols, norm_axis));
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

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
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
