// The input-feature norms of the Wanda metric (Sec. 2.1 Eq. 1): ||X_j||_2 over all tokens, the
// quantity that the Down-Proj score of Eq. 5 is built like and the paper's main comparison
// system scores every layer with.  sumsq[j] (+)= sum_t X[t, j]^2, norms = sqrt(sumsq).
//
// The pass is bound by reading X once (HBM).  Two kernels, no atomics, so the result does not
// depend on the order in which workgroups finish:
//   input_partial_kernel  a thread owns the 16 bytes of one column slot (8 bf16 / 4 f32
//                         columns) and the rows of one row block; it adds the squares in f32
//                         and writes its sums to partial[row block][column].
//   input_reduce_kernel   adds the row blocks' partial sums of a column in f64, in a fixed order,
//                         and writes sumsq (optionally added to what is there) and the norm.
#include "select.h"

namespace dass {

constexpr int kInBlock = 256;     // threads = column slots per workgroup
constexpr int kInRows = 512;      // rows per row block
constexpr int kInUnroll = 8;      // rows in flight per thread

template <int DT>
__global__ __launch_bounds__(kInBlock) void input_partial_kernel(
    const void *__restrict__ Xv, int64_t T, int64_t ldx, int64_t d, float *__restrict__ partial)
{
    constexpr int EPV = DT == DASS_BF16 ? 8 : 4;
    constexpr int EB = DT == DASS_BF16 ? 2 : 4;
    const int64_t slots = d / EPV;
    const uint32_t nbx = (uint32_t)((slots + kInBlock - 1) / kInBlock);
    const uint32_t bx = blockIdx.x % nbx, rb = blockIdx.x / nbx;
    const int64_t slot = (int64_t)bx * kInBlock + threadIdx.x;
    if (slot >= slots)
        return;
    const int64_t r0 = (int64_t)rb * kInRows;
    const int64_t r1 = r0 + kInRows < T ? r0 + kInRows : T;
    const char *X = static_cast<const char *>(Xv) + slot * 16;

    float acc[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e)
        acc[e] = 0.0f;
    int64_t r = r0;
    for (; r + kInUnroll <= r1; r += kInUnroll) {
        u32x4 v[kInUnroll];
#pragma unroll
        for (int k = 0; k < kInUnroll; ++k)
            v[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(X + (r + k) * ldx * EB));
#pragma unroll
        for (int k = 0; k < kInUnroll; ++k)
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                const float x = elem_of<DT>(v[k], e);
                acc[e] = fmaf(x, x, acc[e]);
            }
    }
    for (; r < r1; ++r) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(X + r * ldx * EB));
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            const float x = elem_of<DT>(v, e);
            acc[e] = fmaf(x, x, acc[e]);
        }
    }
    float *out = partial + (int64_t)rb * d + slot * EPV;
#pragma unroll
    for (int q = 0; q < EPV / 4; ++q) {
        u32x4 w;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = __float_as_uint(acc[4 * q + i]);
        *reinterpret_cast<u32x4 *>(out + 4 * q) = w;
    }
}

// A workgroup owns 64 columns; wavefront w adds the partial sums of every 4th row block
// (w, w + 4, ...) in f64, then the four are added in a fixed order.
__global__ __launch_bounds__(256) void input_reduce_kernel(
    const float *__restrict__ partial, int64_t n_row_blocks, int64_t d, float *__restrict__ sumsq,
    int accumulate, float *__restrict__ norms)
{
    __shared__ double part[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t j = (int64_t)blockIdx.x * 64 + lane;
    double s = 0.0;
    if (j < d) {
        int64_t b = w;
        for (; b + 12 < n_row_blocks; b += 16) {   // four loads in flight
            const float x0 = partial[b * d + j], x1 = partial[(b + 4) * d + j], x2 = partial[(b + 8) * d + j],
                        x3 = partial[(b + 12) * d + j];
            s += (double)x0;
            s += (double)x1;
            s += (double)x2;
            s += (double)x3;
        }
        for (; b < n_row_blocks; b += 4)
            s += (double)partial[b * d + j];
    }
    part[w][lane] = s;
    __syncthreads();
    if (w == 0 && j < d) {
        double total = accumulate ? (double)sumsq[j] : 0.0;
        total += part[0][lane];
        total += part[1][lane];
        total += part[2][lane];
        total += part[3][lane];
        const float s32 = (float)total;
        sumsq[j] = s32;
        if (norms)
            norms[j] = (float)sqrt((double)s32);
    }
}

}  // namespace dass

extern "C" size_t dass_input_norms_workspace_bytes(int64_t T, int64_t d)
{
    if (T <= 0 || d <= 0)
        return 0;
    const int64_t n_row_blocks = (T + dass::kInRows - 1) / dass::kInRows;
    return dass::round_up((size_t)n_row_blocks * (size_t)d * sizeof(float), 256);
}

extern "C" dass_status dass_input_norms(const void *X, int64_t T, int64_t ldx, int64_t d, dass_dtype dt,
                                        float *sumsq, int accumulate, float *norms_out, void *workspace,
                                        size_t workspace_bytes, void *hip_stream)
{
    using namespace dass;
    const char *fn = "dass_input_norms";
    if (!X || !sumsq)
        return fail(DASS_ERR_NULL, "%s: X and sumsq must not be NULL", fn);
    if (!valid_dtype(dt))
        return fail(DASS_ERR_DTYPE, "%s: unknown dtype %d", fn, (int)dt);
    if (T <= 0 || d <= 0)
        return fail(DASS_ERR_SHAPE, "%s: T=%lld d=%lld must be positive", fn, (long long)T, (long long)d);
    if (ldx < d)
        return fail(DASS_ERR_SHAPE, "%s: ldx=%lld smaller than d=%lld", fn, (long long)ldx, (long long)d);
    if (d % 8 != 0)
        return fail(DASS_ERR_SHAPE, "%s: d=%lld must be a multiple of 8", fn, (long long)d);
    if (!aligned16(X) || !aligned16(sumsq) || (norms_out && !aligned16(norms_out)))
        return fail(DASS_ERR_ALIGN, "%s: X, sumsq and norms_out must be 16-byte aligned", fn);
    if (ldx % vec_elems(dt) != 0)
        return fail(DASS_ERR_ALIGN, "%s: ldx=%lld must be a multiple of %d elements", fn, (long long)ldx,
                    vec_elems(dt));
    const size_t need = dass_input_norms_workspace_bytes(T, d);
    if (!workspace || workspace_bytes < need)
        return fail(DASS_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn, need,
                    workspace ? workspace_bytes : (size_t)0);
    if (!aligned16(workspace))
        return fail(DASS_ERR_ALIGN, "%s: workspace must be 16-byte aligned", fn);

    const int64_t n_row_blocks = (T + kInRows - 1) / kInRows;
    const int64_t slots = d / vec_elems(dt);
    const int64_t nbx = (slots + kInBlock - 1) / kInBlock;
    if (nbx * n_row_blocks > 0x7fffffffLL)
        return fail(DASS_ERR_SHAPE, "%s: too many tokens for one launch; split them", fn);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    float *partial = static_cast<float *>(workspace);
    if (dt == DASS_BF16)
        hipLaunchKernelGGL(input_partial_kernel<DASS_BF16>, dim3((unsigned)(nbx * n_row_blocks)), dim3(kInBlock), 0,
                           stream, X, T, ldx, d, partial);
    else
        hipLaunchKernelGGL(input_partial_kernel<DASS_F32>, dim3((unsigned)(nbx * n_row_blocks)), dim3(kInBlock), 0,
                           stream, X, T, ldx, d, partial);
    dass_status s = check_launch("input-norm kernel");
    if (s != DASS_OK)
        return s;
    hipLaunchKernelGGL(input_reduce_kernel, dim3((unsigned)((d + 63) / 64)), dim3(256), 0, stream,
                       (const float *)partial, n_row_blocks, d, sumsq, accumulate, norms_out);
    return check_launch("input-norm reduction");
}
