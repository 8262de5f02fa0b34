// Status strings, the thread-local error text, argument checks shared by the
// stage-2 entry points, and the factor kernel f = norm^alpha (Sec. 3 Eq. 4 with
// exponent alpha, Eq. 5 with exponent 1).
#include "dass_internal.h"

namespace dass {

char *error_buffer()
{
    static thread_local char buf[kErrorBufferSize] = {0};
    return buf;
}

dass_status check_score_args(const char *fn, const void *W, int64_t rows, int64_t cols, int64_t ld,
                             int dt, const float *norms, int norm_axis, int group_axis,
                             double alpha, const void *workspace, size_t workspace_bytes,
                             size_t workspace_needed)
{
    if (!W || !norms)
        return fail(DASS_ERR_NULL, "%s: W and norms must not be NULL", fn);
    if (!valid_dtype(dt))
        return fail(DASS_ERR_DTYPE, "%s: unknown dtype %d", fn, dt);
    if (!valid_axis(norm_axis) || !valid_axis(group_axis))
        return fail(DASS_ERR_ARG, "%s: axis must be DASS_AXIS_ROWS or DASS_AXIS_COLS", fn);
    if (rows <= 0 || cols <= 0)
        return fail(DASS_ERR_SHAPE, "%s: rows=%lld cols=%lld must be positive", fn,
                    (long long)rows, (long long)cols);
    if (ld < cols)
        return fail(DASS_ERR_SHAPE, "%s: ld=%lld smaller than cols=%lld", fn, (long long)ld,
                    (long long)cols);
    if (cols % 8 != 0)
        return fail(DASS_ERR_SHAPE, "%s: cols=%lld must be a multiple of 8", fn, (long long)cols);
    if (!std::isfinite(alpha) || alpha < 0.0)
        return fail(DASS_ERR_ARG, "%s: alpha must be finite and >= 0", fn);
    if (!aligned16(W) || !aligned16(norms))
        return fail(DASS_ERR_ALIGN, "%s: W and norms must be 16-byte aligned", fn);
    if (ld % vec_elems(dt) != 0)
        return fail(DASS_ERR_ALIGN, "%s: ld=%lld must be a multiple of %d elements", fn,
                    (long long)ld, vec_elems(dt));
    if (workspace_needed > 0) {
        if (!workspace || workspace_bytes < workspace_needed)
            return fail(DASS_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", fn,
                        workspace_needed, workspace ? workspace_bytes : (size_t)0);
        if (!aligned16(workspace))
            return fail(DASS_ERR_ALIGN, "%s: workspace must be 16-byte aligned", fn);
    }
    return DASS_OK;
}

// mode 0: f = 1, mode 1: f = norm, mode 2: f = sqrt(norm), mode 3: f = pow(norm, alpha).
// The f64 square root rounded to f32 is the correctly rounded f32 square root:
// sqrt of an f32 is never closer than 2^-51 (relative) to the midpoint of two
// adjacent f32 values, far more than the f64 routine's error.
__global__ void factor_kernel(const float *__restrict__ norms, int64_t n, int mode, double alpha,
                              float *__restrict__ f)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n)
        return;
    const double x = (double)norms[i];
    double v;
    if (mode == 0)
        v = 1.0;
    else if (mode == 1)
        v = x;
    else if (mode == 2)
        v = sqrt(x);
    else
        v = pow(x, alpha);
    f[i] = (float)v;
}

dass_status launch_factor(const float *norms, int64_t n, double alpha, float *f, hipStream_t stream)
{
    const int mode = alpha == 0.0 ? 0 : alpha == 1.0 ? 1 : alpha == 0.5 ? 2 : 3;
    const int block = 256;
    const unsigned grid = (unsigned)((n + block - 1) / block);
    hipLaunchKernelGGL(factor_kernel, dim3(grid), dim3(block), 0, stream, norms, n, mode, alpha, f);
    return check_launch("factor kernel");
}

}  // namespace dass

extern "C" const char *dass_status_string(dass_status s)
{
    switch (s) {
    case DASS_OK: return "DASS_OK";
    case DASS_ERR_NULL: return "DASS_ERR_NULL";
    case DASS_ERR_SHAPE: return "DASS_ERR_SHAPE";
    case DASS_ERR_DTYPE: return "DASS_ERR_DTYPE";
    case DASS_ERR_ARG: return "DASS_ERR_ARG";
    case DASS_ERR_ALIGN: return "DASS_ERR_ALIGN";
    case DASS_ERR_WORKSPACE: return "DASS_ERR_WORKSPACE";
    case DASS_ERR_HIP: return "DASS_ERR_HIP";
    }
    return "DASS_ERR_UNKNOWN";
}

extern "C" const char *dass_last_error_string(void) { return dass::error_buffer(); }

extern "C" int dass_version(void) { return 300; }  // 0.3.0: input norms, MLP output, 2:4 storage form, sparse down projection
