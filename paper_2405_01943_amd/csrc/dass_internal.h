// Library-internal helpers shared by the entry points of libdass: error
// reporting, argument checks, launch checks.  Nothing here is exported.
#pragma once

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "../../include/dass.h"

namespace dass {

// Thread-local text of the most recent failure on this thread.
char *error_buffer();
constexpr size_t kErrorBufferSize = 512;

inline dass_status fail(dass_status s, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), kErrorBufferSize, fmt, ap);
    va_end(ap);
    return s;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool valid_dtype(int dt) { return dt == DASS_F32 || dt == DASS_BF16; }
inline bool valid_axis(int a) { return a == DASS_AXIS_ROWS || a == DASS_AXIS_COLS; }
inline int elem_bytes(int dt) { return dt == DASS_BF16 ? 2 : 4; }
inline int vec_elems(int dt) { return 16 / elem_bytes(dt); }  // elements per 16-byte access

inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Turn a failed launch into DASS_ERR_HIP with the runtime's message.
inline dass_status check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail(DASS_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return DASS_OK;
}

// Checks shared by the two stage-2 entry points (everything except the
// selection-specific arguments).  Returns DASS_OK or the failure.
dass_status check_score_args(const char *fn, const void *W, int64_t rows, int64_t cols, int64_t ld,
                             int dt, const float *norms, int norm_axis, int group_axis,
                             double alpha, const void *workspace, size_t workspace_bytes,
                             size_t workspace_needed);

// Enqueue f[i] = norms[i]^alpha (see include/dass.h for the special cases).
dass_status launch_factor(const float *norms, int64_t n, double alpha, float *f, hipStream_t stream);

}  // namespace dass
