// Calls every entry point of include/dass.h with arguments that must be rejected on the host, in a
// build of the library whose host code carries AddressSanitizer and UndefinedBehaviorSanitizer
// (tests/test_sanitizers.py builds and runs it; no GPU is needed: every call returns before its first
// HIP call).  Prints one line per call, "<label> <status name>"; the test holds the expected names.
#include <cstdio>
#include <cmath>

#include "../include/dass.h"

static void *const FAKE = reinterpret_cast<void *>(0x1000);       // aligned, never dereferenced
static void *const FAKE2 = reinterpret_cast<void *>(0x10000000);
static void *const FAKE3 = reinterpret_cast<void *>(0x20000000);
static void *const ODD = reinterpret_cast<void *>(0x1004);

static void show(const char *label, dass_status s)
{
    std::printf("%s %s\n", label, dass_status_string(s));
    if (s != DASS_OK && dass_last_error_string()[0] == '\0')
        std::printf("%s MISSING-ERROR-TEXT\n", label);
}

static dass_status nm(void *W, int64_t rows, int64_t cols, int64_t ld, int dt, const void *norms, int na, int ga,
                      double alpha, int n, int m, void *ws, size_t wsb)
{
    return dass_score_mask_nm(W, rows, cols, ld, (dass_dtype)dt, static_cast<const float *>(norms), (dass_axis)na,
                              (dass_axis)ga, alpha, n, m, nullptr, ws, wsb, nullptr);
}

int main()
{
    const float *F = static_cast<const float *>(FAKE);
    // ---- dass_score_mask_nm
    show("nm_null_W", nm(nullptr, 64, 64, 64, 1, FAKE, 1, 1, 1.0, 2, 4, FAKE, 4096));
    show("nm_null_norms", nm(FAKE, 64, 64, 64, 1, nullptr, 1, 1, 1.0, 2, 4, FAKE, 4096));
    show("nm_dtype", nm(FAKE, 64, 64, 64, 5, FAKE, 1, 1, 1.0, 2, 4, FAKE, 4096));
    show("nm_rows0", nm(FAKE, 0, 64, 64, 1, FAKE, 1, 1, 1.0, 2, 4, FAKE, 4096));
    show("nm_ld", nm(FAKE, 64, 64, 56, 1, FAKE, 1, 1, 1.0, 2, 4, FAKE, 4096));
    show("nm_cols8", nm(FAKE, 64, 60, 64, 1, FAKE, 1, 1, 1.0, 2, 4, FAKE, 4096));
    show("nm_ragged_groups", nm(FAKE, 6, 64, 64, 1, FAKE, 0, 0, 1.0, 2, 4, FAKE, 4096));
    show("nm_m3", nm(FAKE, 64, 64, 64, 1, FAKE, 1, 1, 1.0, 2, 3, FAKE, 4096));
    show("nm_keep_all", nm(FAKE, 64, 64, 64, 1, FAKE, 1, 1, 1.0, 4, 4, FAKE, 4096));
    show("nm_alpha_nan", nm(FAKE, 64, 64, 64, 1, FAKE, 1, 1, std::nan(""), 2, 4, FAKE, 4096));
    show("nm_alpha_neg", nm(FAKE, 64, 64, 64, 1, FAKE, 1, 1, -0.5, 2, 4, FAKE, 4096));
    show("nm_axis", nm(FAKE, 64, 64, 64, 1, FAKE, 2, 1, 1.0, 2, 4, FAKE, 4096));
    show("nm_align", nm(ODD, 64, 64, 64, 1, FAKE, 1, 1, 1.0, 2, 4, FAKE, 4096));
    show("nm_ld_align", nm(FAKE, 64, 64, 68, 1, FAKE, 1, 1, 1.0, 2, 4, FAKE, 4096));
    show("nm_no_ws", nm(FAKE, 64, 64, 64, 1, FAKE, 1, 1, 1.0, 2, 4, nullptr, 0));
    show("nm_small_ws", nm(FAKE, 64, 64, 64, 1, FAKE, 1, 1, 1.0, 2, 4, FAKE, 8));
    show("nm_huge", nm(FAKE, int64_t(1) << 62, 8, 8, 1, FAKE, 1, 0, 1.0, 2, 4, FAKE, 4096));
    std::printf("nm_ws_bytes %zu\n", dass_nm_workspace_bytes(11008, 4096, DASS_AXIS_ROWS));
    // ---- batched
    {
        dass_nm_task t[3];
        for (auto &k : t)
            k = dass_nm_task{FAKE, 64, 64, 64, F, DASS_AXIS_COLS, DASS_AXIS_COLS, 1.0, nullptr};
        show("batched_empty", dass_score_mask_nm_batched(t, 0, DASS_BF16, 2, 4, FAKE, 4096, nullptr));
        t[1].W = nullptr;
        show("batched_null_task1", dass_score_mask_nm_batched(t, 3, DASS_BF16, 2, 4, FAKE, 4096, nullptr));
        std::printf("batched_text %s\n", dass_last_error_string());
        t[1].W = FAKE;
        t[2].cols = 60;
        show("batched_shape_task2", dass_score_mask_nm_batched(t, 3, DASS_BF16, 2, 4, FAKE, 4096, nullptr));
        show("batched_null_array", dass_score_mask_nm_batched(nullptr, 3, DASS_BF16, 2, 4, FAKE, 4096, nullptr));
        show("batched_negative", dass_score_mask_nm_batched(t, -1, DASS_BF16, 2, 4, FAKE, 4096, nullptr));
        std::printf("batched_ws_bytes %zu\n", dass_nm_batched_workspace_bytes(t, 3));
    }
    // ---- unstructured, both forms
    auto un = [&](void *W, int64_t cols, int64_t n_prune, void *ws, size_t wsb) {
        return dass_score_mask_unstructured(W, 64, cols, 64, DASS_BF16, F, DASS_AXIS_COLS, DASS_AXIS_COLS, 1.0, n_prune,
                                            nullptr, ws, wsb, nullptr);
    };
    show("un_neg", un(FAKE, 64, -1, FAKE, 4096));
    show("un_too_many", un(FAKE, 64, 65, FAKE, 4096));
    show("un_no_ws", un(FAKE, 64, 8, nullptr, 0));
    show("un_null", un(nullptr, 64, 8, FAKE, 4096));
    show("un_cols", un(FAKE, 12, 8, FAKE, 4096));
    std::printf("un_ws_bytes %zu\n", dass_unstructured_workspace_bytes(28672, 8192, DASS_BF16, DASS_AXIS_ROWS, DASS_AXIS_ROWS));
    show("un_static_limit", dass_score_mask_unstructured_static(FAKE, 65544, 8, 8, DASS_BF16, F, DASS_AXIS_ROWS,
                                                                DASS_AXIS_COLS, 1.0, 4, nullptr, nullptr));
    // ---- calibration
    auto cal = [&](const void *X, int64_t T, int64_t ldx, int64_t d, int dt, int act, float *sumsq, int64_t ldw) {
        return dass_calib_norms(X, T, ldx, FAKE, FAKE, ldw, d, 8, (dass_dtype)dt, (dass_act)act, sumsq, 0, nullptr, nullptr,
                                0, nullptr);
    };
    float *S = static_cast<float *>(FAKE);
    show("calib_null", cal(nullptr, 16, 64, 64, 1, 0, S, 64));
    show("calib_null_sumsq", cal(FAKE, 16, 64, 64, 1, 0, nullptr, 64));
    show("calib_dtype", cal(FAKE, 16, 64, 64, 2, 0, S, 64));
    show("calib_act", cal(FAKE, 16, 64, 64, 1, 4, S, 64));
    show("calib_T0", cal(FAKE, 0, 64, 64, 1, 0, S, 64));
    show("calib_d8", cal(FAKE, 16, 64, 60, 1, 0, S, 64));
    show("calib_ldx", cal(FAKE, 16, 32, 64, 1, 0, S, 64));
    show("calib_align", cal(ODD, 16, 64, 64, 1, 0, S, 64));
    show("calib_ldw_align", cal(FAKE, 16, 64, 64, 1, 0, S, 68));
    show("calib_too_many_tiles", cal(FAKE, int64_t(1) << 40, 64, 64, 1, 0, S, 64));
    show("calib_too_many_tiles_f32", cal(FAKE, int64_t(1) << 40, 64, 64, 0, 0, S, 64));
    show("calib_too_many_tiles_ragged_d", cal(FAKE, int64_t(1) << 42, 40, 40, 1, 0, S, 40));
    // ---- input norms
    auto inn = [&](const void *X, int64_t T, int64_t ldx, int64_t d, int dt, float *sumsq, void *ws, size_t wsb) {
        return dass_input_norms(X, T, ldx, d, (dass_dtype)dt, sumsq, 0, nullptr, ws, wsb, nullptr);
    };
    show("in_null", inn(nullptr, 64, 64, 64, 1, S, FAKE, 1 << 20));
    show("in_dtype", inn(FAKE, 64, 64, 64, 7, S, FAKE, 1 << 20));
    show("in_T0", inn(FAKE, 0, 64, 64, 1, S, FAKE, 1 << 20));
    show("in_d", inn(FAKE, 64, 64, 60, 1, S, FAKE, 1 << 20));
    show("in_align", inn(ODD, 64, 64, 64, 1, S, FAKE, 1 << 20));
    show("in_ws", inn(FAKE, 64, 64, 64, 1, S, FAKE, 64));
    std::printf("in_ws_bytes %zu\n", dass_input_norms_workspace_bytes(262144, 4096));
    // ---- MLP output
    auto fwd = [&](const void *X, int64_t T, int64_t d, int64_t d_int, int dt, void *out, int64_t ldo, size_t wsb) {
        return dass_mlp_forward(X, T, d, FAKE, FAKE, d, FAKE, d_int, d, d_int, (dass_dtype)dt, DASS_ACT_SILU, out, ldo, FAKE,
                                wsb, nullptr);
    };
    show("fwd_null", fwd(nullptr, 256, 128, 192, 1, FAKE, 128, 1 << 20));
    show("fwd_out_null", fwd(FAKE, 256, 128, 192, 1, nullptr, 128, 1 << 20));
    show("fwd_dtype", fwd(FAKE, 256, 128, 192, 0, FAKE, 128, 1 << 20));
    show("fwd_T0", fwd(FAKE, 0, 128, 192, 1, FAKE, 128, 1 << 20));
    show("fwd_d64", fwd(FAKE, 256, 96, 192, 1, FAKE, 96, 1 << 20));
    show("fwd_align", fwd(FAKE, 256, 128, 192, 1, ODD, 128, 1 << 20));
    show("fwd_ldo", fwd(FAKE, 256, 128, 192, 1, FAKE, 132, 1 << 20));
    show("fwd_ws", fwd(FAKE, 256, 128, 192, 1, FAKE, 128, 256 * 192 * 2 - 1));
    std::printf("fwd_ws_bytes %zu\n", dass_mlp_forward_workspace_bytes(256, 128, 192, DASS_BF16));
    // ---- compressed form and the sparse down projection
    auto cmp = [&](const void *W, int64_t rows, int64_t cols, int dt, int axis, void *V, int64_t ldv, void *M, int64_t ldm,
                   void *surplus) {
        return dass_compress_24(W, rows, cols, 64, (dass_dtype)dt, (dass_axis)axis, V, ldv, static_cast<uint8_t *>(M), ldm,
                                static_cast<long long *>(surplus), nullptr);
    };
    show("cmp_null", cmp(nullptr, 64, 64, 1, 1, FAKE2, 32, FAKE3, 8, nullptr));
    show("cmp_meta_null", cmp(FAKE, 64, 64, 1, 1, FAKE2, 32, nullptr, 8, nullptr));
    show("cmp_dtype", cmp(FAKE, 64, 64, 5, 1, FAKE2, 32, FAKE3, 8, nullptr));
    show("cmp_axis", cmp(FAKE, 64, 64, 1, 2, FAKE2, 32, FAKE3, 8, nullptr));
    show("cmp_cols", cmp(FAKE, 64, 60, 1, 1, FAKE2, 32, FAKE3, 8, nullptr));
    show("cmp_rows4", cmp(FAKE, 62, 64, 1, 0, FAKE2, 64, FAKE3, 32, nullptr));
    show("cmp_ldv", cmp(FAKE, 64, 64, 1, 1, FAKE2, 24, FAKE3, 8, nullptr));
    show("cmp_align", cmp(FAKE, 64, 64, 1, 1, ODD, 32, FAKE3, 8, nullptr));
    show("cmp_surplus_align", cmp(FAKE, 64, 64, 1, 1, FAKE2, 32, FAKE3, 8, ODD));
    show("cmp_overlap", cmp(FAKE, 64, 64, 1, 1, FAKE, 32, FAKE3, 8, nullptr));
    auto spd = [&](const void *Y, int64_t T, int64_t d, int64_t d_int, int dt, int64_t ldm, int64_t ldo) {
        return dass_down_proj_sparse24(Y, T, d_int, FAKE2, d_int / 2, static_cast<const uint8_t *>(FAKE3), ldm, d, d_int,
                                       (dass_dtype)dt, FAKE, ldo, nullptr);
    };
    show("spd_null", spd(nullptr, 256, 128, 192, 1, 24, 128));
    show("spd_dtype", spd(FAKE, 256, 128, 192, 0, 24, 128));
    show("spd_T0", spd(FAKE, 0, 128, 192, 1, 24, 128));
    show("spd_d8", spd(FAKE, 256, 100, 192, 1, 24, 128));
    show("spd_ldm", spd(FAKE, 256, 128, 192, 1, 20, 128));
    show("spd_ldm_align", spd(FAKE, 256, 128, 192, 1, 26, 128));
    show("spd_ldo", spd(FAKE, 256, 128, 192, 1, 24, 132));
    std::printf("version %d\n", dass_version());
    std::printf("unknown_status %s\n", dass_status_string((dass_status)99));
    std::printf("all ok\n");
    return 0;
}
