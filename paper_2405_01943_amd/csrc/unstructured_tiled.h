// Unstructured selection by streaming passes: column lines over 64-column tiles
// (unstructured_tiled.hip), row lines by workgroups that own whole rows (unstructured_rows.hip);
// called from the entry points in unstructured.hip.
#pragma once

#include "dass_internal.h"

namespace dass {

// Where the passes keep their intermediate results, as byte offsets into one region of the
// caller's workspace, and the launch shape.  fits = false: the matrix does not take this path.
struct TiledPlan {
    bool fits;
    int slabs;           // row slabs a column group is cut into (one workgroup each)
    int64_t slab_rows;   // rows per slab
    int64_t groups;      // groups of 64 columns
    size_t off_fs, off_win, off_part, off_sel, off_cnt, off_list;
    size_t bytes;        // size of the region
};

// Column lines of W [rows, cols] with the factor varying along the line, exponent 0.5 or 1.
// mask_out: NULL, or where the keep bits go; a mask that is not made of whole aligned 32-bit words
// does not take this path (its bits are corrected with 32-bit atomics).
TiledPlan plan_tiled(int64_t rows, int64_t cols, int64_t ld, int dt, const uint8_t *mask_out = nullptr);

// Enqueue the passes.  `flag` (one device word, 4-byte aligned, outside `region`) is cleared by
// the first kernel and set by any later one that meets a case the passes do not decide (a factor
// or product outside the range of the two-term f32 score, a threshold outside the sampled window,
// more equal leading terms at the threshold than a list holds).  When it is set, W has not been
// written: the caller's next launches, gated on the flag, redo the whole matrix.
dass_status launch_tiled(const char *fn, const TiledPlan &p, void *W, int64_t rows, int64_t cols, int64_t ld, int dt,
                         const float *norms, int fmode, uint32_t n_keep, uint8_t *mask_out, uint32_t *flag,
                         void *region, hipStream_t stream);

// ---- row lines (unstructured_rows.hip): one launch, a workgroup owns kRowlinesBlock whole rows ----
constexpr int kRowlinesBlock = 8;

struct RowlinesPlan {
    bool fits;
    int64_t blocks;      // workgroups = blocks of kRowlinesBlock rows
    int chunks;          // the columns' factors are staged in LDS in so many chunks ...
    int64_t chunk_cols;  // ... of so many columns (a multiple of 8; the last chunk may be shorter)
    size_t smem;         // dynamic LDS of the kernel
    size_t todo_bytes;   // one word per block in the caller's workspace
};

// Row lines of W [rows, cols] with the factor varying along the line, exponent 0.5 or 1.
RowlinesPlan plan_rowlines(int64_t rows, int64_t cols, int64_t ld, int dt, const uint8_t *mask_out = nullptr);

// Enqueue the kernel.  todo[b] is written for every block b of kRowlinesBlock rows: 0 if the
// block's rows are done, 1 if they were left for the caller's next launch, gated per block.
dass_status launch_rowlines(const char *fn, const RowlinesPlan &p, void *W, int64_t rows, int64_t cols, int64_t ld, int dt,
                            const float *norms, int fmode, uint32_t n_keep, uint8_t *mask_out, uint32_t *todo,
                            hipStream_t stream);

}  // namespace dass
