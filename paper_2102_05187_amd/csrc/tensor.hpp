// Level-format tensor descriptor (host side) shared by the API and the kernel launchers.
//
// A tensor is `order` levels, each tagged D / CU / CN / S and carrying int32 pos / crd arrays,
// plus one fp64 value array (paper Section 4 and Section 6.1 "Sparse Tensor Data Type").  The
// arrays live in device memory; the descriptor keeps them behind reference-counted holders so a
// TTV / TTM result can share the uncontracted levels of its input without copying them.
#pragma once

#include <hip/hip_runtime.h>
#include <cstdint>
#include <memory>
#include <vector>

#include "../../include/comet.h"

namespace comet {

// One device array; frees its memory on destruction only if the library allocated it.
struct DevArray {
    void  *ptr   = nullptr;
    size_t bytes = 0;
    bool   owned = false;
    DevArray() = default;
    DevArray(void *p, size_t b, bool o) : ptr(p), bytes(b), owned(o) {}
    DevArray(const DevArray &) = delete;
    DevArray &operator=(const DevArray &) = delete;
    ~DevArray() { if (owned && ptr) (void)hipFree(ptr); }
};
using DevRef = std::shared_ptr<DevArray>;

inline DevRef borrow(const void *p, size_t bytes) {
    return std::make_shared<DevArray>(const_cast<void *>(p), bytes, false);
}
// Allocates `bytes` of device memory (at least 16 so that empty arrays still have an address).
inline DevRef dev_alloc(size_t bytes) {
    void *p = nullptr;
    if (hipMalloc(&p, bytes < 16 ? 16 : bytes) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    return std::make_shared<DevArray>(p, bytes, true);
}

enum class Format { CSR, DCSR, COO2, COO3, CSF3, CSF3_DENSE_LEAF, COO3_DENSE_LEAF, OTHER };

// Items per tile of the nonzero-tiled kernels (a multiple of every per-wave chunk they use).
constexpr int kTile = 4096;
// Items per chunk of the wavefront-per-chunk kernel (one wavefront's share of a tile).
constexpr int kChunk = 1024;

// The segments (rows / fibers) of a compressed level that a sweep does NOT take, copied out as a [CU,CU] matrix
// of their own: row r of the copy holds the nonzeros of one such segment and stands for result row rows[r].
// The nonzero-tiled kernel then walks them without the long segments in between -- skipping those inside the
// original arrays saves little: the lane groups of a wavefront sit 128 items apart, a wavefront step is free
// only where all of them skip, and the per-tile work stays.
struct LightCopy {
    int64_t nrows = 0, nnz = 0;
    DevRef  root;         // int32 [2]: {0, nrows}
    DevRef  rows;         // int32 [nrows]: result row of row r of the copy, increasing
    DevRef  pos;          // int32 [nrows + 1]
    DevRef  crd;          // int32 [nnz]
    DevRef  vals;         // double [nnz]
    size_t bytes() const { return (size_t)nnz * 12 + (size_t)nrows * 8; }
};

// Plan of the heavy-row sweep of SpMM (kernels_heavy.hip), built once at creation for matrices whose long
// rows hold a large share of the nonzeros.  Rows of at least `min_len` nonzeros are "heavy"; each is cut
// into units of roughly equal length, every lane group of the sweep owns `nu` units, and the nonzeros of
// the heavy rows are laid out again as one stream per wavefront in the order the sweep takes them (window
// by window, unit by unit; 16 bytes per stream item, padding included) -- a re-ordered copy of a part of the
// tensor, kept because the order is what makes the cache reuse work.
struct HeavyPlan {
    int64_t nheavy = 0, nunits = 0, heavy_nnz = 0, stream_items = 0;
    int32_t min_len = 0, window = 0, nwin = 0, nu = 0;
    DevRef  units;        // int4 [nunits], longest unit first: {heavy row h, piece q, pieces of the row, row-major unit number}
    DevRef  unit_begin;   // int32 [nheavy + 1]: units of heavy row h (row-major numbers)
    DevRef  hseg;         // int32 [nheavy]: segment (row position) of heavy row h, longest rows first
    DevRef  scrd, scode, sval;   // the streams: column, item code (-1 plain, -2 padding, k >= 0: ends unit slot k's piece), value
    DevRef  block_start;  // int32 [wavefronts + 1]: first super-block (8 groups x 32 positions) of each wavefront's stream
    DevRef  wend;         // int32 [wavefronts][windows per range + 1]: first position of each window in the stream
    LightCopy light;      // all other rows
};

// Plan of the heavy-fiber sweep of TTM (kernels_heavy.hip), built once at creation for order-3 tensors whose
// last mode is small enough for its dense operand to be cut into a few LDS-sized windows of rows and whose long
// fibers (at least `min_len` nonzeros) hold a large share of the nonzeros.  Fibers are sorted by coordinate, so
// the nonzeros of a fiber that fall into one window are consecutive: the plan only holds where they start.
// Two window sizes are kept (index 0: ranks up to 16, index 1: ranks up to 32) so that a window of operand rows
// fills the same 128 KB of LDS for both.
struct FiberPlan {
    int64_t nheavy = 0, heavy_nnz = 0;
    int32_t min_len = 0;
    int32_t window[2] = {0, 0}, nwin[2] = {0, 0};
    DevRef  hseg;         // int32 [nheavy]: leaf segment (fiber) of heavy fiber h, longest fibers first
    DevRef  wstart[2];    // int32 [nheavy][nwin + 1]: first position of fiber h with coordinate >= w * window
    LightCopy light;      // all other fibers (row = fiber)
};

// Per-tensor schedule for the nonzero-tiled kernels, built once at creation.
//   The leaf level's nonzeros are cut into tiles of kTile consecutive positions; seg_begin[t] is
//   the segment (row / fiber) that contains the first nonzero of tile t (seg_begin[0] = 0 and
//   seg_begin[ntiles] = nseg, so leading and trailing empty segments belong to the first and
//   last tile).  For CSF, slice_begin[t] is the slice that contains fiber seg_begin[t].
//   For sorted COO, run_base[t] counts the distinct (i,j) runs that start before tile t.
struct Schedule {
    int64_t nnz = 0, nseg = 0, ntiles = 0;
    DevRef  seg_begin;     // int32 [ntiles + 1]
    DevRef  slice_begin;   // int32 [ntiles + 1]   (CSF3 only)
    DevRef  run_base;      // int32 [ntiles + 1]   (COO3 only)
    int64_t nruns = 0;     // COO3: number of distinct (i,j) pairs
    DevRef  chunk_seg_begin;   // int32 [nchunks + 1]: seg_begin at kChunk granularity
    DevRef  chunk_run_base;    // int32 [nchunks + 1]: run_base at kChunk granularity (COO3 only)
    int64_t nchunks = 0;
    int64_t empty_segments = -1;  // leaf segments without a nonzero (-1 = unknown)
    int64_t max_seg_len = 0;      // longest leaf segment, in nonzeros (0 = unknown)
    int64_t max_parent_len = 0;   // CSF3: most nonzeros under one slice (0 = unknown)
    int64_t max_root_gap = -1;    // compressed root level: longest run of absent root coordinates (-1 = unknown)
    HeavyPlan heavy;              // matrices only; nunits = 0 when the sweep does not apply
    FiberPlan fibers;             // CSF3 only; nheavy = 0 when the sweep does not apply
};

}  // namespace comet

struct comet_tensor {
    int32_t order = 0;
    int64_t dims[COMET_MAX_ORDER] = {0, 0, 0, 0};
    int32_t levels[COMET_MAX_ORDER] = {0, 0, 0, 0};
    int32_t mode_of_level[COMET_MAX_ORDER] = {0, 1, 2, 3};   // tensor mode stored at each level
    comet::DevRef pos[COMET_MAX_ORDER], crd[COMET_MAX_ORDER], vals;
    int64_t pos_len[COMET_MAX_ORDER] = {0, 0, 0, 0};
    int64_t crd_len[COMET_MAX_ORDER] = {0, 0, 0, 0};
    int64_t nvals = 0;
    comet::Format fmt = comet::Format::OTHER;
    comet::Schedule sched;
    int variant = 0;
    bool lean = false;     // created with COMET_LEAN: no sweep plans, no copies

    // Scratch owned by the handle (carry buffers of the tiled kernels and the partial sums of the heavy-row
    // sweep).  It only ever grows: when an operation needs more than there is, a larger buffer is allocated
    // and the old one is kept until the handle is destroyed, so work that was enqueued (or captured into a
    // HIP graph) with the old address never sees freed memory.  `mutable`: operations take the handle as
    // const and still manage this cache (one operation per handle at a time, see comet.h).
    mutable comet::DevRef scratch;
    mutable size_t scratch_bytes = 0;
    mutable std::vector<comet::DevRef> retired_scratch;
    // streams the handle's operations were enqueued on (a few are remembered; destroy waits for them)
    mutable void *used_streams[4] = {nullptr, nullptr, nullptr, nullptr};
    mutable int  n_used_streams = 0;      // > 4: too many to remember, destroy waits for the whole device
    mutable bool used_null_stream = false;

    // a sorted coordinate list keeps a compressed ([CU,CU,CU]) copy of itself for the operations whose
    // kernels need the fiber / slice structure (TTM, MTTKRP); built on their first use
    mutable std::unique_ptr<comet_tensor> shadow;
    // [CU,CU,CU] with a heavy-fiber plan: the short fibers as a matrix handle over the plan's copy (see FiberPlan)
    std::unique_ptr<comet_tensor> light;

    // results of TTV / TTM remember what produced them so the handle can be reused
    const comet_tensor *result_of = nullptr;
    int     result_kind = 0;   // 1 = TTV, 2 = TTM
    int64_t result_R = 0;

    const int32_t *pos_i(int l) const { return pos[l] ? static_cast<const int32_t *>(pos[l]->ptr) : nullptr; }
    const int32_t *crd_i(int l) const { return crd[l] ? static_cast<const int32_t *>(crd[l]->ptr) : nullptr; }
    const double  *vals_d() const { return vals ? static_cast<const double *>(vals->ptr) : nullptr; }
};
