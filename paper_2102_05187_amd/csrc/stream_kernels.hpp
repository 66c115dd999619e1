// Launchers of the nonzero-tiled streaming kernels (definitions in kernels_rank1.hip, kernels_rankR.hip,
// kernels_mttkrp.hip; shared device code in stream_common.hpp).
//
// The leaf level's nonzeros are processed in tiles of kTile consecutive positions regardless of
// where segment (row / fiber / slice) boundaries fall, so a power-law head segment is spread
// over many workgroups.  Partial sums of segments cut by a tile boundary go through a small
// carry buffer in `scratch` and are completed by a fix-up kernel in a fixed order (no atomics,
// results are reproducible run to run).
#pragma once

#include <hip/hip_runtime.h>
#include <cstdint>

#include "kernels.hpp"
#include "tensor.hpp"

namespace comet {

bool   stream_supports_rank(int64_t R);
bool   stream_mttkrp_supports_rank(int64_t R);
bool   stream_supports_coo();
size_t stream_scratch_bytes(int64_t ntiles, int64_t R);

// out[row(s), :] = sum_{p in segment s} vals[p] * Dn[crd[p], :],  row(s) = rowmap ? rowmap[s] : s.
// Every segment of the level is written (empty ones with zeros).  dense_rows = number of rows of Dn.
// plain = true keeps rank-1 work on the per-tile kernel that gathers the vector through L1 (measurement
// baseline) instead of the kernel that stages it in LDS.
hipError_t stream_segreduce(const Schedule &sc, const int32_t *pos, const int32_t *crd, const double *vals,
                            const int32_t *rowmap, const double *Dn, int64_t dense_rows, int64_t R, double *out,
                            void *scratch, bool plain, hipStream_t st, Epilogue ep = Epilogue());

// Sorted COO [CN,S,S]: one output (i, j, value) per run of equal (c0, c1).
hipError_t stream_ttv_coo(const Schedule &sc, const int32_t *c0, const int32_t *c1, const int32_t *c2,
                          const double *vals, const double *v, int64_t dense_rows, int32_t *y0, int32_t *y1, double *yv,
                          void *scratch, bool plain, hipStream_t st);

// ---- heavy-row sweep of SpMM (kernels_heavy.hip) ---------------------------------------------------
// Builds the plan for a [*,CU] matrix level (pos over nseg segments, crd with coordinates < ncols); leaves
// plan.nunits = 0 when the rows of >= min_len nonzeros hold too small a share to matter.  Synchronises.
// rowmap (or null): result row of segment s, composed into the copy of the other rows (plan.light).
hipError_t heavy_plan_build(const int32_t *pos, int64_t nseg, const int32_t *crd, const double *vals, int64_t nnz,
                            int64_t ncols, const int32_t *rowmap, HeavyPlan &plan, hipStream_t st);
// The sweep exists for ranks 16, 32, 48 and 64, as long as the sums of a compute unit's units fit its LDS.
bool   heavy_supports(const HeavyPlan &plan, int64_t R);
size_t heavy_partial_bytes(const HeavyPlan &plan, int64_t R);
// out[row(h), :] = sum over heavy row h of vals * Dn[crd, :] for every heavy row (row(h) = rowmap ?
// rowmap[seg] : seg); `partial` holds heavy_partial_bytes(plan, R).
hipError_t heavy_spmm(const HeavyPlan &plan, const int32_t *rowmap, const double *Dn, int64_t R, double *out, void *partial,
                      hipStream_t st, Epilogue ep = Epilogue());

// ---- heavy-fiber sweep of TTM (kernels_heavy.hip) --------------------------------------------------
// Builds the plan for the leaf level of a [CU,CU,CU] tensor (pos over nseg fibers, crd with coordinates < ncols);
// leaves plan.nheavy = 0 when the operand rows do not fit a few LDS windows or the long fibers hold too small a
// share.  The plan also holds a copy of all other fibers as a [CU,CU] matrix (row = fiber).  Synchronises.
hipError_t fiber_plan_build(const int32_t *pos, int64_t nseg, const int32_t *crd, const double *vals, int64_t nnz,
                            int64_t ncols, FiberPlan &plan, hipStream_t st);
bool   fiber_supports(const FiberPlan &plan, int64_t R);          // ranks 16 and 32
size_t fiber_partial_bytes(const FiberPlan &plan, int64_t R);
// out[fiber, :] = sum over the fiber of vals * Dn[crd, :] for every heavy fiber (Dn has ncols rows of R);
// `partial` holds fiber_partial_bytes(plan, R).
hipError_t fiber_ttm(const FiberPlan &plan, const int32_t *crd, const double *vals, const double *Dn, int64_t ncols,
                     int64_t R, double *out, void *partial, hipStream_t st);

// Number of compute units of the current device (cached per device).
int current_device_cu_count();

// M[crd1[s], :] = sum_{f in slice s} B[crd2[f], :] * (sum_{p in fiber f} vals[p] * C[crd3[p], :]).
// M must have been cleared (or, with an epilogue, scaled by beta) for rows that have no stored slice.
// Every comment above reads "=" as "= alpha * (...) + beta * (old value)" when an epilogue is switched on.
hipError_t stream_mttkrp(const Schedule &sc, const int32_t *pos2, const int32_t *crd1, int64_t nslice,
                         const int32_t *pos3, const int32_t *crd2, const int32_t *crd3, const double *vals,
                         const double *B, const double *C, int64_t R, double *M, void *scratch, hipStream_t st,
                         Epilogue ep = Epilogue());

}  // namespace comet
