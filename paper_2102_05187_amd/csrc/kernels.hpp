// Launchers of the HIP kernels (host functions; definitions in the .hip files).
// All pointers are device pointers; every launcher only enqueues work on `st`.
#pragma once

#include <hip/hip_runtime.h>
#include <cstdint>

namespace comet {

// What a kernel does with a finished result element: off = store the value; on = store
// alpha * value + beta * (what the element held before).  The old element is not read when beta is 0,
// so it may hold anything then (NaN included), as in the BLAS convention.
struct Epilogue {
    double alpha = 1.0, beta = 0.0;
    int on = 0;
};
__device__ __forceinline__ double ep_apply(const Epilogue &ep, double v, const double *p) {
    if (!ep.on) return v;
    return ep.beta != 0.0 ? fma(ep.alpha, v, ep.beta * *p) : ep.alpha * v;
}
// What an element without any contribution becomes under the same rule.
__device__ __forceinline__ double ep_empty(const Epilogue &ep, const double *p) {
    return (ep.on && ep.beta != 0.0) ? ep.beta * *p : 0.0;
}

// ---- utilities (util.hip) -----------------------------------------------------------------------
hipError_t fill_zero_f64(double *p, int64_t n, hipStream_t st);
// p[i] = beta * p[i] (beta == 0: p[i] = 0 without reading it).
hipError_t scale_f64(double *p, int64_t n, double beta, hipStream_t st);
// out[r, :] = 0 for every row r of [0, nrows) that does not occur in the sorted, duplicate-free list idx[0..n).
// beta != 0: those rows are multiplied by beta instead.
hipError_t zero_unstored_rows(const int32_t *idx, int64_t n, int64_t nrows, int64_t R, double *out, hipStream_t st,
                              double beta = 0.0);

// Structure checks; each ORs a bit into *err (device int32, zeroed by the caller) on failure.
hipError_t check_pos(const int32_t *pos, int64_t n, int64_t last, int32_t *err, hipStream_t st);
hipError_t check_crd_range(const int32_t *crd, int64_t n, int64_t dim, int32_t *err, hipStream_t st);
hipError_t check_cu_sorted(const int32_t *pos, int64_t nseg, const int32_t *crd, int64_t n, int32_t *err,
                           hipStream_t st);
hipError_t check_coo_sorted(int order, const int32_t *c0, const int32_t *c1, const int32_t *c2, int64_t n,
                            int32_t *err, hipStream_t st);

// Schedule tables (see Schedule in tensor.hpp).
hipError_t build_seg_begin(const int32_t *pos, int64_t nseg, int64_t nnz, int tile, int64_t ntiles,
                           int32_t *seg_begin, hipStream_t st);
hipError_t build_parent_begin(const int32_t *parent_pos, int64_t nparent, const int32_t *seg_begin,
                              int64_t ntiles, int32_t *parent_begin, hipStream_t st);
hipError_t build_run_base(const int32_t *c0, const int32_t *c1, int64_t nnz, int tile, int64_t ntiles,
                          int32_t *run_base /* [ntiles+1] */, hipStream_t st);
hipError_t max_segment_length(const int32_t *pos, int64_t nseg, int32_t *out_max, hipStream_t st);
hipError_t count_empty_segments(const int32_t *pos, int64_t nseg, int32_t *out_count, hipStream_t st);
// Longest run of coordinates of [0, dim) that do not occur in the sorted list idx[0..n) (*out_max zeroed by the caller).
hipError_t max_coordinate_gap(const int32_t *idx, int64_t n, int64_t dim, int32_t *out_max, hipStream_t st);
hipError_t max_parent_span(const int32_t *parent_pos, int64_t nparent, const int32_t *leaf_pos, int32_t *out_max,
                           hipStream_t st);

// ---- simple family (kernels_simple.hip): one lane group / thread per output element -------------
// out[row(s), :] = sum_{p in [pos[s], pos[s+1])} vals[p] * Dn[crd[p], :]   for s in [0, nseg)
// row(s) = rowmap ? rowmap[s] : s.   R == 1 reads Dn as a vector.
hipError_t simple_segreduce(const int32_t *pos, const int32_t *crd, const double *vals, int64_t nseg,
                            int64_t nnz, const int32_t *rowmap, const double *Dn, int64_t R, double *out,
                            hipStream_t st, Epilogue ep = Epilogue());
// M[crd1[s], :] = sum_{f in slice s} B[crd2[f], :] * (sum_{p in fiber f} vals[p] * C[crd3[p], :])
hipError_t simple_mttkrp(const int32_t *pos2, const int32_t *crd1, int64_t nslice, const int32_t *pos3,
                         const int32_t *crd2, const int32_t *crd3, const double *vals, const double *B,
                         const double *C, int64_t R, double *M, hipStream_t st, Epilogue ep = Epilogue());
// Sorted COO [CN,S,S]: distinct (i,j) runs -> ycrd0/ycrd1/yvals (run_base from the schedule).
hipError_t simple_ttv_coo(const int32_t *c0, const int32_t *c1, const int32_t *c2, const double *vals,
                          int64_t nnz, int tile, int64_t ntiles, const int32_t *run_base, const double *v,
                          int32_t *ycrd0, int32_t *ycrd1, double *yvals, hipStream_t st);

// ---- mode reordering (reorder.hip) ------------------------------------------------------------
// Where the coordinates of nonzero p of the source tensor come from.
struct CoordSource {
    enum Kind { kCsr, kDcsr, kCoo, kCsf3 };
    int kind = kCoo;
    int order = 0;
    int64_t nnz = 0;
    const int32_t *pos[3] = {nullptr, nullptr, nullptr};
    int32_t npos[3] = {0, 0, 0};
    const int32_t *crd[3] = {nullptr, nullptr, nullptr};
};
// 64-bit sort key: new level l takes the coordinate of source level src_level[l], shifted left by
// shift[l] (shift of the last level is 0) and at most mask[l].
struct KeyLayout {
    int src_level[3] = {0, 1, 2};
    int shift[3] = {0, 0, 0};
    uint64_t mask[3] = {0, 0, 0};
};
// Output arrays of the all-compressed-unique storage (pos[0] = {0, #root} is written by the host).
struct CuLevels {
    int32_t *pos[3] = {nullptr, nullptr, nullptr};
    int32_t *crd[3] = {nullptr, nullptr, nullptr};
};
// keys[p] = packed coordinates of nonzero p.  When the three bit fields do not fit 64 bits (`root` non-null)
// the key holds the middle and last level only and the root level's coordinate goes to root[p].
hipError_t reorder_pack_keys(const CoordSource &src, const KeyLayout &lay, uint64_t *keys, uint32_t *root, hipStream_t st);
// Pieces of the two-pass sort for keys wider than 64 bits (stable radix sorts; temp == nullptr only sets
// *temp_bytes): order by (middle, last) carrying the nonzero's number, then by root carrying that order.
hipError_t reorder_iota(uint32_t *out, int64_t n, hipStream_t st);
hipError_t reorder_sort_lo(void *temp, size_t *temp_bytes, const uint64_t *keys_in, uint64_t *keys_out,
                           const uint32_t *idx_in, uint32_t *idx_out, int64_t n, int key_bits, hipStream_t st);
hipError_t reorder_sort_hi(void *temp, size_t *temp_bytes, const uint32_t *keys_in, uint32_t *keys_out,
                           const uint32_t *idx_in, uint32_t *idx_out, int64_t n, int key_bits, hipStream_t st);
hipError_t reorder_gather_u32(const uint32_t *src, const uint32_t *idx, uint32_t *out, int64_t n, hipStream_t st);
hipError_t reorder_gather_pairs(const uint64_t *keys, const double *vals, const uint32_t *idx, uint64_t *keys_out,
                                double *vals_out, int64_t n, hipStream_t st);
// Both follow the two-call convention: temp == nullptr only sets *temp_bytes.
hipError_t reorder_sort_pairs(void *temp, size_t *temp_bytes, const uint64_t *keys_in, uint64_t *keys_out,
                              const double *vals_in, double *vals_out, int64_t n, int key_bits, hipStream_t st);
hipError_t reorder_scan_flags(void *temp, size_t *temp_bytes, const uint64_t *flags, uint64_t *before, int64_t n,
                              hipStream_t st);
// flags: low half counts new (root, middle) prefixes (new rows for order 2), high half new root
// coordinates (order 3).  *err |= 1 if two nonzeros share all coordinates.
// `root` (sorted like keys) is null unless the keys are the wide form described at reorder_pack_keys.
hipError_t reorder_mark_heads(const uint64_t *keys, const uint32_t *root, int64_t n, const KeyLayout &lay, int order,
                              uint64_t *flags, int32_t *err, hipStream_t st);
// Sorted coordinate list out of the keys (crd[l][p] = field l), and the dense-root pos array of a CSR matrix
// out of its compressed rows (out has dim0 + 1 entries).
hipError_t reorder_unpack_keys(const uint64_t *keys, const uint32_t *root, int64_t n, const KeyLayout &lay, int order,
                               const CuLevels &out, hipStream_t st);
// out[f] = crd0[s] for the parent s of position f (pos1[s] <= f < pos1[s+1]), f in [0, nchild).
hipError_t expand_parent_coords(const int32_t *pos1, int64_t nparent, const int32_t *crd0, int64_t nchild, int32_t *out,
                                hipStream_t st);
hipError_t reorder_dense_pos(const int32_t *crd0, int64_t nroot, const int32_t *pos1, int64_t dim0, int64_t n,
                             int32_t *out, hipStream_t st);
hipError_t reorder_cut_levels(const uint64_t *keys, const uint32_t *root, const uint64_t *flags, const uint64_t *before,
                              int64_t n, const KeyLayout &lay, int order, const CuLevels &out, hipStream_t st);

}  // namespace comet
