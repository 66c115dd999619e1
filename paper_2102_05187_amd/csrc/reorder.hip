// Re-storing a tensor with its modes in another level order (all levels compressed-unique).
//
// The contractions walk the level tree from the root, so the contracted mode of TTV / TTM has to sit
// in the last level and the output mode of MTTKRP in the first (paper Section 8.2 defines TTV and TTM
// for the first mode; Section 4 fixes that level l stores one mode).  This file builds the storage
// for any mode order on the device: expand every nonzero to its coordinates, pack them into one
// 64-bit key in the new order, radix-sort (key, value) pairs, and cut the sorted list into the
// pos / crd arrays of the new levels.  None of it is on the timed path of an operation.
#include <cstring>

#include <rocprim/rocprim.hpp>

#include "kernels.hpp"

namespace comet {

namespace {

inline unsigned blocks_for(int64_t n, int per_block) {
    int64_t b = (n + per_block - 1) / per_block;
    return (unsigned)(b < 1 ? 1 : b);
}

// Largest s in [0, n) with pos[s] <= p, for a non-decreasing pos[0..n] with pos[0] <= p < pos[n].
__device__ inline int32_t owner_of(const int32_t *__restrict__ pos, int32_t n, int32_t p) {
    int32_t lo = 0, hi = n;              // invariant: pos[lo] <= p < pos[hi]
    while (hi - lo > 1) {
        int32_t mid = lo + ((hi - lo) >> 1);
        if (pos[mid] <= p) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ void __launch_bounds__(256) k_pack_keys(CoordSource src, KeyLayout lay, uint64_t *__restrict__ keys,
                                                   uint32_t *__restrict__ root) {
    int64_t p64 = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p64 >= src.nnz) return;
    int32_t p = (int32_t)p64;
    uint64_t c[3] = {0, 0, 0};
    switch (src.kind) {
    case CoordSource::kCsr:
        c[0] = (uint64_t)owner_of(src.pos[1], src.npos[1] - 1, p);
        c[1] = (uint64_t)src.crd[1][p];
        break;
    case CoordSource::kDcsr:
        c[0] = (uint64_t)src.crd[0][owner_of(src.pos[1], src.npos[1] - 1, p)];
        c[1] = (uint64_t)src.crd[1][p];
        break;
    case CoordSource::kCoo:
        for (int l = 0; l < src.order; ++l) c[l] = (uint64_t)src.crd[l][p];
        break;
    case CoordSource::kCsf3: {
        int32_t f = owner_of(src.pos[2], src.npos[2] - 1, p);
        int32_t s = owner_of(src.pos[1], src.npos[1] - 1, f);
        c[0] = (uint64_t)src.crd[0][s];
        c[1] = (uint64_t)src.crd[1][f];
        c[2] = (uint64_t)src.crd[2][p];
        break;
    }
    }
    uint64_t key = 0;
    for (int l = root ? 1 : 0; l < src.order; ++l) key |= c[lay.src_level[l]] << lay.shift[l];
    keys[p] = key;
    if (root) root[p] = (uint32_t)c[lay.src_level[0]];
}

// Coordinate of the root level of sorted nonzero p: a field of the key, or (wide keys) a separate array.
__device__ __forceinline__ uint64_t root_of(const uint64_t *__restrict__ keys, const uint32_t *__restrict__ root,
                                            int64_t p, int shift0) {
    return root ? (uint64_t)root[p] : keys[p] >> shift0;
}

__global__ void __launch_bounds__(256) k_iota(uint32_t *__restrict__ out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = (uint32_t)i;
}
__global__ void __launch_bounds__(256) k_gather_u32(const uint32_t *__restrict__ src, const uint32_t *__restrict__ idx,
                                                    uint32_t *__restrict__ out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = src[idx[i]];
}
__global__ void __launch_bounds__(256) k_gather_pairs(const uint64_t *__restrict__ keys, const double *__restrict__ vals,
                                                      const uint32_t *__restrict__ idx, uint64_t *__restrict__ keys_out,
                                                      double *__restrict__ vals_out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) { const uint32_t s = idx[i]; keys_out[i] = keys[s]; vals_out[i] = vals[s]; }
}

// flags[p] = (first nonzero of a new root coordinate ? 1 << 32 : 0) | (first nonzero of a new
// (root, middle) prefix ? 1 : 0); for order 2 only the low half is used (new row).  Equal
// neighbouring keys mean one coordinate stored twice: *err is set.
__global__ void __launch_bounds__(256) k_mark_heads(const uint64_t *__restrict__ keys, const uint32_t *__restrict__ rootc,
                                                    int64_t n, KeyLayout lay, int order, uint64_t *__restrict__ flags,
                                                    int32_t *err) {
    int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= n) return;
    uint64_t k = keys[p];
    uint64_t f;
    if (p == 0) {
        f = order == 3 ? ((uint64_t(1) << 32) | 1u) : 1u;
    } else {
        uint64_t q = keys[p - 1];
        const bool root = root_of(keys, rootc, p, lay.shift[0]) != root_of(keys, rootc, p - 1, lay.shift[0]);
        if (q == k && !root) atomicOr(err, 1);
        if (order == 3) {
            const bool mid = root || (k >> lay.shift[1]) != (q >> lay.shift[1]);
            f = (root ? (uint64_t(1) << 32) : 0) | (mid ? 1u : 0u);
        } else {
            f = root ? 1u : 0u;
        }
    }
    flags[p] = f;
}

// `before[p]` = exclusive prefix sum of flags.  Writes the new levels (see CuLevels).
__global__ void __launch_bounds__(256) k_cut_levels(const uint64_t *__restrict__ keys, const uint32_t *__restrict__ rootc,
                                                    const uint64_t *__restrict__ flags,
                                                    const uint64_t *__restrict__ before, int64_t n, KeyLayout lay,
                                                    int order, CuLevels out) {
    int64_t p64 = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p64 >= n) return;
    const int32_t p = (int32_t)p64;
    const uint64_t k = keys[p], f = flags[p], b = before[p];
    const int32_t lo = (int32_t)(b & 0xffffffffu), hi = (int32_t)(b >> 32);
    const int leaf = order - 1;
    out.crd[leaf][p] = (int32_t)(k & lay.mask[leaf]);
    if (order == 3) {
        if (f & 1u) {
            out.crd[1][lo] = (int32_t)((k >> lay.shift[1]) & lay.mask[1]);
            out.pos[2][lo] = p;
        }
        if (f >> 32) {
            out.crd[0][hi] = (int32_t)root_of(keys, rootc, p64, lay.shift[0]);
            out.pos[1][hi] = lo;
        }
        if (p64 == n - 1) {
            int32_t nmid = lo + (int32_t)(f & 1u), nroot = hi + (int32_t)(f >> 32);
            out.pos[2][nmid] = (int32_t)n;
            out.pos[1][nroot] = nmid;
        }
    } else {
        if (f & 1u) {
            out.crd[0][lo] = (int32_t)root_of(keys, rootc, p64, lay.shift[0]);
            out.pos[1][lo] = p;
        }
        if (p64 == n - 1) out.pos[1][lo + (int32_t)(f & 1u)] = (int32_t)n;
    }
}

// Coordinate-list output: level l of nonzero p is field l of its key.
__global__ void __launch_bounds__(256) k_unpack_keys(const uint64_t *__restrict__ keys, const uint32_t *__restrict__ rootc,
                                                     int64_t n, KeyLayout lay, int order, CuLevels out) {
    int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= n) return;
    const uint64_t k = keys[p];
    out.crd[0][p] = (int32_t)root_of(keys, rootc, p, lay.shift[0]);
    for (int l = 1; l < order; ++l) out.crd[l][p] = (int32_t)((k >> lay.shift[l]) & lay.mask[l]);
}

// Dense root level: pos[r] = number of nonzeros in rows < r, from the compressed rows (sorted row
// coordinates crd0[0..nroot) with first positions pos1[0..nroot]).
__global__ void __launch_bounds__(256) k_dense_pos(const int32_t *__restrict__ crd0, int64_t nroot,
                                                   const int32_t *__restrict__ pos1, int64_t dim0, int64_t n,
                                                   int32_t *__restrict__ out) {
    int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r > dim0) return;
    int64_t lo = 0, hi = nroot;                  // first stored row with coordinate >= r
    while (lo < hi) {
        int64_t mid = lo + ((hi - lo) >> 1);
        if (crd0[mid] < r) lo = mid + 1; else hi = mid;
    }
    out[r] = lo < nroot ? pos1[lo] : (int32_t)n;
}

__global__ void __launch_bounds__(256) k_expand_parent(const int32_t *__restrict__ pos1, int32_t nparent,
                                                       const int32_t *__restrict__ crd0, int64_t nchild,
                                                       int32_t *__restrict__ out) {
    int64_t f = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (f < nchild) out[f] = crd0[owner_of(pos1, nparent, (int32_t)f)];
}

}  // namespace

hipError_t expand_parent_coords(const int32_t *pos1, int64_t nparent, const int32_t *crd0, int64_t nchild, int32_t *out,
                                hipStream_t st) {
    if (nchild <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_expand_parent, dim3(blocks_for(nchild, 256)), dim3(256), 0, st, pos1, (int32_t)nparent, crd0, nchild, out);
    return hipGetLastError();
}

hipError_t reorder_unpack_keys(const uint64_t *keys, const uint32_t *root, int64_t n, const KeyLayout &lay, int order,
                               const CuLevels &out, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_unpack_keys, dim3(blocks_for(n, 256)), dim3(256), 0, st, keys, root, n, lay, order, out);
    return hipGetLastError();
}

hipError_t reorder_dense_pos(const int32_t *crd0, int64_t nroot, const int32_t *pos1, int64_t dim0, int64_t n,
                             int32_t *out, hipStream_t st) {
    hipLaunchKernelGGL(k_dense_pos, dim3(blocks_for(dim0 + 1, 256)), dim3(256), 0, st, crd0, nroot, pos1, dim0, n, out);
    return hipGetLastError();
}

hipError_t reorder_pack_keys(const CoordSource &src, const KeyLayout &lay, uint64_t *keys, uint32_t *root, hipStream_t st) {
    if (src.nnz <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_pack_keys, dim3(blocks_for(src.nnz, 256)), dim3(256), 0, st, src, lay, keys, root);
    return hipGetLastError();
}

hipError_t reorder_iota(uint32_t *out, int64_t n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_iota, dim3(blocks_for(n, 256)), dim3(256), 0, st, out, n);
    return hipGetLastError();
}

hipError_t reorder_sort_lo(void *temp, size_t *temp_bytes, const uint64_t *keys_in, uint64_t *keys_out,
                           const uint32_t *idx_in, uint32_t *idx_out, int64_t n, int key_bits, hipStream_t st) {
    return rocprim::radix_sort_pairs(temp, *temp_bytes, keys_in, keys_out, idx_in, idx_out, (size_t)n, 0u,
                                     (unsigned)key_bits, st);
}

hipError_t reorder_sort_hi(void *temp, size_t *temp_bytes, const uint32_t *keys_in, uint32_t *keys_out,
                           const uint32_t *idx_in, uint32_t *idx_out, int64_t n, int key_bits, hipStream_t st) {
    return rocprim::radix_sort_pairs(temp, *temp_bytes, keys_in, keys_out, idx_in, idx_out, (size_t)n, 0u,
                                     (unsigned)key_bits, st);
}

hipError_t reorder_gather_u32(const uint32_t *src, const uint32_t *idx, uint32_t *out, int64_t n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_gather_u32, dim3(blocks_for(n, 256)), dim3(256), 0, st, src, idx, out, n);
    return hipGetLastError();
}

hipError_t reorder_gather_pairs(const uint64_t *keys, const double *vals, const uint32_t *idx, uint64_t *keys_out,
                                double *vals_out, int64_t n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_gather_pairs, dim3(blocks_for(n, 256)), dim3(256), 0, st, keys, vals, idx, keys_out, vals_out, n);
    return hipGetLastError();
}

hipError_t reorder_sort_pairs(void *temp, size_t *temp_bytes, const uint64_t *keys_in, uint64_t *keys_out,
                              const double *vals_in, double *vals_out, int64_t n, int key_bits, hipStream_t st) {
    return rocprim::radix_sort_pairs(temp, *temp_bytes, keys_in, keys_out, vals_in, vals_out, (size_t)n, 0u,
                                     (unsigned)key_bits, st);
}

hipError_t reorder_mark_heads(const uint64_t *keys, const uint32_t *root, int64_t n, const KeyLayout &lay, int order,
                              uint64_t *flags, int32_t *err, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_mark_heads, dim3(blocks_for(n, 256)), dim3(256), 0, st, keys, root, n, lay, order, flags, err);
    return hipGetLastError();
}

hipError_t reorder_scan_flags(void *temp, size_t *temp_bytes, const uint64_t *flags, uint64_t *before, int64_t n,
                              hipStream_t st) {
    return rocprim::exclusive_scan(temp, *temp_bytes, flags, before, uint64_t(0), (size_t)n,
                                   rocprim::plus<uint64_t>(), st);
}

hipError_t reorder_cut_levels(const uint64_t *keys, const uint32_t *root, const uint64_t *flags, const uint64_t *before,
                              int64_t n, const KeyLayout &lay, int order, const CuLevels &out, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_cut_levels, dim3(blocks_for(n, 256)), dim3(256), 0, st, keys, root, flags, before, n, lay, order,
                       out);
    return hipGetLastError();
}

}  // namespace comet
