// Fill, structure-check and schedule-building kernels (none of them is on the timed path except
// fill_zero_f64, which clears dense results whose rows may have no stored segment).
#include "kernels.hpp"

namespace comet {

static inline unsigned blocks_for(int64_t n, int per_block) {
    int64_t b = (n + per_block - 1) / per_block;
    return (unsigned)(b < 1 ? 1 : b);
}

// ---------------------------------------------------------------------------------------------
// fills
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_fill_zero_f64(double *__restrict__ p, int64_t n) {
    // two doubles per lane per step: 16-byte stores, consecutive lanes on consecutive 16 bytes
    int64_t n2 = n >> 1;
    double2 *p2 = reinterpret_cast<double2 *>(p);
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n2; i += stride)
        p2[i] = make_double2(0.0, 0.0);
    if ((n & 1) && blockIdx.x == 0 && threadIdx.x == 0) p[n - 1] = 0.0;
}

hipError_t fill_zero_f64(double *p, int64_t n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    int64_t want = (n / 2 + 255) / 256;
    unsigned grid = (unsigned)(want < 1 ? 1 : (want > 8192 ? 8192 : want));
    hipLaunchKernelGGL(k_fill_zero_f64, dim3(grid), dim3(256), 0, st, p, n);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256) k_scale_f64(double *__restrict__ p, int64_t n, double beta) {
    int64_t n2 = n >> 1;
    double2 *p2 = reinterpret_cast<double2 *>(p);
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n2; i += stride) {
        const double2 v = p2[i];
        p2[i] = make_double2(beta * v.x, beta * v.y);
    }
    if ((n & 1) && blockIdx.x == 0 && threadIdx.x == 0) p[n - 1] = beta * p[n - 1];
}

hipError_t scale_f64(double *p, int64_t n, double beta, hipStream_t st) {
    if (n <= 0 || beta == 1.0) return hipSuccess;
    if (beta == 0.0) return fill_zero_f64(p, n, st);
    int64_t want = (n / 2 + 255) / 256;
    unsigned grid = (unsigned)(want < 1 ? 1 : (want > 8192 ? 8192 : want));
    hipLaunchKernelGGL(k_scale_f64, dim3(grid), dim3(256), 0, st, p, n, beta);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// structure checks (bits: 1 pos, 2 range, 4 order inside a CU segment, 8 COO order)
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_check_pos(const int32_t *__restrict__ pos, int64_t n, int64_t last,
                                                   int32_t *err) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    bool bad = false;
    int32_t v = pos[i];
    if (i == 0 && v != 0) bad = true;
    if (i == n - 1 && (int64_t)v != last) bad = true;
    if (i + 1 < n && pos[i + 1] < v) bad = true;
    if (v < 0) bad = true;
    if (bad) atomicOr(err, 1);
}

hipError_t check_pos(const int32_t *pos, int64_t n, int64_t last, int32_t *err, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_check_pos, dim3(blocks_for(n, 256)), dim3(256), 0, st, pos, n, last, err);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256) k_check_range(const int32_t *__restrict__ crd, int64_t n, int64_t dim,
                                                     int32_t *err) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    int32_t c = crd[i];
    if (c < 0 || (int64_t)c >= dim) atomicOr(err, 2);
}

hipError_t check_crd_range(const int32_t *crd, int64_t n, int64_t dim, int32_t *err, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_check_range, dim3(blocks_for(n, 256)), dim3(256), 0, st, crd, n, dim, err);
    return hipGetLastError();
}

// index of the last entry of pos[0..n) that is <= x   (pos non-decreasing, pos[0] <= x)
__device__ inline int64_t last_le(const int32_t *__restrict__ pos, int64_t n, int64_t x) {
    int64_t lo = 0, hi = n;           // invariant: pos[lo] <= x, (hi == n or pos[hi] > x)
    while (hi - lo > 1) {
        int64_t mid = lo + ((hi - lo) >> 1);
        if ((int64_t)pos[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// Coordinates must increase strictly inside a segment.  Position p may only fail to exceed its
// predecessor when p is the first position of a segment, i.e. when some pos entry equals p.
__global__ void __launch_bounds__(256) k_check_cu_sorted(const int32_t *__restrict__ pos, int64_t nseg,
                                                         const int32_t *__restrict__ crd, int64_t n,
                                                         int32_t *err) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x + 1;
    if (p >= n) return;
    if (crd[p] > crd[p - 1]) return;
    int64_t s = last_le(pos, nseg + 1, p);
    if ((int64_t)pos[s] != p) atomicOr(err, 4);
}

hipError_t check_cu_sorted(const int32_t *pos, int64_t nseg, const int32_t *crd, int64_t n, int32_t *err,
                           hipStream_t st) {
    if (n <= 1) return hipSuccess;
    hipLaunchKernelGGL(k_check_cu_sorted, dim3(blocks_for(n - 1, 256)), dim3(256), 0, st, pos, nseg, crd, n, err);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256) k_check_coo_sorted(int order, const int32_t *__restrict__ c0,
                                                          const int32_t *__restrict__ c1,
                                                          const int32_t *__restrict__ c2, int64_t n,
                                                          int32_t *err) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x + 1;
    if (p >= n) return;
    bool less;    // tuple(p-1) < tuple(p) lexicographically
    if (c0[p - 1] != c0[p]) less = c0[p - 1] < c0[p];
    else if (c1[p - 1] != c1[p]) less = c1[p - 1] < c1[p];
    else if (order > 2) less = c2[p - 1] < c2[p];
    else less = false;
    if (!less) atomicOr(err, 8);
}

hipError_t check_coo_sorted(int order, const int32_t *c0, const int32_t *c1, const int32_t *c2, int64_t n,
                            int32_t *err, hipStream_t st) {
    if (n <= 1) return hipSuccess;
    hipLaunchKernelGGL(k_check_coo_sorted, dim3(blocks_for(n - 1, 256)), dim3(256), 0, st, order, c0, c1, c2, n, err);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// schedule tables
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_build_seg_begin(const int32_t *__restrict__ pos, int64_t nseg,
                                                         int64_t nnz, int tile, int64_t ntiles,
                                                         int32_t *__restrict__ seg_begin) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t > ntiles) return;
    int64_t s;
    if (t == 0) s = 0;
    else if (t == ntiles) s = nseg;
    else s = last_le(pos, nseg + 1, t * (int64_t)tile);   // the non-empty segment holding that nonzero
    seg_begin[t] = (int32_t)s;
}

hipError_t build_seg_begin(const int32_t *pos, int64_t nseg, int64_t nnz, int tile, int64_t ntiles,
                           int32_t *seg_begin, hipStream_t st) {
    hipLaunchKernelGGL(k_build_seg_begin, dim3(blocks_for(ntiles + 1, 256)), dim3(256), 0, st, pos, nseg, nnz,
                       tile, ntiles, seg_begin);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256) k_build_parent_begin(const int32_t *__restrict__ ppos, int64_t nparent,
                                                            const int32_t *__restrict__ seg_begin,
                                                            int64_t ntiles, int32_t *__restrict__ out) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t > ntiles) return;
    int64_t s;
    if (t == 0) s = 0;
    else if (t == ntiles) s = nparent;
    else s = last_le(ppos, nparent + 1, seg_begin[t]);
    out[t] = (int32_t)s;
}

hipError_t build_parent_begin(const int32_t *parent_pos, int64_t nparent, const int32_t *seg_begin,
                              int64_t ntiles, int32_t *parent_begin, hipStream_t st) {
    hipLaunchKernelGGL(k_build_parent_begin, dim3(blocks_for(ntiles + 1, 256)), dim3(256), 0, st, parent_pos,
                       nparent, seg_begin, ntiles, parent_begin);
    return hipGetLastError();
}

// run_base[t + 1] = number of positions p in tile t that start a new (c0, c1) run
__global__ void __launch_bounds__(256) k_count_runs(const int32_t *__restrict__ c0, const int32_t *__restrict__ c1,
                                                    int64_t nnz, int tile, int32_t *__restrict__ run_base) {
    __shared__ int cnt;
    if (threadIdx.x == 0) cnt = 0;
    __syncthreads();
    int64_t b = (int64_t)blockIdx.x * tile;
    int64_t e = b + tile < nnz ? b + tile : nnz;
    int local = 0;
    for (int64_t p = b + threadIdx.x; p < e; p += blockDim.x)
        local += (p == 0 || c0[p] != c0[p - 1] || c1[p] != c1[p - 1]) ? 1 : 0;
    atomicAdd(&cnt, local);
    __syncthreads();
    if (threadIdx.x == 0) run_base[blockIdx.x + 1] = cnt;
}

// in-place inclusive scan of a[1..n] with a[0] = 0 (one workgroup; n is a few ten thousand at most)
__global__ void __launch_bounds__(1024) k_scan_small(int32_t *__restrict__ a, int64_t n) {
    __shared__ int32_t part[1024];
    int64_t per = (n + 1023) / 1024;
    int64_t lo = 1 + threadIdx.x * per, hi = lo + per;
    if (hi > n + 1) hi = n + 1;
    int32_t s = 0;
    for (int64_t i = lo; i < hi; ++i) s += a[i];
    part[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t run = 0;
        for (int i = 0; i < 1024; ++i) { int32_t v = part[i]; part[i] = run; run += v; }
        a[0] = 0;
    }
    __syncthreads();
    int32_t run = part[threadIdx.x];
    for (int64_t i = lo; i < hi; ++i) { run += a[i]; a[i] = run; }
}

hipError_t build_run_base(const int32_t *c0, const int32_t *c1, int64_t nnz, int tile, int64_t ntiles,
                          int32_t *run_base, hipStream_t st) {
    if (ntiles > 0)
        hipLaunchKernelGGL(k_count_runs, dim3((unsigned)ntiles), dim3(256), 0, st, c0, c1, nnz, tile, run_base);
    hipLaunchKernelGGL(k_scan_small, dim3(1), dim3(1024), 0, st, run_base, ntiles);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256) k_max_seg_len(const int32_t *__restrict__ pos, int64_t nseg,
                                                     int32_t *__restrict__ out) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int32_t m = 0;
    for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s < nseg; s += stride) {
        int32_t l = pos[s + 1] - pos[s];
        m = l > m ? l : m;
    }
    if (m > 0) atomicMax(out, m);
}

hipError_t max_segment_length(const int32_t *pos, int64_t nseg, int32_t *out_max, hipStream_t st) {
    if (nseg <= 0) return hipSuccess;
    int64_t want = (nseg + 255) / 256;
    unsigned grid = (unsigned)(want > 2048 ? 2048 : want);
    hipLaunchKernelGGL(k_max_seg_len, dim3(grid), dim3(256), 0, st, pos, nseg, out_max);
    return hipGetLastError();
}

// longest run of coordinates absent from the sorted list idx[0..n) inside [0, dim)
__global__ void __launch_bounds__(256) k_max_gap(const int32_t *__restrict__ idx, int64_t n, int64_t dim,
                                                 int32_t *__restrict__ out) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int32_t m = 0;
    for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s <= n; s += stride) {
        const int64_t lo = s == 0 ? 0 : (int64_t)idx[s - 1] + 1;
        const int64_t hi = s == n ? dim : (int64_t)idx[s];
        const int32_t l = (int32_t)(hi > lo ? hi - lo : 0);
        m = l > m ? l : m;
    }
    if (m > 0) atomicMax(out, m);
}

hipError_t max_coordinate_gap(const int32_t *idx, int64_t n, int64_t dim, int32_t *out_max, hipStream_t st) {
    int64_t want = (n + 1 + 255) / 256;
    unsigned grid = (unsigned)(want > 2048 ? 2048 : want);
    hipLaunchKernelGGL(k_max_gap, dim3(grid), dim3(256), 0, st, idx, n, dim, out_max);
    return hipGetLastError();
}

// most leaf positions under one parent segment: max over s of pos_leaf[pos_par[s+1]] - pos_leaf[pos_par[s]]
__global__ void __launch_bounds__(256) k_max_parent_span(const int32_t *__restrict__ ppos, int64_t nparent,
                                                         const int32_t *__restrict__ lpos, int32_t *__restrict__ out) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int32_t m = 0;
    for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s < nparent; s += stride) {
        int32_t l = lpos[ppos[s + 1]] - lpos[ppos[s]];
        m = l > m ? l : m;
    }
    if (m > 0) atomicMax(out, m);
}

hipError_t max_parent_span(const int32_t *parent_pos, int64_t nparent, const int32_t *leaf_pos, int32_t *out_max,
                           hipStream_t st) {
    if (nparent <= 0) return hipSuccess;
    int64_t want = (nparent + 255) / 256;
    unsigned grid = (unsigned)(want > 2048 ? 2048 : want);
    hipLaunchKernelGGL(k_max_parent_span, dim3(grid), dim3(256), 0, st, parent_pos, nparent, leaf_pos, out_max);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256) k_count_empty(const int32_t *__restrict__ pos, int64_t nseg,
                                                     int32_t *__restrict__ out) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int32_t c = 0;
    for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s < nseg; s += stride)
        c += pos[s + 1] == pos[s] ? 1 : 0;
    if (c) atomicAdd(out, c);
}

hipError_t count_empty_segments(const int32_t *pos, int64_t nseg, int32_t *out_count, hipStream_t st) {
    if (nseg <= 0) return hipSuccess;
    int64_t want = (nseg + 255) / 256;
    unsigned grid = (unsigned)(want > 2048 ? 2048 : want);
    hipLaunchKernelGGL(k_count_empty, dim3(grid), dim3(256), 0, st, pos, nseg, out_count);
    return hipGetLastError();
}

// Clears the rows of a dense [nrows x R] result whose index is not stored in the sorted list idx[0..n):
// row ranges (idx[s-1], idx[s]) for s = 0..n (with idx[-1] = -1 and idx[n] = nrows).  One thread per
// (gap, 16-byte piece); gaps are short when most rows are stored, which is the case this serves.
__global__ void __launch_bounds__(256) k_zero_unstored_rows(const int32_t *__restrict__ idx, int64_t n, int64_t nrows,
                                                            int R, double *__restrict__ out, double beta) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s <= n; s += stride) {
        const int64_t lo = s == 0 ? 0 : (int64_t)idx[s - 1] + 1;
        const int64_t hi = s == n ? nrows : (int64_t)idx[s];
        if (beta == 0.0) for (int64_t p = lo * R; p < hi * R; ++p) out[p] = 0.0;
        else for (int64_t p = lo * R; p < hi * R; ++p) out[p] = beta * out[p];
    }
}

hipError_t zero_unstored_rows(const int32_t *idx, int64_t n, int64_t nrows, int64_t R, double *out, hipStream_t st,
                              double beta) {
    if (beta == 1.0) return hipSuccess;
    int64_t want = (n + 1 + 255) / 256;
    unsigned grid = (unsigned)(want > 4096 ? 4096 : want);
    hipLaunchKernelGGL(k_zero_unstored_rows, dim3(grid), dim3(256), 0, st, idx, n, nrows, (int)R, out, beta);
    return hipGetLastError();
}

}  // namespace comet
