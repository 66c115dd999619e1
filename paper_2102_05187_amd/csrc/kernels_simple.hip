// Simple kernel family: one lane group (rank 1) or one thread (rank R) per output element.
//
// These kernels follow the loop structure the paper's level rules give directly (Section 6.2,
// Table "Generated code to access nonzeros coordinates"): the compressed-unique loop over
// pos[m]..pos[m+1] with idx = crd[p], values indexed by the leaf position, dense operands
// indexed row-major by the coordinate.  They serve any rank and any segment-length
// distribution, need no scratch memory and no carries, and are the fallback for ranks the tiled
// kernels do not specialise.  Long segments serialise on one lane group, so skewed inputs are
// slow here; the nonzero-tiled family exists for those.
#include "kernels.hpp"

namespace comet {

static inline unsigned nblocks(int64_t n, int per_block) {
    int64_t b = (n + per_block - 1) / per_block;
    return (unsigned)(b < 1 ? 1 : b);
}

// ---- rank 1: G lanes cooperate on one segment, butterfly add inside the group -------------------
template <int G>
__global__ void __launch_bounds__(256) k_seg1_simple(const int32_t *__restrict__ pos, const int32_t *__restrict__ crd,
                                                     const double *__restrict__ vals, int64_t nseg,
                                                     const int32_t *__restrict__ rowmap,
                                                     const double *__restrict__ x, double *__restrict__ out, Epilogue ep) {
    int64_t s = ((int64_t)blockIdx.x * 256 + threadIdx.x) / G;
    int lane = threadIdx.x % G;
    if (s >= nseg) return;                       // whole groups leave together (G divides 64)
    int32_t b = pos[s], e = pos[s + 1];
    double acc = 0.0;
    for (int32_t p = b + lane; p < e; p += G) acc = fma(vals[p], x[crd[p]], acc);
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o, G);
    if (lane == 0) { double *o = out + (rowmap ? (int64_t)rowmap[s] : s); *o = ep_apply(ep, acc, o); }
}

// ---- rank R: thread (s, r), r fastest, so a wavefront reads contiguous pieces of operand rows ---
__global__ void __launch_bounds__(256) k_segR_simple(const int32_t *__restrict__ pos, const int32_t *__restrict__ crd,
                                                     const double *__restrict__ vals, int64_t nseg,
                                                     const int32_t *__restrict__ rowmap,
                                                     const double *__restrict__ Dn, int R,
                                                     double *__restrict__ out, Epilogue ep) {
    int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= nseg * R) return;
    int64_t s = t / R;
    int r = (int)(t - s * R);
    int32_t b = pos[s], e = pos[s + 1];
    double acc = 0.0;
    for (int32_t p = b; p < e; ++p) acc = fma(vals[p], Dn[(int64_t)crd[p] * R + r], acc);
    double *o = out + (rowmap ? (int64_t)rowmap[s] : s) * R + r;
    *o = ep_apply(ep, acc, o);
}

hipError_t simple_segreduce(const int32_t *pos, const int32_t *crd, const double *vals, int64_t nseg,
                            int64_t nnz, const int32_t *rowmap, const double *Dn, int64_t R, double *out,
                            hipStream_t st, Epilogue ep) {
    if (nseg <= 0) return hipSuccess;
    if (R == 1) {
        double mean = (double)nnz / (double)nseg;
        if (mean <= 6.0)
            hipLaunchKernelGGL(k_seg1_simple<4>, dim3(nblocks(nseg * 4, 256)), dim3(256), 0, st, pos, crd, vals, nseg, rowmap, Dn, out, ep);
        else if (mean <= 24.0)
            hipLaunchKernelGGL(k_seg1_simple<16>, dim3(nblocks(nseg * 16, 256)), dim3(256), 0, st, pos, crd, vals, nseg, rowmap, Dn, out, ep);
        else
            hipLaunchKernelGGL(k_seg1_simple<64>, dim3(nblocks(nseg * 64, 256)), dim3(256), 0, st, pos, crd, vals, nseg, rowmap, Dn, out, ep);
    } else {
        hipLaunchKernelGGL(k_segR_simple, dim3(nblocks(nseg * R, 256)), dim3(256), 0, st, pos, crd, vals, nseg, rowmap, Dn, (int)R, out, ep);
    }
    return hipGetLastError();
}

// ---- MTTKRP: thread (slice, r); inner sum over the fiber, scaled by the B row, summed per slice --
__global__ void __launch_bounds__(256) k_mttkrp_simple(const int32_t *__restrict__ pos2, const int32_t *__restrict__ crd1,
                                                       int64_t nslice, const int32_t *__restrict__ pos3,
                                                       const int32_t *__restrict__ crd2, const int32_t *__restrict__ crd3,
                                                       const double *__restrict__ vals, const double *__restrict__ B,
                                                       const double *__restrict__ C, int R, double *__restrict__ M,
                                                       Epilogue ep) {
    int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= nslice * R) return;
    int64_t s = t / R;
    int r = (int)(t - s * R);
    double acc = 0.0;
    for (int32_t f = pos2[s]; f < pos2[s + 1]; ++f) {
        double inner = 0.0;
        for (int32_t p = pos3[f]; p < pos3[f + 1]; ++p) inner = fma(vals[p], C[(int64_t)crd3[p] * R + r], inner);
        acc = fma(B[(int64_t)crd2[f] * R + r], inner, acc);
    }
    double *o = M + (int64_t)crd1[s] * R + r;
    *o = ep_apply(ep, acc, o);
}

hipError_t simple_mttkrp(const int32_t *pos2, const int32_t *crd1, int64_t nslice, const int32_t *pos3,
                         const int32_t *crd2, const int32_t *crd3, const double *vals, const double *B,
                         const double *C, int64_t R, double *M, hipStream_t st, Epilogue ep) {
    if (nslice <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_mttkrp_simple, dim3(nblocks(nslice * R, 256)), dim3(256), 0, st, pos2, crd1, nslice, pos3,
                       crd2, crd3, vals, B, C, (int)R, M, ep);
    return hipGetLastError();
}

// ---- TTV on sorted COO: the thread that holds a run's first nonzero sums the whole run -----------
// One workgroup per tile of `tile` consecutive nonzeros, tile/256 consecutive nonzeros per thread.
// A run's output slot is run_base[tile] + (runs started earlier in the tile).
template <int PER>
__global__ void __launch_bounds__(256) k_ttv_coo_simple(const int32_t *__restrict__ c0, const int32_t *__restrict__ c1,
                                                        const int32_t *__restrict__ c2, const double *__restrict__ vals,
                                                        int64_t nnz, const int32_t *__restrict__ run_base,
                                                        const double *__restrict__ v, int32_t *__restrict__ y0,
                                                        int32_t *__restrict__ y1, double *__restrict__ yv) {
    __shared__ int32_t cnt[256];
    const int tid = threadIdx.x;
    const int64_t b = (int64_t)blockIdx.x * (PER * 256) + (int64_t)tid * PER;
    int heads = 0;
    for (int q = 0; q < PER; ++q) {
        int64_t p = b + q;
        if (p < nnz && (p == 0 || c0[p] != c0[p - 1] || c1[p] != c1[p - 1])) ++heads;
    }
    cnt[tid] = heads;
    __syncthreads();
    if (tid == 0) {
        int32_t run = run_base[blockIdx.x];
        for (int i = 0; i < 256; ++i) { int32_t h = cnt[i]; cnt[i] = run; run += h; }
    }
    __syncthreads();
    int32_t slot = cnt[tid];
    for (int q = 0; q < PER; ++q) {
        int64_t p = b + q;
        if (p >= nnz) break;
        if (!(p == 0 || c0[p] != c0[p - 1] || c1[p] != c1[p - 1])) continue;
        const int32_t i = c0[p], j = c1[p];
        double acc = 0.0;
        for (int64_t w = p; w < nnz && c0[w] == i && c1[w] == j; ++w) acc = fma(vals[w], v[c2[w]], acc);
        y0[slot] = i; y1[slot] = j; yv[slot] = acc;
        ++slot;
    }
}

hipError_t simple_ttv_coo(const int32_t *c0, const int32_t *c1, const int32_t *c2, const double *vals,
                          int64_t nnz, int tile, int64_t ntiles, const int32_t *run_base, const double *v,
                          int32_t *ycrd0, int32_t *ycrd1, double *yvals, hipStream_t st) {
    if (ntiles <= 0) return hipSuccess;
    if (tile != 4096) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_ttv_coo_simple<16>, dim3((unsigned)ntiles), dim3(256), 0, st, c0, c1, c2, vals, nnz, run_base,
                       v, ycrd0, ycrd1, yvals);
    return hipGetLastError();
}

}  // namespace comet
