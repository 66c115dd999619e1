// Calibration kernels: what the memory system of the device delivers for the two access patterns every
// operation of the library is made of -- a plain streaming read, and gathers of whole dense rows by lane groups
// of 8 (16 bytes per lane per load, the mapping of the rank-R kernels) from a table that is L2-resident, larger
// than L2, or larger than every cache.  The benchmark times them next to the operations, so that "what binds"
// is read off measurements taken on the same device in the same run.
#include <hip/hip_runtime.h>
#include <cstdint>

#include "../../include/comet.h"

namespace {

// Each workgroup takes consecutive 32 KB pieces (eight 16-byte loads per lane in flight, each one a contiguous
// 4 KB across the workgroup), workgroups taking the pieces in turn; non-temporal loads as for the operations' streams.
__global__ void __launch_bounds__(256) k_cal_read(const double2 *__restrict__ a, int64_t n2, double *__restrict__ sink) {
    typedef double v2d __attribute__((ext_vector_type(2)));
    const v2d *p = reinterpret_cast<const v2d *>(a);
    constexpr int kPer = 8;
    const int64_t piece = 256 * kPer, npieces = n2 / piece;
    double s = 0.0;
    for (int64_t pc = blockIdx.x; pc < npieces; pc += gridDim.x) {
        const int64_t base = pc * piece + threadIdx.x;
        v2d v[kPer];
#pragma unroll
        for (int u = 0; u < kPer; ++u) v[u] = __builtin_nontemporal_load(p + base + 256 * u);
#pragma unroll
        for (int u = 0; u < kPer; ++u) s += v[u].x + v[u].y;
    }
    for (int64_t i = npieces * piece + (int64_t)blockIdx.x * 256 + threadIdx.x; i < n2; i += (int64_t)gridDim.x * 256) {
        const v2d v = p[i];
        s += v.x + v.y;
    }
    if (s == 1.2345e300) sink[0] = s;                      // never true for finite data: keeps the loads alive
}

// Every lane group of 8 gathers `steps` rows of R doubles (R a multiple of 16) at pseudo-random row numbers.
template <int NL>
__global__ void __launch_bounds__(256) k_cal_gather(const double *__restrict__ table, uint32_t nrows, int R, int steps,
                                                    double *__restrict__ sink) {
    const uint32_t gid = (blockIdx.x * 256u + threadIdx.x) >> 3;
    const int j = threadIdx.x & 7;
    uint32_t st = gid * 2654435761u + 0x7F4A7C15u;
    st ^= st >> 15; st *= 0x2C1B3C6Du; st ^= st >> 12;
    double acc = 0.0;
    for (int s = 0; s < steps; s += 4) {
        st = st * 1664525u + 1013904223u;
        double2 v[4][NL];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t h = (st >> u) ^ (0x5bd1e995u * (uint32_t)(u + 1));
            const uint32_t row = (uint32_t)(((uint64_t)(h >> 3) * nrows) >> 29);     // uniform over [0, nrows)
            const double *p = table + (size_t)row * R + 2 * j;
#pragma unroll
            for (int q = 0; q < NL; ++q) v[u][q] = *reinterpret_cast<const double2 *>(p + 16 * q);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int q = 0; q < NL; ++q) acc += v[u][q].x + v[u][q].y;
    }
    if (acc == 1.2345e300) sink[0] = acc;
}

}  // namespace

extern "C" {

comet_status comet_calibrate_read(const double *data, int64_t n, double *sink, void *stream) {
    if (!data || !sink || n < 2) return COMET_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(data) & 15u) return COMET_ERR_INVALID_ARG;
    hipLaunchKernelGGL(k_cal_read, dim3(8192), dim3(256), 0, (hipStream_t)stream, reinterpret_cast<const double2 *>(data), n / 2, sink);
    return hipGetLastError() == hipSuccess ? COMET_OK : COMET_ERR_DEVICE;
}

comet_status comet_calibrate_gather(const double *table, int64_t nrows, int64_t R, int64_t gathers, double *sink, void *stream) {
    if (!table || !sink || nrows < 1 || nrows >= (int64_t(1) << 29) || gathers < 1) return COMET_ERR_INVALID_ARG;
    if (R != 16 && R != 32 && R != 64) return COMET_ERR_UNSUPPORTED;
    if (reinterpret_cast<uintptr_t>(table) & 15u) return COMET_ERR_INVALID_ARG;
    const int groups = 2048 * 32;                               // 2048 workgroups of 32 lane groups
    int64_t steps = (gathers + groups - 1) / groups;
    steps = (steps + 3) / 4 * 4;
    if (steps > (int64_t(1) << 30)) return COMET_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (R == 16) hipLaunchKernelGGL(k_cal_gather<1>, dim3(2048), dim3(256), 0, st, table, (uint32_t)nrows, 16, (int)steps, sink);
    else if (R == 32) hipLaunchKernelGGL(k_cal_gather<2>, dim3(2048), dim3(256), 0, st, table, (uint32_t)nrows, 32, (int)steps, sink);
    else hipLaunchKernelGGL(k_cal_gather<4>, dim3(2048), dim3(256), 0, st, table, (uint32_t)nrows, 64, (int)steps, sink);
    return hipGetLastError() == hipSuccess ? COMET_OK : COMET_ERR_DEVICE;
}

}  // extern "C"
