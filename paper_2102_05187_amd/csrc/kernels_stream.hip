#include "stream_kernels.hpp"
namespace comet {
bool stream_supports_rank(int64_t) { return false; }
bool stream_mttkrp_supports_rank(int64_t) { return false; }
size_t stream_scratch_bytes(int64_t, int64_t) { return 16; }
hipError_t stream_segreduce(const Schedule &, const int32_t *, const int32_t *, const double *, const int32_t *,
                            const double *, int64_t, double *, void *, hipStream_t) { return hipErrorNotSupported; }
hipError_t stream_ttv_coo(const Schedule &, const int32_t *, const int32_t *, const int32_t *, const double *,
                          const double *, int32_t *, int32_t *, double *, void *, hipStream_t) { return hipErrorNotSupported; }
hipError_t stream_mttkrp(const Schedule &, const int32_t *, const int32_t *, int64_t, const int32_t *, const int32_t *,
                         const int32_t *, const double *, const double *, const double *, int64_t, double *, void *,
                         hipStream_t) { return hipErrorNotSupported; }
}
