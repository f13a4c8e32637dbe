// Launch wrappers of the logit-distance kernels (ldd.hip).  Shapes are validated by the callers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/imm.h"

namespace imm {
namespace k {

// tv_out[i], kl_out[i] for row i of X (deployed) against row i of Y (reference); either may be null.
hipError_t ldd_tv_kl(hipStream_t stream, const float* X, const float* Y, uint64_t T, uint64_t n, uint64_t ld,
                     double* tv_out, double* kl_out);

// out[i] = top-K distance of row i of X for the index set idx[i*K .. i*K+K).
hipError_t topk_distance(hipStream_t stream, const float* X, uint64_t T, uint64_t n, uint64_t ld, const int32_t* idx,
                         uint32_t K, double* out);

// *count_dev = number of i < T with dist[i] > t1 (count_dev is cleared first, on the stream).
hipError_t tail_count(hipStream_t stream, const double* dist, uint64_t T, double t1, unsigned long long* count_dev);

}  // namespace k
}  // namespace imm
