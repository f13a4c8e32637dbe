// Launch wrappers of the logit-distance kernels (ldd.hip).  Shapes are validated by the callers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/imm.h"

namespace imm {
namespace k {

// tv_out[i], kl_out[i] for row i of X (deployed) against row i of Y (reference); either may be null.
// Working memory: `slots`, `posts`, `sums`, `counters` of ldd_slot_bytes(T, n), ldd_post_bytes(T),
// ldd_sum_bytes(T), ldd_counter_bytes(T) bytes in the state ldd_init_sync
// leaves them in (once after allocation; the kernel restores that state before it ends).
// `wait_polls` bounds how often a workgroup looks for the rest of its row before it does without.
size_t ldd_slot_bytes(uint64_t T, uint64_t n);
size_t ldd_post_bytes(uint64_t T);
size_t ldd_sum_bytes(uint64_t T);
size_t ldd_counter_bytes(uint64_t T);
hipError_t ldd_init_sync(hipStream_t stream, uint64_t* slots, size_t slot_bytes, uint64_t* posts, size_t post_bytes,
                         uint64_t* sums, size_t sum_bytes, uint32_t* counters, size_t counter_bytes);
hipError_t ldd_tv_kl(hipStream_t stream, const float* X, const float* Y, uint64_t T, uint64_t n, uint64_t ld,
                     uint64_t* slots, uint64_t* posts, uint64_t* sums, uint32_t* counters, uint64_t wait_polls,
                     double* tv_out, double* kl_out);

// out[i] = top-K distance of row i of X for the index set idx[i*K .. i*K+K).
hipError_t topk_distance(hipStream_t stream, const float* X, uint64_t T, uint64_t n, uint64_t ld, const int32_t* idx,
                         uint32_t K, double* out);

// *count_dev = number of i < T with dist[i] > t1 (count_dev is cleared first, on the stream).
hipError_t tail_count(hipStream_t stream, const double* dist, uint64_t T, double t1, unsigned long long* count_dev);

}  // namespace k
}  // namespace imm
