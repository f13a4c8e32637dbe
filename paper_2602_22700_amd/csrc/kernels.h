// Launch wrappers of the gfx950 kernels.  Every wrapper validates nothing: shapes
// and alignment are checked by the callers in prover.cpp, which also own the
// buffers.  All launches are asynchronous on `stream`.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/imm.h"

namespace imm {
namespace k {

struct Point {
    uint64_t v[IMM_MAX_ROUNDS];
};

// dst[i] = src[i] mod p
hipError_t encode(hipStream_t stream, const void* src, int dtype, uint64_t count, uint64_t* dst);

// eq vectors of two points in one launch: outA has 2^tA entries, outB has 2^tB.
// Either count may be 0 (vector [1]).  First coordinate = most significant bit.
hipError_t eq_build2(hipStream_t stream, const Point& ptA, int tA, uint64_t* outA, const Point& ptB, int tB,
                     uint64_t* outB);

// Geometry of a split reduction: how many partial vectors a launch writes.
struct Split {
    uint32_t nsplit;      // number of partial vectors
    uint64_t per_split;   // rows (or columns) covered by one partial vector
};
Split plan_over_rows(uint64_t rows, uint64_t cols);
Split plan_over_cols(uint64_t rows, uint64_t cols);

// partial[s][j] = sum over the rows i of split s of eq[i] * T[i][j]   (j < cols)
hipError_t reduce_over_rows(hipStream_t stream, const void* T, int dtype, uint64_t rows, uint64_t cols, uint64_t ld,
                            const uint64_t* eq_rows, uint64_t* partial, Split sp);

// partial[s][i] = sum over the columns j of split s of eq[j] * T[i][j]   (i < rows)
hipError_t reduce_over_cols(hipStream_t stream, const void* T, int dtype, uint64_t rows, uint64_t cols, uint64_t ld,
                            const uint64_t* eq_cols, uint64_t* partial, Split sp);

// out[j] = sum_s partial[s][j] for j < len, 0 for len <= j < padded
hipError_t combine(hipStream_t stream, const uint64_t* partial, uint32_t nsplit, uint64_t len, uint64_t padded,
                   uint64_t* out);

// out[0] = sum_i x[i] * y[i], i < len
hipError_t dot(hipStream_t stream, const uint64_t* x, const uint64_t* y, uint64_t len, uint64_t* out);

// Number of uint64_t words of scratch that round() needs for tables of length L.
uint64_t round_scratch_words(uint64_t L);

// One sumcheck round on tables a, b of length L (power of two, >= 2).
//   fold = false: g(0,1,2) of the tables as they are -> out3.
//   fold = true : bind the leading variable to r in place (length becomes L/2), then
//                 g(0,1,2) of the folded tables -> out3; when L == 2 the folded tables
//                 have one entry and out3 = (a[0], b[0], 0).
hipError_t round(hipStream_t stream, uint64_t* a, uint64_t* b, uint64_t L, bool fold, uint64_t r, uint64_t* out3,
                 uint64_t* scratch);

}  // namespace k
}  // namespace imm
