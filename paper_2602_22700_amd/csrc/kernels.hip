// gfx950 kernels of the matmul sumcheck prover: field encoding, eq-vector build,
// the two streaming partial-evaluation reductions, and the per-round
// "evaluate g(0,1,2) + fold" kernel.  Wave size is 64 throughout.
//
// The protocol these serve (paper section 5.2 item 2 instantiated as a sumcheck
// for C = A.B over Goldilocks) and all conventions are stated in include/imm.h.
#include "kernels.h"

#include "goldilocks_device.h"
#include "sha256_device.h"

namespace imm {
namespace k {
namespace {

constexpr int kBlock = 256;  // 4 waves
constexpr int kWaves = kBlock / 64;

// ------------------------------------------------------------------ helpers
// Two adjacent table entries are fetched with one load.  Tables are streamed exactly once,
// so their loads and the encoder's stores are non-temporal: they do not displace the eq
// vectors and the partial results from the caches, and on this part they reach a markedly
// higher share of the HBM rate than plain accesses.
typedef unsigned long long v2u64 __attribute__((ext_vector_type(2)));

template <typename S> struct RawPair;
template <> struct RawPair<int8_t> { using type = uint16_t; };
template <> struct RawPair<int16_t> { using type = uint32_t; };
template <> struct RawPair<int64_t> { using type = v2u64; };
template <> struct RawPair<uint64_t> { using type = v2u64; };

template <typename S> __device__ __forceinline__ uint64_t to_field(S v) { return gl::enc((int64_t)v); }
template <> __device__ __forceinline__ uint64_t to_field<uint64_t>(uint64_t v) { return v; }

template <typename S> __device__ __forceinline__ typename RawPair<S>::type load_pair(const S* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const typename RawPair<S>::type*>(p));
}
template <typename S> __device__ __forceinline__ S load_one(const S* p) { return __builtin_nontemporal_load(p); }

template <typename S> __device__ __forceinline__ void unpack(typename RawPair<S>::type raw, uint64_t& f0, uint64_t& f1);
template <> __device__ __forceinline__ void unpack<int8_t>(uint16_t raw, uint64_t& f0, uint64_t& f1) {
    f0 = gl::enc((int64_t)(int8_t)(raw & 0xFF));
    f1 = gl::enc((int64_t)(int8_t)(raw >> 8));
}
template <> __device__ __forceinline__ void unpack<int16_t>(uint32_t raw, uint64_t& f0, uint64_t& f1) {
    f0 = gl::enc((int64_t)(int16_t)(raw & 0xFFFF));
    f1 = gl::enc((int64_t)(int16_t)(raw >> 16));
}
template <> __device__ __forceinline__ void unpack<int64_t>(v2u64 raw, uint64_t& f0, uint64_t& f1) {
    f0 = gl::enc((int64_t)raw.x);
    f1 = gl::enc((int64_t)raw.y);
}
template <> __device__ __forceinline__ void unpack<uint64_t>(v2u64 raw, uint64_t& f0, uint64_t& f1) {
    f0 = raw.x;
    f1 = raw.y;
}

// Keeps the loads written above this point above it: the empty statement may touch memory as far as
// the optimiser knows (so it does not sink a load past it, next to its first use), and the scheduling
// barrier holds the instruction scheduler to the same order.  What is written above are the requests
// for data that is only needed later; what follows works on data requested earlier.
__device__ __forceinline__ void loads_stay_above() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

__device__ __forceinline__ uint64_t wave_sum(uint64_t v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = gl::add(v, __shfl_down(v, off, 64));
    return v;  // valid in lane 0
}

// Sum of one field element per thread over a block of kBlock threads; result valid in thread 0.
// `lds` holds kWaves words and may be reused after the call returns (ends with a barrier).
__device__ __forceinline__ uint64_t block_sum(uint64_t v, uint64_t* lds) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    uint64_t total = 0;
    if (threadIdx.x == 0) {
        total = lds[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) total = gl::add(total, lds[w]);
    }
    __syncthreads();
    return total;
}

// ------------------------------------------------------------------ partial vectors summed by the last workgroup
// Where a reduction is split over several workgroups per output, each writes a partial vector and
// the sum is usually a launch of its own.  Inside a launch that goes on for much longer (the
// reduction of the other, larger operand) the sum can be had for nothing: a workgroup that has
// written its partial vector counts itself in on its block of outputs, and the one that finds it
// is the last sums the block.  Partial values and counters are written with agent-scope atomic
// stores (they go through to the level all XCDs share) and read with agent-scope atomic loads;
// nothing relies on the order in which such stores become visible: an empty word is kNoValue, which
// no canonical field element can be, so every word says for itself whether it is there, and the
// summing workgroup looks again until it is (the count only tells it that the words are on their
// way).  It puts kNoValue back as it goes and zeroes the counter, so the next launch finds the
// memory as this one did.  The looking again is bounded; if the bound were ever reached the word
// taken is kNoValue, which the round kernels recognise as not canonical and report.
constexpr uint32_t kHandoverPolls = 1u << 22;

__device__ __forceinline__ void put_word(uint64_t* p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t peek_word(const uint64_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct Handover {
    uint32_t* counters;  // one per block of outputs (grid x index), zero between launches
    uint64_t* out;       // the summed vector
    uint64_t padded;     // out[len .. padded) is zeroed by the workgroup (0, 0)
};

// Called by every thread of workgroup (bx, by) of a split reduction after it has put_word() its W
// partial values partial[by * len + first + c * stride], c < W (those below len).  `last` is a word
// of LDS.  The summing workgroup asks for the words of many splits at once: one after the other,
// each a round trip to memory, they would take longer than the reduction itself.
constexpr int kHandoverBatch = 16;  // splits whose words a thread has in flight together
#ifndef IMM_HANDOVER_MAX_SPLITS
#define IMM_HANDOVER_MAX_SPLITS 16
#endif
constexpr uint64_t kHandoverMaxSplits = IMM_HANDOVER_MAX_SPLITS;  // partial vectors per launch where they are summed this way

template <int W>
__device__ __forceinline__ void sum_by_last_arriver(const Handover& h, uint64_t* __restrict__ partial, uint32_t nsplit,
                                                    uint64_t len, uint32_t bx, uint32_t by, uint64_t first, uint64_t stride,
                                                    uint32_t* last) {
    if (bx == 0 && by == 0)
        for (uint64_t j = len + threadIdx.x; j < h.padded; j += kBlock) h.out[j] = 0;
    __syncthreads();  // every wave of the workgroup has issued its stores
    if (threadIdx.x == 0) {
        const uint32_t before = __hip_atomic_fetch_add(h.counters + bx, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *last = before + 1 == nsplit;
    }
    __syncthreads();
    if (!*last) return;
    uint64_t v[W];
#pragma unroll
    for (int c = 0; c < W; ++c) v[c] = 0;
    for (uint32_t s0 = 0; s0 < nsplit; s0 += kHandoverBatch) {
        uint64_t t[W][kHandoverBatch];
#pragma unroll
        for (int c = 0; c < W; ++c)
#pragma unroll
            for (int j = 0; j < kHandoverBatch; ++j) {
                const uint64_t col = first + c * stride;
                t[c][j] = (col < len && s0 + j < nsplit) ? peek_word(partial + (uint64_t)(s0 + j) * len + col) : 0;
            }
#pragma unroll
        for (int c = 0; c < W; ++c)
#pragma unroll
            for (int j = 0; j < kHandoverBatch; ++j) {
                const uint64_t col = first + c * stride;
                if (col < len && s0 + j < nsplit) {
                    const uint64_t* word = partial + (uint64_t)(s0 + j) * len + col;
                    uint64_t x = t[c][j];
                    for (uint32_t spin = 0; x == kNoValue && spin < kHandoverPolls; ++spin) x = peek_word(word);
                    v[c] = (x == kNoValue || v[c] == kNoValue) ? kNoValue : gl::add(v[c], x);
                }
            }
    }
    // The words go back to empty in a pass of their own: a store among the loads above would have each
    // wait for a word also wait for the store before it to come back from memory.
    for (uint32_t sidx = 0; sidx < nsplit; ++sidx)
#pragma unroll
        for (int c = 0; c < W; ++c)
            if (first + c * stride < len) put_word(partial + (uint64_t)sidx * len + first + c * stride, kNoValue);
#pragma unroll
    for (int c = 0; c < W; ++c)
        if (first + c * stride < len) h.out[first + c * stride] = v[c];
    if (threadIdx.x == 0) __hip_atomic_store(h.counters + bx, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ------------------------------------------------------------------ encode
// The work of workgroup `block` out of `nblocks` that share the array.
template <typename S, bool VEC>
__device__ __forceinline__ void encode_block(const S* __restrict__ src, uint64_t* __restrict__ dst, uint64_t count,
                                             uint32_t block, uint32_t nblocks) {
    const uint64_t stride = (uint64_t)nblocks * kBlock;
    const uint64_t t = (uint64_t)block * kBlock + threadIdx.x;
    if (VEC) {
        // one wave reads 64 adjacent pairs and writes 1 KiB of contiguous field elements
        const uint64_t pairs = count >> 1;
        for (uint64_t p = t; p < pairs; p += stride) {
            v2u64 o;
            uint64_t f0, f1;
            // the narrow source is read with ordinary loads; only the 8x larger output streams
            unpack<S>(*reinterpret_cast<const typename RawPair<S>::type*>(src + 2 * p), f0, f1);
            o.x = f0;
            o.y = f1;
            __builtin_nontemporal_store(o, reinterpret_cast<v2u64*>(dst + 2 * p));
        }
        if ((count & 1) && t == 0) dst[count - 1] = to_field<S>(src[count - 1]);
    } else {
        for (uint64_t i = t; i < count; i += stride) dst[i] = to_field<S>(src[i]);
    }
}

template <typename S, bool VEC>
__global__ __launch_bounds__(kBlock) void encode_kernel(const S* __restrict__ src, uint64_t* __restrict__ dst,
                                                        uint64_t count) {
    encode_block<S, VEC>(src, dst, count, blockIdx.x, gridDim.x);
}

// workgroups that encode `count` entries, and whether the two-entries-per-thread form applies
template <typename S>
uint32_t encode_blocks(const void* src, const uint64_t* dst, uint64_t count, bool* vec) {
    *vec = (reinterpret_cast<uintptr_t>(src) % (2 * sizeof(S)) == 0) && (reinterpret_cast<uintptr_t>(dst) % 16 == 0);
    const uint64_t items = *vec ? (count + 1) / 2 : count;
    uint64_t blocks = (items + kBlock - 1) / kBlock;  // one item per thread: many small blocks stream best
    if (blocks > (1u << 22)) blocks = 1u << 22;
    return (uint32_t)blocks;
}

template <typename S>
hipError_t launch_encode(hipStream_t stream, const void* src, uint64_t count, uint64_t* dst) {
    if (count == 0) return hipSuccess;
    bool vec;
    const uint32_t blocks = encode_blocks<S>(src, dst, count, &vec);
    if (vec)
        hipLaunchKernelGGL((encode_kernel<S, true>), dim3((unsigned)blocks), dim3(kBlock), 0, stream,
                           static_cast<const S*>(src), dst, count);
    else
        hipLaunchKernelGGL((encode_kernel<S, false>), dim3((unsigned)blocks), dim3(kBlock), 0, stream,
                           static_cast<const S*>(src), dst, count);
    return hipGetLastError();
}

// ------------------------------------------------------------------ eq vectors
// out[i] = prod_k (bit_k(i) ? r_k : 1 - r_k), bit_1 = most significant bit of i.
// Each entry is an independent product of t factors: no synchronisation, and the
// result is the same canonical value the doubling recurrence gives.
// The points are kernel arguments.  The body below is expanded inside the kernels, not called: as
// long as a kernel reads its own struct arguments with constant indices they come straight from
// the argument segment, while handing them to a function, even an inlined one, makes every thread
// of the launch keep a private 512-byte copy.
#define IMM_EQ_BUILD2_BODY(ptA, tA, outA, ptB, tB, outB, planesB, block)                          \
    do {                                                                                          \
        uint64_t idx_ = (uint64_t)(block) * kBlock + threadIdx.x;                                 \
        const uint64_t nA_ = 1ull << (tA), nB_ = 1ull << (tB);                                    \
        const bool second_ = idx_ >= nA_;                                                         \
        if (second_) idx_ -= nA_;                                                                 \
        const int t_ = second_ ? (tB) : (tA);                                                     \
        uint64_t w_ = 1;                                                                          \
        _Pragma("unroll") for (int kk_ = 0; kk_ < IMM_MAX_ROUNDS; ++kk_) {                        \
            if (kk_ < t_) {                                                                       \
                const uint64_t r_ = second_ ? (ptB).v[kk_] : (ptA).v[kk_];                        \
                const uint64_t f_ = ((idx_ >> (t_ - 1 - kk_)) & 1) ? r_ : gl::sub(1, r_);         \
                w_ = gl::mul(w_, f_);                                                             \
            }                                                                                     \
        }                                                                                         \
        if (!second_ || idx_ < nB_) (second_ ? (outB) : (outA))[idx_] = w_;                       \
        if (second_ && idx_ < nB_ && (planesB) != nullptr) eq_planes_store((planesB), idx_, w_);  \
    } while (0)

// The second vector once more, cut into bytes for the int8 reduction: for every four neighbouring
// entries 4g .. 4g+3 eight words, word k holding byte k of each of the four (entry 4g in the low
// byte).  A dot product of such a word with four table bytes is the sum of four byte products.
__device__ __forceinline__ void eq_planes_store(uint32_t* planes, uint64_t idx, uint64_t w) {
    uint8_t* pb = reinterpret_cast<uint8_t*>(planes) + (idx >> 2) * 32 + (idx & 3);
#pragma unroll
    for (int k = 0; k < 8; ++k) pb[4 * k] = (uint8_t)(w >> (8 * k));
}

__global__ __launch_bounds__(kBlock) void eq_build2_kernel(Point ptA, int tA, uint64_t* __restrict__ outA, Point ptB,
                                                           int tB, uint64_t* __restrict__ outB,
                                                           uint32_t* __restrict__ planesB) {
    IMM_EQ_BUILD2_BODY(ptA, tA, outA, ptB, tB, outB, planesB, blockIdx.x);
}

// Everything a proof launches before its reductions, in one grid: the eq vectors of both points
// (first workgroups), the widening of A from int16 and the widening of B from int8.  The three are
// independent of one another; as launches of their own the two short ones cost their ramp and a gap.
struct FrontArgs {
    const int16_t* srcA;
    uint64_t* dstA;
    uint64_t countA;
    const int8_t* srcB;
    uint64_t* dstB;
    uint64_t countB;
    uint64_t* eqA;
    uint64_t* eqB;
    int tA, tB;
    uint32_t blocks_eq, blocks_A, blocks_B;
};
template <bool VA, bool VB>
__global__ __launch_bounds__(kBlock) void front_kernel(FrontArgs f, Point ptA, Point ptB) {
    uint32_t b = blockIdx.x;
    if (b < f.blocks_eq) {
        IMM_EQ_BUILD2_BODY(ptA, f.tA, f.eqA, ptB, f.tB, f.eqB, static_cast<uint32_t*>(nullptr), b);
        return;
    }
    b -= f.blocks_eq;
    if (b < f.blocks_A)
        encode_block<int16_t, VA>(f.srcA, f.dstA, f.countA, b, f.blocks_A);
    else
        encode_block<int8_t, VB>(f.srcB, f.dstB, f.countB, b - f.blocks_A, f.blocks_B);
}

// ------------------------------------------------------------------ sum of per-split partial vectors
// 64 outputs per block; the four waves take the splits s = w, w + 4, ... and meet in LDS.
__device__ __forceinline__ void combine_block(const uint64_t* __restrict__ partial, uint32_t nsplit, uint64_t len,
                                              uint64_t padded, uint64_t* __restrict__ out, uint32_t block,
                                              uint64_t (*lds)[64]) {
    const uint32_t lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint64_t j = (uint64_t)block * 64 + lane;
    uint64_t v = 0;
    if (j < len) {
#pragma unroll 8
        for (uint32_t s = w; s < nsplit; s += kWaves) v = gl::add(v, partial[(uint64_t)s * len + j]);
    }
    lds[w][lane] = v;
    __syncthreads();
    if (w == 0 && j < padded) {
#pragma unroll
        for (int k = 1; k < kWaves; ++k) v = gl::add(v, lds[k][lane]);
        out[j] = v;
    }
}

// ------------------------------------------------------------------ reduction over the columns (row-wise)
// Block = R consecutive rows x one column split.  A lane owns the column pairs
// (2*tid, 2*tid+1) + 512*u of the split, so one wave load covers 1 KiB of a row and the
// eq pair is loaded once and reused for the R rows (one row per block costs a tenth of the
// rate: the eq pairs come from L2 but take the same path into the CU as the table).  In the
// full-tile path all R*U 16-byte loads of a trip are issued before the first multiply of the
// trip before it, which is what keeps enough bytes in flight per CU to stream at HBM rate.
// One trip's requests of a lane: U eq pairs and R x U pairs of table entries.
template <typename S, int R, int U>
struct ColsTrip {
    ulonglong2 e[U];
    typename RawPair<S>::type x[U][R];
};
template <typename S, int R, int U>
__device__ __forceinline__ void cols_trip_load(ColsTrip<S, R, U>& t, const S* __restrict__ base, uint64_t ld,
                                               const uint64_t* __restrict__ eqb, uint64_t p) {
#pragma unroll
    for (int u = 0; u < U; ++u) t.e[u] = *reinterpret_cast<const ulonglong2*>(eqb + 2 * (p + u * kBlock));
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int r = 0; r < R; ++r) t.x[u][r] = load_pair<S>(base + r * ld + 2 * (p + u * kBlock));
}
template <typename S, int R, int U>
__device__ __forceinline__ void cols_trip_accumulate(const ColsTrip<S, R, U>& t, gl::Acc (&acc)[R]) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int r = 0; r < R; ++r) {
            uint64_t f0, f1;
            unpack<S>(t.x[u][r], f0, f1);
            gl::acc_mac(acc[r], f0, t.e[u].x);
            gl::acc_mac(acc[r], f1, t.e[u].y);
        }
}
template <typename S, int R, int U>
__device__ __forceinline__ void cols_full_tile(const S* __restrict__ base, uint64_t ld, const uint64_t* __restrict__ eqb,
                                               uint64_t npairs, gl::Acc (&acc)[R]) {
    using Raw = typename RawPair<S>::type;
    uint64_t p = threadIdx.x;
    // Whole trips (the same number for every lane), two sets of registers: the requests of the next
    // trip go out before the current one is worked on, so a wave always has a trip's worth of loads
    // in flight.  The loop has one path (no request behind a branch).
    const uint64_t trips = npairs / (U * kBlock);
    if (trips) {
        constexpr uint64_t kStep = (uint64_t)U * kBlock;
        uint64_t at = 0;  // the trip to ask for next
        auto next_trip = [&]() { return p + (at++) * kStep; };
        ColsTrip<S, R, U> ta, tb;
        cols_trip_load(ta, base, ld, eqb, next_trip());
        uint64_t t = 0;  // trips asked for so far, less one: ta holds the t-th
        while (t + 2 < trips) {
            cols_trip_load(tb, base, ld, eqb, next_trip());
            loads_stay_above();
            cols_trip_accumulate(ta, acc);
            cols_trip_load(ta, base, ld, eqb, next_trip());
            loads_stay_above();
            cols_trip_accumulate(tb, acc);
            t += 2;
        }
        if (t + 1 < trips) {
            cols_trip_load(tb, base, ld, eqb, next_trip());
            loads_stay_above();
            cols_trip_accumulate(ta, acc);
            cols_trip_accumulate(tb, acc);
        } else {
            cols_trip_accumulate(ta, acc);
        }
        p += trips * kStep;
    }
    for (; p < npairs; p += kBlock) {
        ulonglong2 e = *reinterpret_cast<const ulonglong2*>(eqb + 2 * p);
        Raw x[R];
#pragma unroll
        for (int r = 0; r < R; ++r) x[r] = load_pair<S>(base + r * ld + 2 * p);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            uint64_t f0, f1;
            unpack<S>(x[r], f0, f1);
            gl::acc_mac(acc[r], f0, e.x);
            gl::acc_mac(acc[r], f1, e.y);
        }
    }
}

// The work of workgroup (bx, by) of the grid (row blocks, column splits).
template <typename S, int R, int U, bool VEC>
__device__ __forceinline__ void reduce_over_cols_block(const S* __restrict__ T, uint64_t ld, uint64_t rows, uint64_t cols,
                                                       const uint64_t* __restrict__ eq, uint64_t* __restrict__ partial,
                                                       uint64_t cols_per_split, uint32_t bx, uint32_t by, uint64_t* lds) {
    const uint64_t row0 = (uint64_t)bx * R;
    const uint64_t c_begin = (uint64_t)by * cols_per_split;
    uint64_t c_end = c_begin + cols_per_split;
    if (c_end > cols) c_end = cols;
    const uint64_t span = c_end - c_begin;

    gl::Acc acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) gl::acc_clear(acc[r]);

    const S* base = T + row0 * ld + c_begin;
    const uint64_t* eqb = eq + c_begin;
    uint64_t done = 0;  // columns of the split already accumulated
    if (VEC && row0 + R <= rows) {
        cols_full_tile<S, R, U>(base, ld, eqb, span >> 1, acc);
        done = span & ~uint64_t(1);
    }
    // whatever is left: a ragged last tile, an odd last column, or an unaligned table
    for (uint64_t c = done + threadIdx.x; c < span; c += kBlock) {
        uint64_t e = eqb[c];
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (row0 + r < rows) gl::acc_mac(acc[r], to_field<S>(load_one<S>(base + r * ld + c)), e);
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        uint64_t total = block_sum(gl::acc_reduce(acc[r]), lds);
        if (threadIdx.x == 0 && row0 + r < rows) partial[(uint64_t)by * rows + row0 + r] = total;
    }
}

template <typename S, int R, int U, bool VEC>
__global__ __launch_bounds__(kBlock) void reduce_over_cols_kernel(const S* __restrict__ T, uint64_t ld, uint64_t rows,
                                                                  uint64_t cols, const uint64_t* __restrict__ eq,
                                                                  uint64_t* __restrict__ partial,
                                                                  uint64_t cols_per_split) {
    __shared__ uint64_t lds[kWaves];
    reduce_over_cols_block<S, R, U, VEC>(T, ld, rows, cols, eq, partial, cols_per_split, blockIdx.x, blockIdx.y, lds);
}

// The same reduction (single column split) with the sum of another reduction's partial vectors riding
// in the same launch: the first `cblocks` workgroups do that sum, a few microseconds of work that
// would otherwise hold a launch slot of its own between two long kernels (placed last in the grid
// they made the launch half a microsecond longer).
struct CombineArgs {
    const uint64_t* partial;
    uint32_t nsplit;
    uint64_t len, padded;
    uint64_t* out;
};
template <typename S, int R, int U, bool VEC>
__global__ __launch_bounds__(kBlock) void reduce_over_cols_and_combine_kernel(const S* __restrict__ T, uint64_t ld,
                                                                              uint64_t rows, uint64_t cols,
                                                                              const uint64_t* __restrict__ eq,
                                                                              uint64_t* __restrict__ partial,
                                                                              CombineArgs c, uint32_t cblocks) {
    __shared__ uint64_t lds[kWaves][64];
    if (blockIdx.x < cblocks)
        combine_block(c.partial, c.nsplit, c.len, c.padded, c.out, blockIdx.x, lds);
    else
        reduce_over_cols_block<S, R, U, VEC>(T, ld, rows, cols, eq, partial, cols, blockIdx.x - cblocks, 0, &lds[0][0]);
}

constexpr int kRowsPerBlock = 2;
constexpr int kColsUnroll = 2;

template <typename S>
hipError_t launch_over_cols(hipStream_t stream, const void* T, uint64_t rows, uint64_t cols, uint64_t ld,
                            const uint64_t* eq, uint64_t* partial, Split sp) {
    const bool vec = (reinterpret_cast<uintptr_t>(T) % (2 * sizeof(S)) == 0) && (ld % 2 == 0) &&
                     (sp.per_split % 2 == 0) && (reinterpret_cast<uintptr_t>(eq) % 16 == 0);
    dim3 grid((unsigned)((rows + kRowsPerBlock - 1) / kRowsPerBlock), sp.nsplit);
    if (vec)
        hipLaunchKernelGGL((reduce_over_cols_kernel<S, kRowsPerBlock, kColsUnroll, true>), grid, dim3(kBlock), 0,
                           stream, static_cast<const S*>(T), ld, rows, cols, eq, partial, sp.per_split);
    else
        hipLaunchKernelGGL((reduce_over_cols_kernel<S, kRowsPerBlock, kColsUnroll, false>), grid, dim3(kBlock), 0,
                           stream, static_cast<const S*>(T), ld, rows, cols, eq, partial, sp.per_split);
    return hipGetLastError();
}

// ------------------------------------------------------------------ row-wise reduction of an int8 table
// Reads the weights as they are stored (1 byte per entry instead of 8).  With x' = x + 128 in
// [0, 255] (a sign-bit flip of the byte) the sum over a row is
//     sum_y eq[y] x[y] = sum_y eq[y] x'[y]  -  128 * sum_y eq[y],
// and with eq[y] cut into its eight bytes e_k[y],
//     sum_y eq[y] x'[y] = sum_k 2^(8k) sum_y e_k[y] x'[y].
// The inner sums are sums of byte products, which v_dot4_u32_u8 forms four at a time: one operand is
// a word of the table (four neighbouring columns of a row), the other the word of the eq vector's
// byte planes that holds byte k of the same four columns (see eq_planes_store).  Eight such
// instructions take in four entries: two per entry with nothing to unpack, where 32-bit multiplies
// need a byte extraction and two multiply-adds each.  A lane owns 16 adjacent columns (one 16-byte
// load per row) and keeps their 32 plane words in registers while it walks the R rows of the block,
// so the eq vector costs 128/(16 R) bytes of L2 traffic per byte of table.  The correction term comes
// from the same registers (dot products with a word of ones).  Sums stay in 32-bit registers: a dot
// product adds less than 2^18, and a split is short enough (kI8MaxSplit) for the sum over a whole
// wave to stay below 2^32.  The loads of the next pass are issued before the current one is worked on, so a wave has
// memory requests in flight while it computes.
#ifndef IMM_I8_ROWS
#define IMM_I8_ROWS 8
#endif
#ifndef IMM_I8_MIN_BLOCKS
#define IMM_I8_MIN_BLOCKS 512
#endif
#ifndef IMM_I8_GROUPS
#define IMM_I8_GROUPS 1
#endif
constexpr int kI8Rows = IMM_I8_ROWS;              // rows per block
constexpr int kI8Groups = IMM_I8_GROUPS;          // groups of four columns per lane and pass (4: 16-byte table loads)
constexpr int kI8LaneCols = 4 * kI8Groups;
constexpr uint64_t kI8ColsPerPass = (uint64_t)kI8LaneCols * kBlock;  // columns one block pass covers
constexpr uint64_t kI8MaxSplit = 1ull << 17;      // columns per split: a wave's sum of a plane stays below 2^32

typedef unsigned int v4u32 __attribute__((ext_vector_type(4)));

// value = lo + hi * 2^32 as a canonical residue (any lo, hi)
__device__ __forceinline__ uint64_t combine_limb_sums(uint64_t lo, uint64_t hi) {
    uint64_t low = lo + (hi << 32);
    uint64_t high = (hi >> 32) + (low < lo ? 1 : 0);
    return gl::reduce128(low, high);
}

// sum_k p[k] 2^(8k) for four 32-bit plane sums: below 2^57
__device__ __forceinline__ uint64_t gather_planes(const uint32_t* p) {
    return (uint64_t)p[0] + ((uint64_t)p[1] << 8) + ((uint64_t)p[2] << 16) + ((uint64_t)p[3] << 24);
}

// Sum of a 32-bit value over the 64 lanes of a wave, valid in lane 63 (no overflow check).  Six
// additions whose second operand comes from another lane through the data-parallel-primitive path
// of the vector ALU (shifts by 1, 2, 4, 8 lanes within each row of 16, then the last lane of a row
// into the following row, then lane 31 into the upper half): no trip through the LDS crossbar, whose
// latency a chain of shuffles pays at every step.
[[maybe_unused]] __device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);   // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
    return v;
}

typedef unsigned int i8_words __attribute__((ext_vector_type(kI8Groups)));  // a lane's table bytes of one row
struct I8Pass {
    i8_words x[kI8Rows];
    v4u32 e[2 * kI8Groups];  // plane words of the lane's columns: e[2g] planes 0..3, e[2g+1] planes 4..7 of group g
};

// Zeros to read in place of eq weights where there is nothing left to fetch.  (Not const: a constant
// would live in another address space than the eq vectors, and a load from "one or the other" would
// then be a generic one, which the hardware does not keep in order with the loads from the table.)
__device__ uint64_t zero_words[16];

// `real` false: nothing is left for this lane to fetch; it then reads zeros in place of the plane
// words (and the first bytes of the split, whatever they are), which add nothing to any sum.  So
// the loads of a pass are issued by every lane in every pass, the loop below has one path, and the
// number of requests a wave has in flight at any point is known when the kernel is compiled: the
// wait for the current pass's data then leaves the next pass's requests in flight.  (With a branch
// around the loads the compiler moves them into the branch that uses their data, behind the work on
// the current pass, or has to wait for everything where the paths meet.)
// rowp[r]: start of the split in row r (the same for every lane); off: the lane's column in the split.
__device__ __forceinline__ void i8_load(I8Pass& f, const int8_t* const (&rowp)[kI8Rows], const uint32_t* __restrict__ planes,
                                        uint32_t off, bool real) {
    const uint32_t x_off = real ? off : 0;
#pragma unroll
    for (int r = 0; r < kI8Rows; ++r)
        f.x[r] = __builtin_nontemporal_load(reinterpret_cast<const i8_words*>(rowp[r] + x_off));
    const v4u32* pe = real ? reinterpret_cast<const v4u32*>(planes + 2 * (uint64_t)off)  // 8 words per 4 columns
                           : reinterpret_cast<const v4u32*>(zero_words);
#pragma unroll
    for (int j = 0; j < 2 * kI8Groups; ++j) f.e[j] = pe[j];
}

__device__ __forceinline__ void i8_accumulate(const I8Pass& f, uint32_t (&acc)[kI8Rows][8], uint32_t (&ks)[8]) {
#pragma unroll
    for (int g = 0; g < kI8Groups; ++g) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            ks[k] = __builtin_amdgcn_udot4(0x01010101u, f.e[2 * g][k], ks[k], false);
            ks[4 + k] = __builtin_amdgcn_udot4(0x01010101u, f.e[2 * g + 1][k], ks[4 + k], false);
        }
#pragma unroll
        for (int r = 0; r < kI8Rows; ++r) {
            const uint32_t w = f.x[r][g] ^ 0x80808080u;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                acc[r][k] = __builtin_amdgcn_udot4(w, f.e[2 * g][k], acc[r][k], false);
                acc[r][4 + k] = __builtin_amdgcn_udot4(w, f.e[2 * g + 1][k], acc[r][4 + k], false);
            }
        }
    }
}

// Sums of a wave's plane accumulators, left in out[]: out[2t], out[2t + 1] the sums of the two 32-bit
// limbs of table row t (planes 0..3 and 4..7 gathered), out[2R + k] the wave's sum of plane k of the
// eq weights themselves.  All sums are below 2^32 (kI8MaxSplit).
// With eight rows there are 72 values to add up over 64 lanes.  A butterfly per value is six steps
// each; here the values are first folded onto fewer lanes two at a time -- a swap of the upper half
// of one register with the lower half of another and one addition leave one register holding one
// value's sum over pairs of lanes in its lower half and the other's in its upper half; the same with
// the 16-lane rows -- so that 18 registers are left, each holding four different values, one per row
// of 16 lanes, and only those take the four steps within a row.  Lane 15 of row rho of the wave then
// holds, for t0 = 0, 1, all planes of table row t = 4 (rho >> 1) + 2 (rho & 1) + t0.
__device__ __forceinline__ uint32_t fold_halves(uint32_t lower, uint32_t upper) {
    const auto s = __builtin_amdgcn_permlane32_swap(lower, upper, false, false);
    return s[0] + s[1];  // lanes 0..31: `lower` over lane pairs (l, l + 32); lanes 32..63: `upper` likewise
}
__device__ __forceinline__ uint32_t fold_rows(uint32_t even, uint32_t odd) {
    const auto s = __builtin_amdgcn_permlane16_swap(even, odd, false, false);
    return s[0] + s[1];  // rows 0 and 2: `even` over row pairs (0, 1) and (2, 3); rows 1 and 3: `odd` likewise
}
__device__ __forceinline__ uint32_t row_sum_u32(uint32_t v) {  // valid in the last lane of each row of 16
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);  // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);  // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);  // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);  // row_shr:8
    return v;
}

__device__ __forceinline__ void i8_wave_totals(uint32_t (&acc)[kI8Rows][8], uint32_t (&ks)[8],
                                               uint64_t (&out)[2 * kI8Rows + 8], uint32_t lane) {
    if constexpr (kI8Rows == 8) {
        uint32_t y[2][8], ky[2];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
#pragma unroll
            for (int t0 = 0; t0 < 2; ++t0) {
                const uint32_t x0 = fold_halves(acc[t0][k], acc[t0 + 4][k]);      // table rows t0 | t0 + 4
                const uint32_t x1 = fold_halves(acc[t0 + 2][k], acc[t0 + 6][k]);  // table rows t0 + 2 | t0 + 6
                y[t0][k] = row_sum_u32(fold_rows(x0, x1));  // rows of 16: t0, t0 + 2, t0 + 4, t0 + 6
            }
        }
#pragma unroll
        for (int k0 = 0; k0 < 2; ++k0) {
            const uint32_t x0 = fold_halves(ks[k0], ks[k0 + 4]);
            const uint32_t x1 = fold_halves(ks[k0 + 2], ks[k0 + 6]);
            ky[k0] = row_sum_u32(fold_rows(x0, x1));  // rows of 16: planes k0, k0 + 2, k0 + 4, k0 + 6
        }
        if ((lane & 15) == 15) {
            const uint32_t rho = lane >> 4, base = 4 * (rho >> 1) + 2 * (rho & 1);
#pragma unroll
            for (int t0 = 0; t0 < 2; ++t0) {
                out[2 * (base + t0)] = gather_planes(&y[t0][0]);
                out[2 * (base + t0) + 1] = gather_planes(&y[t0][4]);
                out[2 * kI8Rows + base + t0] = ky[t0];
            }
        }
    } else {
#pragma unroll
        for (int r = 0; r < kI8Rows; ++r)
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[r][k] = wave_sum_u32(acc[r][k]);
#pragma unroll
        for (int k = 0; k < 8; ++k) ks[k] = wave_sum_u32(ks[k]);
        if (lane == 63) {
#pragma unroll
            for (int r = 0; r < kI8Rows; ++r) {
                out[2 * r] = gather_planes(&acc[r][0]);
                out[2 * r + 1] = gather_planes(&acc[r][4]);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) out[2 * kI8Rows + k] = ks[k];
        }
    }
}

__device__ __forceinline__ void reduce_over_cols_i8_block(const int8_t* __restrict__ T, uint64_t ld, uint64_t rows,
                                                          uint64_t cols, const uint32_t* __restrict__ planes,
                                                          uint64_t* __restrict__ partial, uint64_t cols_per_split,
                                                          uint32_t bx, uint32_t by, uint64_t (*lds)[2 * kI8Rows + 8]) {
    constexpr int R = kI8Rows;
    const uint64_t row0 = (uint64_t)bx * R;
    const uint64_t c_begin = (uint64_t)by * cols_per_split;
    uint64_t c_end = c_begin + cols_per_split;
    if (c_end > cols) c_end = cols;

    uint32_t acc[R][8], ks[8];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[r][k] = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) ks[k] = 0;
    // rows past the end of the table are read from the last valid row and dropped at the end
    const int8_t* rowp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) rowp[r] = T + (row0 + r < rows ? row0 + r : rows - 1) * ld + c_begin;
    const uint32_t* split_planes = planes + 2 * c_begin;

    // Every lane runs the same number of passes (where a lane has nothing left, see i8_load).  The data
    // of two passes beyond the current one is on its way at any time -- one pass ahead leaves the
    // 2 x 4 waves that a CU holds of this kernel with too few bytes in flight to keep HBM busy -- so
    // the loop takes three passes per turn, and the one or two left over follow it: their data was
    // asked for in the loop's last turn (or before it).
    const uint32_t span = (uint32_t)(c_end - c_begin);
    const uint32_t passes = (span + (uint32_t)kI8ColsPerPass - 1) / (uint32_t)kI8ColsPerPass;
    constexpr uint32_t kStep = (uint32_t)kI8ColsPerPass;
    uint32_t off = kI8LaneCols * threadIdx.x;
    I8Pass fa, fb, fc;
    i8_load(fa, rowp, split_planes, off, off < span);
    off += kStep;
    i8_load(fb, rowp, split_planes, off, off < span);
    uint32_t pass = 0;
    for (; pass + 2 < passes; pass += 3) {
        off += kStep;
        i8_load(fc, rowp, split_planes, off, off < span);
        loads_stay_above();
        i8_accumulate(fa, acc, ks);
        off += kStep;
        i8_load(fa, rowp, split_planes, off, off < span);
        loads_stay_above();
        i8_accumulate(fb, acc, ks);
        off += kStep;
        i8_load(fb, rowp, split_planes, off, off < span);
        loads_stay_above();
        i8_accumulate(fc, acc, ks);
    }
    if (pass < passes) i8_accumulate(fa, acc, ks);
    if (pass + 1 < passes) i8_accumulate(fb, acc, ks);

    const uint32_t lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    i8_wave_totals(acc, ks, lds[w], lane);
    __syncthreads();
    if (threadIdx.x < R && row0 + threadIdx.x < rows) {
        const int r = threadIdx.x;
        uint64_t a = 0, b = 0, ka = 0, kb = 0;
#pragma unroll
        for (int k = 0; k < kWaves; ++k) {
            a += lds[k][2 * r]; b += lds[k][2 * r + 1];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                ka += lds[k][2 * R + q] << (8 * q);
                kb += lds[k][2 * R + 4 + q] << (8 * q);
            }
        }
        const uint64_t sum = combine_limb_sums(a, b);
        const uint64_t corr = gl::mul(128, combine_limb_sums(ka, kb));
        partial[(uint64_t)by * rows + row0 + r] = gl::sub(sum, corr);
    }
}

__global__ __launch_bounds__(kBlock) void reduce_over_cols_i8_kernel(const int8_t* __restrict__ T, uint64_t ld,
                                                                     uint64_t rows, uint64_t cols,
                                                                     const uint32_t* __restrict__ planes,
                                                                     uint64_t* __restrict__ partial,
                                                                     uint64_t cols_per_split) {
    __shared__ uint64_t lds[kWaves][2 * kI8Rows + 8];
    reduce_over_cols_i8_block(T, ld, rows, cols, planes, partial, cols_per_split, blockIdx.x, blockIdx.y, lds);
}

// The fast int8 kernel needs 16-byte aligned rows and whole groups of a lane's columns.
bool i8_fast_shape(uint64_t cols) { return cols % 16 == 0; }

// ------------------------------------------------------------------ reduction over the rows (column-wise)
// A lane owns two adjacent columns; a block walks the rows of its split, kRowsUnroll rows
// per trip with all loads issued first.  The eq weight of a row is the same for every lane
// (a scalar load).
constexpr int kRowsUnroll = 8;

// The work of workgroup (bx, by) of the grid (column blocks, row splits).  FINISH: the partial
// vectors are handed over as described above and the last workgroup of a column block sums them;
// otherwise they are left for a later launch, and the block has no barriers.
template <typename S, bool VEC, bool FINISH>
__device__ __forceinline__ void reduce_over_rows_block(const S* __restrict__ T, uint64_t ld, uint64_t rows, uint64_t cols,
                                                       const uint64_t* __restrict__ eq, uint64_t* __restrict__ partial,
                                                       uint64_t rows_per_split, uint32_t bx, uint32_t by,
                                                       const Handover& h, uint32_t nsplit, uint32_t* last) {
    const uint64_t r_begin = (uint64_t)by * rows_per_split;
    uint64_t r_end = r_begin + rows_per_split;
    if (r_end > rows) r_end = rows;
    uint64_t* out = partial + (uint64_t)by * cols;
    auto emit = [&](uint64_t j, uint64_t v) {
        if (FINISH) put_word(out + j, v);
        else out[j] = v;
    };
    if (VEC) {
        using Raw = typename RawPair<S>::type;
        const uint64_t col = ((uint64_t)bx * kBlock + threadIdx.x) * 2;
        gl::Acc a0, a1;
        gl::acc_clear(a0);
        gl::acc_clear(a1);
        if (col + 1 < cols) {
            const S* p = T + r_begin * ld + col;
            uint64_t i = r_begin;
            for (; i + kRowsUnroll <= r_end; i += kRowsUnroll, p += kRowsUnroll * ld) {
                Raw x[kRowsUnroll];
                uint64_t ew[kRowsUnroll];
#pragma unroll
                for (int u = 0; u < kRowsUnroll; ++u) x[u] = load_pair<S>(p + u * ld);
#pragma unroll
                for (int u = 0; u < kRowsUnroll; ++u) ew[u] = eq[i + u];
                // keep the loads of a trip together: without this the scheduler sinks each load
                // next to its use and the wave has a single request in flight
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < kRowsUnroll; ++u) {
                    uint64_t e = ew[u], f0, f1;
                    unpack<S>(x[u], f0, f1);
                    gl::acc_mac(a0, f0, e);
                    gl::acc_mac(a1, f1, e);
                }
            }
            for (; i < r_end; ++i, p += ld) {
                uint64_t e = eq[i], f0, f1;
                unpack<S>(load_pair<S>(p), f0, f1);
                gl::acc_mac(a0, f0, e);
                gl::acc_mac(a1, f1, e);
            }
            emit(col, gl::acc_reduce(a0));
            emit(col + 1, gl::acc_reduce(a1));
        } else if (col < cols) {  // last column of an odd-width table
            for (uint64_t i = r_begin; i < r_end; ++i) gl::acc_mac(a0, to_field<S>(T[i * ld + col]), eq[i]);
            emit(col, gl::acc_reduce(a0));
        }
        if (FINISH) sum_by_last_arriver<2>(h, partial, nsplit, cols, bx, by, col, 1, last);
    } else {
        const uint64_t col = (uint64_t)bx * kBlock + threadIdx.x;
        if (col < cols) {
            gl::Acc a0;
            gl::acc_clear(a0);
            for (uint64_t i = r_begin; i < r_end; ++i) gl::acc_mac(a0, to_field<S>(T[i * ld + col]), eq[i]);
            emit(col, gl::acc_reduce(a0));
        }
        if (FINISH) sum_by_last_arriver<1>(h, partial, nsplit, cols, bx, by, col, 1, last);
    }
}

template <typename S, bool VEC>
__global__ __launch_bounds__(kBlock) void reduce_over_rows_kernel(const S* __restrict__ T, uint64_t ld, uint64_t rows,
                                                                  uint64_t cols, const uint64_t* __restrict__ eq,
                                                                  uint64_t* __restrict__ partial,
                                                                  uint64_t rows_per_split) {
    reduce_over_rows_block<S, VEC, false>(T, ld, rows, cols, eq, partial, rows_per_split, blockIdx.x, blockIdx.y,
                                          Handover{}, 0, nullptr);
}

// ------------------------------------------------------------------ column-wise reduction of an int16 table
// Reads the activations as they are stored (2 bytes per entry instead of 8).  With x' = x + 32768 in
// [0, 65535] (a sign-bit flip) the sum over the rows of a split is
//     sum_i eq[i] x[i][j] = sum_i eq[i] x'[i][j]  -  32768 * sum_i eq[i],
// and the products of a 32-bit limb of eq[i] with x' are below 2^48, so a lane adds up to 2^15 of
// them into a plain 64-bit register: two v_mad_u64_u32 per entry, no carries, one modular reduction
// per column at the end.  A lane owns 8 adjacent columns (one 16-byte load per row); the eq weight
// of a row is the same for every lane and comes from a scalar load.  The loads of the next trip of
// kRowsUnroll rows are issued before the current trip is worked on.
constexpr uint64_t kI16MaxSplit = 1ull << 15;  // rows per split: keeps the 64-bit sums below 2^63
constexpr int kI16Cols = 8;                    // columns per lane

__device__ __forceinline__ void i16_load(v4u32 (&x)[kRowsUnroll], const int16_t* p, uint64_t ld) {
#pragma unroll
    for (int u = 0; u < kRowsUnroll; ++u) x[u] = __builtin_nontemporal_load(reinterpret_cast<const v4u32*>(p + u * ld));
}

__device__ __forceinline__ void i16_row(const v4u32& x, uint64_t e, uint64_t (&lo)[kI16Cols], uint64_t (&hi)[kI16Cols],
                                        uint64_t& klo, uint64_t& khi) {
    const uint32_t e0 = (uint32_t)e, e1 = (uint32_t)(e >> 32);
    klo += e0;
    khi += e1;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t w = x[q] ^ 0x80008000u;
        const uint32_t v0 = w & 0xFFFFu, v1 = w >> 16;
        lo[2 * q] += (uint64_t)e0 * v0;
        hi[2 * q] += (uint64_t)e1 * v0;
        lo[2 * q + 1] += (uint64_t)e0 * v1;
        hi[2 * q + 1] += (uint64_t)e1 * v1;
    }
}

// Workgroup (bx, by): 64 lanes x 8 = 512 columns, the rows of split by; its four waves take a quarter
// of those rows each and meet in LDS (wave_sums), so that a launch leaves a quarter of the partial
// vectors it would with one row range per workgroup.
constexpr int kI16BlockCols = 64 * kI16Cols;

template <bool FINISH>
__device__ __forceinline__ void reduce_over_rows_i16_block(const int16_t* __restrict__ T, uint64_t ld, uint64_t rows,
                                                           uint64_t cols, const uint64_t* __restrict__ eq,
                                                           uint64_t* __restrict__ partial, uint64_t rows_per_split,
                                                           uint32_t bx, uint32_t by, const Handover& h, uint32_t nsplit,
                                                           uint32_t* last, uint64_t (*wave_sums)[kI16BlockCols]) {
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // known to be the same for the whole wave
    const uint64_t s_begin = (uint64_t)by * rows_per_split;
    uint64_t s_end = s_begin + rows_per_split;
    if (s_end > rows) s_end = rows;
    uint64_t per_wave = (s_end - s_begin + kWaves - 1) / kWaves;
    per_wave = (per_wave + kRowsUnroll - 1) / kRowsUnroll * kRowsUnroll;
    uint64_t r_begin = s_begin + w * per_wave, r_end = r_begin + per_wave;
    if (r_begin > s_end) r_begin = s_end;
    if (r_end > s_end) r_end = s_end;
    const uint64_t col = (uint64_t)bx * kI16BlockCols + lane * kI16Cols;
    uint64_t lo[kI16Cols], hi[kI16Cols], klo = 0, khi = 0;
#pragma unroll
    for (int c = 0; c < kI16Cols; ++c) lo[c] = hi[c] = 0;
    if (col < cols) {  // cols is a multiple of kI16Cols here
        const int16_t* p = T + r_begin * ld + col;
        uint64_t i = r_begin;
        // Whole trips of kRowsUnroll rows, two per turn of the loop; the loads of the next trip go out
        // before the current one is worked on.  Where there is no next trip the lane reads its first
        // bytes of the table again, with zeros for eq weights (one path through the loop: see i8_load).
        const uint64_t trips = (r_end - r_begin) / kRowsUnroll;
        const int16_t* first_bytes = T + col;
        if (trips) {
            v4u32 xa[kRowsUnroll], xb[kRowsUnroll];
            i16_load(xa, p, ld);
            for (uint64_t t = 0; t < trips; t += 2) {
                const bool next = t + 1 < trips, after = t + 2 < trips;
                i16_load(xb, next ? p + kRowsUnroll * ld : first_bytes, next ? ld : 0);
                loads_stay_above();
#pragma unroll
                for (int u = 0; u < kRowsUnroll; ++u) i16_row(xa[u], eq[i + u], lo, hi, klo, khi);
                i16_load(xa, after ? p + 2 * kRowsUnroll * ld : first_bytes, after ? ld : 0);
                loads_stay_above();
                const uint64_t* eq_next = next ? eq + i + kRowsUnroll : zero_words;
#pragma unroll
                for (int u = 0; u < kRowsUnroll; ++u) i16_row(xb[u], eq_next[u], lo, hi, klo, khi);
                i += 2 * kRowsUnroll;
                p += 2 * kRowsUnroll * ld;
            }
            i = r_begin + trips * kRowsUnroll;
            p = T + i * ld + col;
        }
        for (; i < r_end; ++i, p += ld)
            i16_row(__builtin_nontemporal_load(reinterpret_cast<const v4u32*>(p)), eq[i], lo, hi, klo, khi);
    }
    const uint64_t corr = gl::mul(32768, combine_limb_sums(klo, khi));
#pragma unroll
    for (int c = 0; c < kI16Cols; ++c) wave_sums[w][lane * kI16Cols + c] = gl::sub(combine_limb_sums(lo[c], hi[c]), corr);
    __syncthreads();
    uint64_t* out = partial + (uint64_t)by * cols;
#pragma unroll
    for (int c = 0; c < kI16BlockCols / kBlock; ++c) {
        const uint32_t j = threadIdx.x + c * kBlock;
        const uint64_t jc = (uint64_t)bx * kI16BlockCols + j;
        if (jc < cols) {
            uint64_t v = wave_sums[0][j];
#pragma unroll
            for (int k = 1; k < kWaves; ++k) v = gl::add(v, wave_sums[k][j]);
            if (FINISH) put_word(out + jc, v);
            else out[jc] = v;
        }
    }
    if (FINISH)
        sum_by_last_arriver<kI16BlockCols / kBlock>(h, partial, nsplit, cols, bx, by,
                                                    (uint64_t)bx * kI16BlockCols + threadIdx.x, kBlock, last);
}

__global__ __launch_bounds__(kBlock) void reduce_over_rows_i16_kernel(const int16_t* __restrict__ T, uint64_t ld,
                                                                      uint64_t rows, uint64_t cols,
                                                                      const uint64_t* __restrict__ eq,
                                                                      uint64_t* __restrict__ partial,
                                                                      uint64_t rows_per_split) {
    __shared__ uint64_t wave_sums[kWaves][kI16BlockCols];
    reduce_over_rows_i16_block<false>(T, ld, rows, cols, eq, partial, rows_per_split, blockIdx.x, blockIdx.y, Handover{}, 0,
                                      nullptr, wave_sums);
}

// The fast int16 kernel needs 16-byte rows and whole 8-column groups.
bool i16_fast_shape(const void* T, uint64_t cols, uint64_t ld) {
    return cols % kI16Cols == 0 && ld % kI16Cols == 0 && reinterpret_cast<uintptr_t>(T) % 16 == 0;
}

// ------------------------------------------------------------------ both reductions of a statement in one launch
// The table of A is small next to B's (67 MB against 470 MB at the FFN shape): on its own its kernel
// spends a third of its time filling and draining the machine.  Here the workgroups of the
// row-direction reduction of A come first in the grid of the column-direction reduction of B, so
// they stream alongside it, and the last of them to finish a block of columns sums that block's
// partial vectors while B's reduction is still running.  Only the aligned forms of the operand
// combinations that the prover produces are covered (both widened; int16 activations with widened
// or with int8 weights).
struct ReduceArgs {
    const void* T;
    uint64_t ld, rows, cols;
    const void* eq;  // the eq vector; for an int8 table its byte planes
    uint64_t* partial;
    uint64_t per_split;
    uint32_t grid_x, grid_y;
};

// A_I16: the int16 table of A takes the 8-columns-per-lane kernel (else two columns per lane).
template <typename SA, typename SB, bool A_I16, bool B_IS_I8>
__global__ __launch_bounds__(kBlock) void reduce_both_kernel(ReduceArgs a, Handover ha, ReduceArgs b) {
    __shared__ uint64_t lds[kWaves][2 * kI8Rows + 8];
    __shared__ uint64_t wave_sums[A_I16 ? kWaves : 1][A_I16 ? kI16BlockCols : 1];
    __shared__ uint32_t last;
    const uint32_t a_blocks = a.grid_x * a.grid_y;
    const bool is_a = blockIdx.x < a_blocks;
    const uint32_t a_id = blockIdx.x, b_id = blockIdx.x - a_blocks;
    if (is_a) {
        const uint32_t bx = a_id % a.grid_x, by = a_id / a.grid_x;
        if constexpr (A_I16)
            reduce_over_rows_i16_block<true>(static_cast<const int16_t*>(a.T), a.ld, a.rows, a.cols,
                                             static_cast<const uint64_t*>(a.eq), a.partial, a.per_split, bx, by, ha,
                                             a.grid_y, &last, wave_sums);
        else
            reduce_over_rows_block<SA, true, true>(static_cast<const SA*>(a.T), a.ld, a.rows, a.cols,
                                                   static_cast<const uint64_t*>(a.eq), a.partial, a.per_split, bx, by, ha,
                                                   a.grid_y, &last);
    } else {
        const uint32_t id = b_id;
        if (B_IS_I8)
            reduce_over_cols_i8_block(static_cast<const int8_t*>(b.T), b.ld, b.rows, b.cols,
                                      static_cast<const uint32_t*>(b.eq), b.partial, b.per_split, id % b.grid_x,
                                      id / b.grid_x, lds);
        else
            reduce_over_cols_block<SB, kRowsPerBlock, kColsUnroll, true>(static_cast<const SB*>(b.T), b.ld, b.rows, b.cols,
                                                                         static_cast<const uint64_t*>(b.eq), b.partial,
                                                                         b.per_split, id % b.grid_x, id / b.grid_x,
                                                                         &lds[0][0]);
    }
}

template <typename S>
hipError_t launch_over_rows(hipStream_t stream, const void* T, uint64_t rows, uint64_t cols, uint64_t ld,
                            const uint64_t* eq, uint64_t* partial, Split sp) {
    const bool vec = (reinterpret_cast<uintptr_t>(T) % (2 * sizeof(S)) == 0) && (ld % 2 == 0);
    const uint64_t lanes = vec ? (cols + 1) / 2 : cols;
    dim3 grid((unsigned)((lanes + kBlock - 1) / kBlock), sp.nsplit);
    if (vec)
        hipLaunchKernelGGL((reduce_over_rows_kernel<S, true>), grid, dim3(kBlock), 0, stream, static_cast<const S*>(T),
                           ld, rows, cols, eq, partial, sp.per_split);
    else
        hipLaunchKernelGGL((reduce_over_rows_kernel<S, false>), grid, dim3(kBlock), 0, stream,
                           static_cast<const S*>(T), ld, rows, cols, eq, partial, sp.per_split);
    return hipGetLastError();
}

// words[i] = value, i < count
__global__ __launch_bounds__(kBlock) void fill_words_kernel(uint64_t* __restrict__ words, uint64_t count, uint64_t value) {
    for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += (uint64_t)gridDim.x * kBlock)
        words[i] = value;
}

// ------------------------------------------------------------------ combine / dot
__global__ __launch_bounds__(kBlock) void combine_kernel(const uint64_t* __restrict__ partial, uint32_t nsplit,
                                                         uint64_t len, uint64_t padded, uint64_t* __restrict__ out) {
    __shared__ uint64_t lds[kWaves][64];
    combine_block(partial, nsplit, len, padded, out, blockIdx.x, lds);
}

__global__ __launch_bounds__(kBlock) void dot_kernel(const uint64_t* __restrict__ x, const uint64_t* __restrict__ y,
                                                     uint64_t len, uint64_t* __restrict__ out) {
    __shared__ uint64_t lds[kWaves];
    gl::Acc acc;
    gl::acc_clear(acc);
    for (uint64_t i = threadIdx.x; i < len; i += kBlock) gl::acc_mac(acc, x[i], y[i]);
    uint64_t total = block_sum(gl::acc_reduce(acc), lds);
    if (threadIdx.x == 0) out[0] = total;
}

// ------------------------------------------------------------------ sumcheck round
// FOLD = false: pair (i, i + L/2), i < L/2, of the tables as they are.
// FOLD = true : item i < L/4 reads entries i, i + L/4, i + L/2, i + 3L/4 of each
// table, binds the leading variable (entries i and i + L/4 are rewritten in place;
// no other item touches them) and evaluates the next round's pair (i, i + L/4).
template <bool FOLD>
__global__ __launch_bounds__(kBlock) void round_kernel(uint64_t* __restrict__ a, uint64_t* __restrict__ b, uint64_t L,
                                                       uint64_t r, uint64_t* __restrict__ out /*[gridDim.x][3]*/) {
    __shared__ uint64_t lds[kWaves];
    const uint64_t stride = (uint64_t)gridDim.x * kBlock;
    const uint64_t h = L >> 1;
    uint64_t g0 = 0, g1 = 0, g2 = 0;
    const uint64_t items = FOLD ? (L >> 2) : h;
    const uint64_t q = L >> 2;
    for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < items; i += stride) {
        uint64_t a0, a1, b0, b1;
        if (FOLD) {
            uint64_t x0 = a[i], x1 = a[i + q], x2 = a[i + h], x3 = a[i + h + q];
            uint64_t y0 = b[i], y1 = b[i + q], y2 = b[i + h], y3 = b[i + h + q];
            a0 = gl::add(x0, gl::mul(r, gl::sub(x2, x0)));
            a1 = gl::add(x1, gl::mul(r, gl::sub(x3, x1)));
            b0 = gl::add(y0, gl::mul(r, gl::sub(y2, y0)));
            b1 = gl::add(y1, gl::mul(r, gl::sub(y3, y1)));
            a[i] = a0; a[i + q] = a1;
            b[i] = b0; b[i + q] = b1;
        } else {
            a0 = a[i]; a1 = a[i + h];
            b0 = b[i]; b1 = b[i + h];
        }
        uint64_t a2 = gl::sub(gl::add(a1, a1), a0);  // table value at t = 2: 2*x1 - x0
        uint64_t b2 = gl::sub(gl::add(b1, b1), b0);
        g0 = gl::add(g0, gl::mul(a0, b0));
        g1 = gl::add(g1, gl::mul(a1, b1));
        g2 = gl::add(g2, gl::mul(a2, b2));
    }
    g0 = block_sum(g0, lds);
    g1 = block_sum(g1, lds);
    g2 = block_sum(g2, lds);
    if (threadIdx.x == 0) {
        out[3 * blockIdx.x + 0] = g0;
        out[3 * blockIdx.x + 1] = g1;
        out[3 * blockIdx.x + 2] = g2;
    }
}

// Large tables: the same round with two adjacent items per thread, so that every access is a
// 16-byte one and all eight (four without fold) loads of a trip are in flight together.  The
// upper halves are dead after the fold and are read non-temporally; the lower halves are
// rewritten in place and read again by the next round, so they use ordinary accesses unless
// the tables are far larger than the last-level cache (STREAM), where everything streams.
// The three sums are accumulated lazily and reduced once per thread.
__device__ __forceinline__ v2u64 ld2(const uint64_t* p) { return *reinterpret_cast<const v2u64*>(p); }
__device__ __forceinline__ v2u64 ld2_nt(const uint64_t* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const v2u64*>(p));
}
template <bool STREAM> __device__ __forceinline__ void st2(uint64_t* p, uint64_t x, uint64_t y) {
    v2u64 v;
    v.x = x;
    v.y = y;
    if (STREAM)
        __builtin_nontemporal_store(v, reinterpret_cast<v2u64*>(p));
    else
        *reinterpret_cast<v2u64*>(p) = v;
}
__device__ __forceinline__ uint64_t fold1(uint64_t lo, uint64_t hi, uint64_t r) {
    return gl::add(lo, gl::mul(r, gl::sub(hi, lo)));
}
__device__ __forceinline__ void pair_eval_lazy(gl::Acc& s0, gl::Acc& s1, gl::Acc& s2, uint64_t a0, uint64_t a1,
                                               uint64_t b0, uint64_t b1) {
    gl::acc_mac(s0, a0, b0);
    gl::acc_mac(s1, a1, b1);
    gl::acc_mac(s2, gl::sub(gl::add(a1, a1), a0), gl::sub(gl::add(b1, b1), b0));
}

template <bool FOLD, bool STREAM>
__global__ __launch_bounds__(kBlock) void round_wide_kernel(uint64_t* __restrict__ a, uint64_t* __restrict__ b,
                                                            uint64_t L, uint64_t r,
                                                            uint64_t* __restrict__ out /*[gridDim.x][3]*/) {
    __shared__ uint64_t lds[kWaves];
    const uint64_t stride = (uint64_t)gridDim.x * kBlock;
    const uint64_t h = L >> 1, q = L >> 2;
    const uint64_t pairs = (FOLD ? q : h) >> 1;  // the item count is even here
    gl::Acc s0, s1, s2;
    gl::acc_clear(s0);
    gl::acc_clear(s1);
    gl::acc_clear(s2);
    for (uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x; t < pairs; t += stride) {
        const uint64_t i = 2 * t;
        if (FOLD) {
            v2u64 x0 = STREAM ? ld2_nt(a + i) : ld2(a + i), x1 = STREAM ? ld2_nt(a + i + q) : ld2(a + i + q);
            v2u64 y0 = STREAM ? ld2_nt(b + i) : ld2(b + i), y1 = STREAM ? ld2_nt(b + i + q) : ld2(b + i + q);
            v2u64 x2 = ld2_nt(a + i + h), x3 = ld2_nt(a + i + h + q);
            v2u64 y2 = ld2_nt(b + i + h), y3 = ld2_nt(b + i + h + q);
            __builtin_amdgcn_sched_barrier(0);
            uint64_t a0x = fold1(x0.x, x2.x, r), a0y = fold1(x0.y, x2.y, r);
            uint64_t a1x = fold1(x1.x, x3.x, r), a1y = fold1(x1.y, x3.y, r);
            uint64_t b0x = fold1(y0.x, y2.x, r), b0y = fold1(y0.y, y2.y, r);
            uint64_t b1x = fold1(y1.x, y3.x, r), b1y = fold1(y1.y, y3.y, r);
            st2<STREAM>(a + i, a0x, a0y);
            st2<STREAM>(a + i + q, a1x, a1y);
            st2<STREAM>(b + i, b0x, b0y);
            st2<STREAM>(b + i + q, b1x, b1y);
            pair_eval_lazy(s0, s1, s2, a0x, a1x, b0x, b1x);
            pair_eval_lazy(s0, s1, s2, a0y, a1y, b0y, b1y);
        } else {
            v2u64 x0 = STREAM ? ld2_nt(a + i) : ld2(a + i), x1 = STREAM ? ld2_nt(a + i + h) : ld2(a + i + h);
            v2u64 y0 = STREAM ? ld2_nt(b + i) : ld2(b + i), y1 = STREAM ? ld2_nt(b + i + h) : ld2(b + i + h);
            __builtin_amdgcn_sched_barrier(0);
            pair_eval_lazy(s0, s1, s2, x0.x, x1.x, y0.x, y1.x);
            pair_eval_lazy(s0, s1, s2, x0.y, x1.y, y0.y, y1.y);
        }
    }
    uint64_t g0 = block_sum(gl::acc_reduce(s0), lds);
    uint64_t g1 = block_sum(gl::acc_reduce(s1), lds);
    uint64_t g2 = block_sum(gl::acc_reduce(s2), lds);
    if (threadIdx.x == 0) {
        out[3 * blockIdx.x + 0] = g0;
        out[3 * blockIdx.x + 1] = g1;
        out[3 * blockIdx.x + 2] = g2;
    }
}

__global__ __launch_bounds__(kBlock) void round_finish_kernel(const uint64_t* __restrict__ part, uint32_t nblk,
                                                              uint64_t* __restrict__ out3) {
    __shared__ uint64_t lds[kWaves];
    uint64_t g0 = 0, g1 = 0, g2 = 0;
    for (uint32_t i = threadIdx.x; i < nblk; i += kBlock) {
        g0 = gl::add(g0, part[3 * i]);
        g1 = gl::add(g1, part[3 * i + 1]);
        g2 = gl::add(g2, part[3 * i + 2]);
    }
    g0 = block_sum(g0, lds);
    g1 = block_sum(g1, lds);
    g2 = block_sum(g2, lds);
    if (threadIdx.x == 0) {
        out3[0] = g0; out3[1] = g1; out3[2] = g2;
    }
}

// Last fold (L == 2): one entry per table remains.
__global__ void fold_last_kernel(uint64_t* __restrict__ a, uint64_t* __restrict__ b, uint64_t r,
                                 uint64_t* __restrict__ out3) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    uint64_t va = gl::add(a[0], gl::mul(r, gl::sub(a[1], a[0])));
    uint64_t vb = gl::add(b[0], gl::mul(r, gl::sub(b[1], b[0])));
    a[0] = va;
    b[0] = vb;
    out3[0] = va; out3[1] = vb; out3[2] = 0;
}

// ------------------------------------------------------------------ all rounds in one launch
// One workgroup runs every remaining round of a proof: evaluate g_k(0,1,2), hash it into the
// transcript on the device, squeeze r_k, fold, repeat.  The tables have at most kRoundsMaxL
// entries (they stay L2-resident), so the loop is bound by the three SHA-256 compressions per
// round that lane 0 performs, not by memory; the host is not involved until the final copy.
constexpr int kRoundsBlock = 1024;
constexpr uint64_t kRoundsLdsTable = 4096;  // entries per table that the host-transcript loop keeps in LDS
constexpr uint32_t kRoundsTaskMax = 512;    // longest table whose round is cut into one-multiplication tasks
constexpr int kRoundsWaves = kRoundsBlock / 64;

struct Triple {
    uint64_t g0, g1, g2;
};

__device__ __forceinline__ Triple rounds_block_sum(Triple v, uint64_t (*lds)[3]) {
    v.g0 = wave_sum(v.g0);
    v.g1 = wave_sum(v.g1);
    v.g2 = wave_sum(v.g2);
    if ((threadIdx.x & 63) == 0) {
        lds[threadIdx.x >> 6][0] = v.g0;
        lds[threadIdx.x >> 6][1] = v.g1;
        lds[threadIdx.x >> 6][2] = v.g2;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kRoundsWaves; ++w) {
            v.g0 = gl::add(v.g0, lds[w][0]);
            v.g1 = gl::add(v.g1, lds[w][1]);
            v.g2 = gl::add(v.g2, lds[w][2]);
        }
    }
    return v;  // valid in thread 0
}

__device__ __forceinline__ void pair_eval(Triple& acc, uint64_t a0, uint64_t a1, uint64_t b0, uint64_t b1) {
    uint64_t a2 = gl::sub(gl::add(a1, a1), a0);
    uint64_t b2 = gl::sub(gl::add(b1, b1), b0);
    acc.g0 = gl::add(acc.g0, gl::mul(a0, b0));
    acc.g1 = gl::add(acc.g1, gl::mul(a1, b1));
    acc.g2 = gl::add(acc.g2, gl::mul(a2, b2));
}

__global__ __launch_bounds__(kRoundsBlock) void rounds_kernel(uint64_t* __restrict__ a, uint64_t* __restrict__ b,
                                                             uint64_t L, int rounds, int first_k, int absorb_claim,
                                                             sha::State st_in, uint64_t* __restrict__ words,
                                                             uint32_t* __restrict__ state_out) {
    __shared__ uint64_t lds[kRoundsWaves][3];
    __shared__ uint64_t r_shared;
    const uint32_t tid = threadIdx.x;
    uint32_t s[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) s[i] = st_in.h[i];

    // evaluation of the current tables (no fold yet)
    Triple g = {0, 0, 0};
    {
        const uint64_t h = L >> 1;
        int bad = 0;
        for (uint64_t i = tid; i < h; i += kRoundsBlock) {
            const uint64_t x0 = a[i], x1 = a[i + h], y0 = b[i], y1 = b[i + h];
            bad |= (x0 >= gl::P) | (x1 >= gl::P) | (y0 >= gl::P) | (y1 >= gl::P);
            pair_eval(g, x0, x1, y0, y1);
        }
        if (__syncthreads_or(bad)) {  // the reductions did not deliver canonical field elements
            if (tid == 0) words[kWordVA] = kNoValue;
            return;
        }
    }
    g = rounds_block_sum(g, lds);
    if (tid == 0 && absorb_claim) {
        uint64_t c0 = gl::add(g.g0, g.g1);
        words[kWordC0] = c0;
        sha::absorb_words(s, sha::TAG_CLMC, &c0, 1);
    }

    for (int kk = 0; kk < rounds; ++kk) {
        if (tid == 0) {
            const uint64_t gw[3] = {g.g0, g.g1, g.g2};
            words[kWordG + 3 * (first_k + kk) + 0] = gw[0];
            words[kWordG + 3 * (first_k + kk) + 1] = gw[1];
            words[kWordG + 3 * (first_k + kk) + 2] = gw[2];
            sha::absorb_words(s, sha::TAG_RND, gw, 3);
            const uint64_t r = sha::challenge(s);
            words[kWordR + first_k + kk] = r;
            r_shared = r;
        }
        __syncthreads();
        const uint64_t r = r_shared;
        g = {0, 0, 0};
        const uint64_t h = L >> 1, q = L >> 2;
        if (L == 2) {
            if (tid == 0) {
                g.g0 = gl::add(a[0], gl::mul(r, gl::sub(a[1], a[0])));
                g.g1 = gl::add(b[0], gl::mul(r, gl::sub(b[1], b[0])));
                a[0] = g.g0;
                b[0] = g.g1;
            }
        } else {
            for (uint64_t i = tid; i < q; i += kRoundsBlock) {
                uint64_t x0 = a[i], x1 = a[i + q], x2 = a[i + h], x3 = a[i + h + q];
                uint64_t y0 = b[i], y1 = b[i + q], y2 = b[i + h], y3 = b[i + h + q];
                uint64_t a0 = gl::add(x0, gl::mul(r, gl::sub(x2, x0)));
                uint64_t a1 = gl::add(x1, gl::mul(r, gl::sub(x3, x1)));
                uint64_t b0 = gl::add(y0, gl::mul(r, gl::sub(y2, y0)));
                uint64_t b1 = gl::add(y1, gl::mul(r, gl::sub(y3, y1)));
                a[i] = a0; a[i + q] = a1;
                b[i] = b0; b[i + q] = b1;
                pair_eval(g, a0, a1, b0, b1);
            }
            g = rounds_block_sum(g, lds);  // contains a barrier: the folded entries are visible to the block
        }
        L = h;
        __syncthreads();
    }
    if (tid == 0) {
        // after the last fold g holds (a[0], b[0], -)
        const uint64_t fin[2] = {g.g0, g.g1};
        words[kWordVA] = fin[0];
        words[kWordVB] = fin[1];
        sha::absorb_words(s, sha::TAG_FIN, fin, 2);
#pragma unroll
        for (int i = 0; i < 8; ++i) state_out[i] = s[i];
    }
}

// One challenge from a given state, by the routine the loop above uses (for tests of its rare branch).
__global__ void challenge_kernel(sha::State st_in, uint64_t* __restrict__ value, uint32_t* __restrict__ state_out) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    uint32_t s[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) s[i] = st_in.h[i];
    value[0] = sha::challenge(s);
#pragma unroll
    for (int i = 0; i < 8; ++i) state_out[i] = s[i];
}

// ------------------------------------------------------------------ all rounds in one launch, host hashes
// Same loop as rounds_kernel, but the transcript stays on the host: the workgroup posts g_k into a
// mailbox in pinned host memory and lane 0 polls the slot where the host thread (spinning on the same
// mailbox inside the prove call) deposits r_k: a word of the mailbox, or of a block of device
// memory that the host can write into.  Slots start as kMailEmpty, a value no canonical
// field element can take, so one 8-byte access both signals and carries the value.  The wait is
// bounded: after `spin_limit` polls, or when the host posts kMailAbort, every wave leaves the
// kernel and status[0] is set.
__device__ __forceinline__ void mail_post(uint64_t* slot, uint64_t v) {
    __hip_atomic_store(slot, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
__device__ __forceinline__ uint64_t mail_peek(const uint64_t* slot) {
    return __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// The eq vectors of a proof whose points are not known yet when its kernels are queued: in a chain of
// proofs the points come out of the transcript of the proof before, whose round loop the host is
// still serving.  The kernel is queued behind that loop's kernel and waits (bounded) for the host to
// write the points into `gate`: words rx[0..tA) and ry[0..tB), kMailEmpty until then.  Every word says
// for itself whether it is there, so their order of arrival does not matter.  A word that is not a
// canonical element when the wait ends (never written, or kMailAbort) makes every workgroup leave
// without writing anything; the host, which then knows why, discards what the kernels behind compute.
__global__ __launch_bounds__(kBlock) void eq_build2_gated_kernel(const Gate* __restrict__ gate, uint64_t spin_limit, int tA,
                                                                 uint64_t* __restrict__ outA, int tB,
                                                                 uint64_t* __restrict__ outB,
                                                                 uint32_t* __restrict__ planesB) {
    __shared__ Point ptA, ptB;
    __shared__ int dead;
    const uint32_t tid = threadIdx.x;
    if (tid < 64) {  // lane i < 32 fetches rx[i], lane 32 + i fetches ry[i]
        const uint32_t i = tid & 31;
        const bool second = tid >= 32;
        const bool need = (int)i < (second ? tB : tA);
        const uint64_t* word = second ? &gate->ry[i] : &gate->rx[i];
        uint64_t v = 0;
        if (need) {
            v = kMailEmpty;
            for (uint64_t spin = 0; spin < spin_limit; ++spin) {
                v = mail_peek(word);
                if (v != kMailEmpty) break;
                __builtin_amdgcn_s_sleep(4);
            }
        }
        (second ? ptB : ptA).v[i] = v;
        const int bad = __any(need && v >= gl::P);
        if (tid == 0) dead = bad;
    }
    __syncthreads();
    if (dead) return;
    IMM_EQ_BUILD2_BODY(ptA, tA, outA, ptB, tB, outB, planesB, blockIdx.x);
}

// While the host hashes g_k, the device already prepares round k+1: after the fold with r_k the
// entries are x + r_k dx, so each value g_{k+1}(t) is a quadratic c0 + c1 r_k + c2 r_k^2 whose
// coefficients depend only on the tables as they are now.  The block computes the nine
// coefficients before r_k arrives; when it does, three lanes evaluate one quadratic each and post
// g_{k+1} at once, and the in-place fold runs while the host is busy with g_{k+1}.  The critical
// path of a round is then one host hash and one PCIe round trip.
struct Quad3 {
    uint64_t c[3][3];  // c[t][e]: coefficient of r^e in g(t)
};

__device__ __forceinline__ void quad_accumulate(uint64_t (&c)[3], uint64_t A, uint64_t dA, uint64_t B, uint64_t dB) {
    const uint64_t p0 = gl::mul(A, B), p2 = gl::mul(dA, dB);
    const uint64_t pm = gl::mul(gl::add(A, dA), gl::add(B, dB));  // = p0 + (A dB + dA B) + p2
    c[0] = gl::add(c[0], p0);
    c[1] = gl::add(c[1], gl::sub(gl::sub(pm, p0), p2));
    c[2] = gl::add(c[2], p2);
}

// Sum the nine coefficients over the block into fin9 (visible to all threads on return).  A single wave
// issues an instruction every few nanoseconds, so the reduction is spread out: every thread of
// an active wave drops its nine values into LDS, then wave v adds up column v (one value per
// lane and active wave, then a wave64 shuffle tree), so the nine sums proceed side by side.
__device__ __forceinline__ void quad_block_sum(const Quad3& qd, uint32_t active_waves, uint64_t (*red)[kRoundsBlock],
                                               uint64_t* fin9) {
    const uint32_t tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (w < active_waves) {
#pragma unroll
        for (int t = 0; t < 3; ++t)
#pragma unroll
            for (int e = 0; e < 3; ++e) red[3 * t + e][tid] = qd.c[t][e];
    }
    __syncthreads();
    if (w < 9) {
        uint64_t v = red[w][lane];
        for (uint32_t j = 1; j < active_waves; ++j) v = gl::add(v, red[w][lane + 64 * j]);
        v = wave_sum(v);
        if (lane == 0) fin9[w] = v;
    }
    __syncthreads();
}

// The loop for tables that fit into LDS (2 x 4096 entries), which is every table that has not gone
// through the one-launch-per-round prefix.  A round is a chain of dependent steps, and a single wave
// issues an instruction every two to four nanoseconds, so what counts is the number of instructions
// a wave executes between the arrival of r_k and the moment the coefficients of the next message
// are ready.  The work of a round is therefore cut into tasks of one modular multiplication each,
// spread over all 1024 threads:
//   fold tasks     one per table entry: x[j] <- x[j] + r (x[j + h] - x[j]);
//   product tasks  nine per group of four entries (i, i+q, i+h, i+h+q of the folded tables): with
//                  A_t, A_t + dA_t the lower/upper entries seen from evaluation point t = 0, 1, 2
//                  (likewise B), the products A_t B_t, dA_t dB_t and (A_t + dA_t)(B_t + dB_t), whose
//                  sums S0_t, S2_t, Sm_t give g(t) = S0_t + r (Sm_t - S0_t - S2_t) + r^2 S2_t.
// A wave works on one kind of product at a time (task = kind * padded group count + group), adds its
// 64 products by shuffles, and lane 0 adds the sum to the wave's slot of that kind; nine threads
// add the slots up.  The tables never leave LDS; a[0], b[0] go out through the mailbox.
__device__ __forceinline__ void rounds_in_lds(const uint64_t* ga, const uint64_t* gb, uint64_t L0, int first, int rounds,
                                              int tail_rounds, uint64_t fold_r,
                                              Mailbox* mb, const uint64_t* reply, uint64_t spin_limit, uint64_t* status,
                                              uint64_t (*near)[kRoundsLdsTable], uint64_t (*part)[kRoundsWaves],
                                              uint64_t (*red)[kRoundsBlock], uint64_t* fin9, uint64_t (*lds3)[3],
                                              uint64_t* r_shared) {
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // first == 0: the tables come in as they are and round 1 starts here.  first > 0: the loop takes
    // over before round first + 1 from the loop on tables in global memory: the tables there still
    // have 2 L0 entries and are bound to fold_r = r_first on their way into LDS; the message of round
    // first + 1 has gone out already.
    uint32_t L = (uint32_t)L0;
    int bad = 0;  // an entry that is no canonical field element: the reductions did not deliver
    for (uint32_t i = tid; i < L; i += kRoundsBlock) {
        uint64_t x = ga[i], y = gb[i];
        bad |= (x >= gl::P) | (y >= gl::P);
        if (first) {
            x = gl::add(x, gl::mul(fold_r, gl::sub(ga[i + L], x)));
            y = gl::add(y, gl::mul(fold_r, gl::sub(gb[i + L], y)));
        }
        near[0][i] = x;
        near[1][i] = y;
    }
    if (tid < 9 * kRoundsWaves) part[tid / kRoundsWaves][tid % kRoundsWaves] = 0;
    if (__syncthreads_or(bad) && !first) {
        if (tid == 0) {
            for (int t = 0; t < 3; ++t) mail_post(&mb->g[0][t], kMailFail);
            status[0] = 1;
        }
        return;
    }

    if (!first) {  // round 1: plain evaluation of the tables as they are
        Triple g = {0, 0, 0};
        for (uint32_t i = tid; i < (L >> 1); i += kRoundsBlock)
            pair_eval(g, near[0][i], near[0][i + (L >> 1)], near[1][i], near[1][i + (L >> 1)]);
        g = rounds_block_sum(g, lds3);
        if (tid == 0) {
            mail_post(&mb->g[0][0], g.g0);
            mail_post(&mb->g[0][1], g.g1);
            mail_post(&mb->g[0][2], g.g2);
        }
    }

    // Product sums of the message after the next challenge, from tables of length len >= 4.
    // Expects part[][] zeroed and the tables visible; ends with fin9 valid and part[][] zeroed again.
    auto prepare = [&](uint32_t len) {
        const uint32_t h = len >> 1, q = len >> 2;
        const uint32_t qpad = q < 64 ? 64 : q;  // a power of two: one kind of product per wave and trip
        const uint32_t qshift = 31 - __builtin_clz(qpad);
        for (uint32_t task = tid; task < 9 * qpad; task += kRoundsBlock) {
            const uint32_t v = task >> qshift, i = task & (qpad - 1), kind = v / 3, t = v % 3;
            uint64_t val = 0;
            if (i < q) {
                uint64_t lo[2], up[2];  // A_t and A_t + dA_t, then the same for B
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    const uint64_t f0 = near[tb][i], f1 = near[tb][i + q], f2 = near[tb][i + h], f3 = near[tb][i + h + q];
                    lo[tb] = t == 0 ? f0 : t == 1 ? f1 : gl::sub(gl::add(f1, f1), f0);
                    up[tb] = t == 0 ? f2 : t == 1 ? f3 : gl::sub(gl::add(f3, f3), f2);
                }
                const uint64_t x = kind == 0 ? lo[0] : kind == 2 ? up[0] : gl::sub(up[0], lo[0]);
                const uint64_t y = kind == 0 ? lo[1] : kind == 2 ? up[1] : gl::sub(up[1], lo[1]);
                val = gl::mul(x, y);
            }
            val = wave_sum(val);
            if (lane == 0) part[v][wave] = gl::add(part[v][wave], val);
        }
        __syncthreads();
        if (tid < 192) {  // three whole waves: 16 neighbouring lanes add up the slots of one kind
            const uint32_t v = tid / kRoundsWaves, w = tid % kRoundsWaves;
            uint64_t total = v < 9 ? part[v][w] : 0;
#pragma unroll
            for (int off = kRoundsWaves / 2; off > 0; off >>= 1) total = gl::add(total, __shfl_down(total, off, 64));
            if (v < 9 && w == 0) fin9[v] = total;  // S0_t at t, S2_t at 3 + t, Sm_t at 6 + t
        }
        __syncthreads();
        if (tid < 9 * kRoundsWaves) part[tid / kRoundsWaves][tid % kRoundsWaves] = 0;  // ordered by the next barrier
    };
    // Long tables (more than kRoundsTaskMax entries after the fold) have enough groups of four to keep
    // every thread busy with a whole group: fold its eight entries with r (if `fold`), form the nine
    // products, one reduction of nine values per thread at the end.  Fewer instructions in total, a
    // longer chain per thread; below that length the chain is what costs, above it the total.
    auto prepare_by_groups = [&](uint32_t len, bool fold, uint64_t r) {
        const uint32_t h = len >> 1, q = len >> 2;
        Quad3 sums;
#pragma unroll
        for (int kind = 0; kind < 3; ++kind) sums.c[kind][0] = sums.c[kind][1] = sums.c[kind][2] = 0;
        for (uint32_t i = tid; i < q; i += kRoundsBlock) {
            const uint32_t j[4] = {i, i + q, i + h, i + h + q};
            uint64_t f[2][4];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    uint64_t x = near[tb][j[e]];
                    if (fold) {
                        x = gl::add(x, gl::mul(r, gl::sub(near[tb][j[e] + len], x)));
                        near[tb][j[e]] = x;
                    }
                    f[tb][e] = x;
                }
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                uint64_t lo[2], up[2];
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    lo[tb] = t == 0 ? f[tb][0] : t == 1 ? f[tb][1] : gl::sub(gl::add(f[tb][1], f[tb][1]), f[tb][0]);
                    up[tb] = t == 0 ? f[tb][2] : t == 1 ? f[tb][3] : gl::sub(gl::add(f[tb][3], f[tb][3]), f[tb][2]);
                }
                sums.c[0][t] = gl::add(sums.c[0][t], gl::mul(lo[0], lo[1]));
                sums.c[1][t] = gl::add(sums.c[1][t], gl::mul(gl::sub(up[0], lo[0]), gl::sub(up[1], lo[1])));
                sums.c[2][t] = gl::add(sums.c[2][t], gl::mul(up[0], up[1]));
            }
        }
        const uint32_t active = (q + 63) / 64 < (uint32_t)kRoundsWaves ? (q + 63) / 64 : (uint32_t)kRoundsWaves;
        quad_block_sum(sums, active, red, fin9);  // fin9[3 kind + t]; its barriers also publish the folded entries
    };
    if (L > kRoundsTaskMax) prepare_by_groups(L, false, 0);
    else if (L >= 4) prepare(L);

    const int dev_rounds = rounds - tail_rounds;  // the rounds whose challenge this kernel binds
    for (int kk = first; kk < dev_rounds; ++kk) {
        const uint32_t h = L >> 1;
        // Wave 0: lane 0 waits for r_{kk+1}; lanes 0..2 then evaluate one value each of g_{kk+2} and
        // post it to the host before the tables are touched.
        if (tid < 64) {
            uint64_t r = kMailEmpty;
            if (tid == 0)
                for (uint64_t spin = 0; spin < spin_limit; ++spin) {
                    r = mail_peek(&reply[kk]);
                    if (r != kMailEmpty) break;
                }
            r = __shfl(r, 0, 64);
            if (r < gl::P && L >= 4 && tid < 3) {
                const uint64_t s0 = fin9[tid], s2 = fin9[3 + tid], sm = fin9[6 + tid];
                const uint64_t c1 = gl::sub(gl::sub(sm, s0), s2);
                mail_post(&mb->g[kk + 1][tid], gl::add(s0, gl::mul(r, gl::add(c1, gl::mul(r, s2)))));
            }
            if (tid == 0) *r_shared = r;
        }
        __syncthreads();
        const uint64_t r = *r_shared;
        if (r >= gl::P) {  // no answer within the limit, or the host gave up: uniform exit
            if (tid == 0) status[0] = 1;
            return;
        }
        if (h > kRoundsTaskMax) {
            prepare_by_groups(h, true, r);
            L = h;
            continue;
        }
        // bind the leading variable, one entry per task: entries h .. 2h-1 are only read
        for (uint32_t task = tid; task < 2 * h; task += kRoundsBlock) {
            const uint32_t tb = task >= h ? 1 : 0, j = task - tb * h;
            const uint64_t x = near[tb][j];
            near[tb][j] = gl::add(x, gl::mul(r, gl::sub(near[tb][j + h], x)));
        }
        __syncthreads();
        L = h;
        if (L >= 4 && kk + 1 < dev_rounds) prepare(L);
    }
    if (tail_rounds) {  // the host finishes: it gets the tables as they are now, 2^tail_rounds entries each
        for (uint32_t i = tid; i < 2 * L; i += kRoundsBlock) mail_post(&mb->tail[i >= L ? 1 : 0][i >= L ? i - L : i], near[i >= L ? 1 : 0][i >= L ? i - L : i]);
        if (tid == 0) status[0] = 0;
        return;
    }
    if (tid == 0) {
        mail_post(&mb->fin[0], near[0][0]);
        mail_post(&mb->fin[1], near[1][0]);
        status[0] = 0;
    }
}

// One workgroup per proof: independent proofs run their round loops side by side, each with its
// own tables and mailbox, while one host thread serves all mailboxes in turn.
__global__ __launch_bounds__(kRoundsBlock) void rounds_mailbox_kernel(RoundsJobs jobs, Mailbox* mailboxes,
                                                                     const uint64_t* replies, uint64_t spin_limit,
                                                                     uint64_t* __restrict__ status_all) {
    uint64_t* a = jobs.job[blockIdx.x].a;
    uint64_t* b = jobs.job[blockIdx.x].b;
    uint64_t L = jobs.job[blockIdx.x].L;
    const int rounds = jobs.job[blockIdx.x].rounds;
    const int tail_rounds = jobs.job[blockIdx.x].tail_rounds;
    Mailbox* mb = mailboxes + blockIdx.x;
    const uint64_t* reply = replies ? replies + (uint64_t)blockIdx.x * IMM_MAX_ROUNDS : mb->r;
    uint64_t* status = status_all + blockIdx.x;
    __shared__ uint64_t lds3[kRoundsWaves][3];
    __shared__ uint64_t red[9][kRoundsBlock];  // 72 KiB of the CU's 160 KiB
    __shared__ uint64_t fin9[9];
    __shared__ uint64_t r_shared;
    __shared__ uint64_t near[2][kRoundsLdsTable];  // 64 KiB: tables short enough live here from the start
    __shared__ uint64_t part[9][kRoundsWaves];
    const uint32_t tid = threadIdx.x;

    if (L <= kRoundsLdsTable) {  // the usual case: tables of at most 4096 entries
        rounds_in_lds(a, b, L, 0, rounds, tail_rounds, 0, mb, reply, spin_limit, status, near, part, red, fin9, lds3, &r_shared);
        return;
    }

    // Longer tables (up to kRoundsMaxL entries, 16-byte aligned) start out in global memory, which for one
    // workgroup means: every trip to memory costs a microsecond or two whatever it fetches.  So a thread
    // asks for everything a trip needs at once, as 16-byte accesses (two neighbouring groups of four
    // entries per table), before it computes or stores anything, and round 1 and the coefficients of
    // round 2 come out of one pass over the tables.
    auto clear = [](Quad3& qd) {
#pragma unroll
        for (int t = 0; t < 3; ++t) qd.c[t][0] = qd.c[t][1] = qd.c[t][2] = 0;
    };
    auto accumulate = [](Quad3& qd, uint64_t x0, uint64_t x1, uint64_t xh0, uint64_t xh1, uint64_t y0, uint64_t y1,
                         uint64_t yh0, uint64_t yh1) {
        const uint64_t dx0 = gl::sub(xh0, x0), dx1 = gl::sub(xh1, x1), dy0 = gl::sub(yh0, y0), dy1 = gl::sub(yh1, y1);
        quad_accumulate(qd.c[0], x0, dx0, y0, dy0);
        quad_accumulate(qd.c[1], x1, dx1, y1, dy1);
        quad_accumulate(qd.c[2], gl::sub(gl::add(x1, x1), x0), gl::sub(gl::add(dx1, dx1), dx0),
                        gl::sub(gl::add(y1, y1), y0), gl::sub(gl::add(dy1, dy1), dy0));
    };
    auto waves_for = [](uint64_t items) {
        return (uint32_t)((items + 63) / 64 < kRoundsWaves ? (items + 63) / 64 : kRoundsWaves);
    };
    auto pair_at = [](const uint64_t* p) { return *reinterpret_cast<const v2u64*>(p); };
    auto pair_to = [](uint64_t* p, uint64_t x, uint64_t y) {
        v2u64 v;
        v.x = x;
        v.y = y;
        *reinterpret_cast<v2u64*>(p) = v;
    };

    // The coefficients of g_2(t) as polynomials in r_1: a thread takes the groups i, i + 1 (entries i,
    // i + q, i + h, i + h + q of each table).  Round 1 needs no pass of its own: g_1(r) = g_2(0) + g_2(1)
    // as polynomials in r, so its three values are those two quadratics at r = 0, 1, 2.
    {
        const uint64_t h = L >> 1, q = L >> 2;  // L > 4096: q is a multiple of 1024
        int bad = 0;
        Quad3 qd;
        clear(qd);
        for (uint64_t i = 2 * (uint64_t)tid; i < q; i += 2 * kRoundsBlock) {
            const v2u64 x0 = pair_at(a + i), x1 = pair_at(a + i + q), x2 = pair_at(a + i + h), x3 = pair_at(a + i + h + q);
            const v2u64 y0 = pair_at(b + i), y1 = pair_at(b + i + q), y2 = pair_at(b + i + h), y3 = pair_at(b + i + h + q);
            __builtin_amdgcn_sched_barrier(0);
            bad |= (x0.x >= gl::P) | (x1.x >= gl::P) | (x2.x >= gl::P) | (x3.x >= gl::P) | (y0.x >= gl::P) | (y1.x >= gl::P) |
                   (y2.x >= gl::P) | (y3.x >= gl::P) | (x0.y >= gl::P) | (x1.y >= gl::P) | (x2.y >= gl::P) | (x3.y >= gl::P) |
                   (y0.y >= gl::P) | (y1.y >= gl::P) | (y2.y >= gl::P) | (y3.y >= gl::P);
            accumulate(qd, x0.x, x1.x, x2.x, x3.x, y0.x, y1.x, y2.x, y3.x);
            accumulate(qd, x0.y, x1.y, x2.y, x3.y, y0.y, y1.y, y2.y, y3.y);
        }
        if (__syncthreads_or(bad)) {  // the reductions did not deliver canonical field elements
            if (tid == 0) {
                for (int t = 0; t < 3; ++t) mail_post(&mb->g[0][t], kMailFail);
                status[0] = 1;
            }
            return;
        }
        quad_block_sum(qd, waves_for(q / 2), red, fin9);
        if (tid < 3) {  // g_1(tid) = sum over t = 0, 1 of c0 + tid c1 + tid^2 c2
            const uint64_t c0 = gl::add(fin9[0], fin9[3]), c1 = gl::add(fin9[1], fin9[4]), c2 = gl::add(fin9[2], fin9[5]);
            const uint64_t r = tid;
            mail_post(&mb->g[0][tid], gl::add(c0, gl::mul(r, gl::add(c1, gl::mul(r, c2)))));
        }
    }

    for (int kk = 0; kk < rounds; ++kk) {
        const uint64_t h = L >> 1;
        // fin9 holds the coefficients of g_{kk+2}.  Wave 0: lane 0 waits for r_{kk+1}; lanes 0..2 then
        // evaluate one value each, g_{kk+2}(t) = c0 + r (c1 + r c2), and post it to the host before the
        // tables are touched.
        if (tid < 64) {
            uint64_t r = kMailEmpty;
            if (tid == 0)
                for (uint64_t spin = 0; spin < spin_limit; ++spin) {
                    r = mail_peek(&reply[kk]);
                    if (r != kMailEmpty) break;
                }
            r = __shfl(r, 0, 64);
            if (r < gl::P && tid < 3)
                mail_post(&mb->g[kk + 1][tid],
                          gl::add(fin9[3 * tid], gl::mul(r, gl::add(fin9[3 * tid + 1], gl::mul(r, fin9[3 * tid + 2])))));
            if (tid == 0) r_shared = r;
        }
        __syncthreads();
        const uint64_t r = r_shared;
        if (r >= gl::P) {  // no answer within the limit, or the host gave up: uniform exit
            if (tid == 0) status[0] = 1;
            return;
        }
        if (h <= kRoundsLdsTable) {  // from here on the tables fit into LDS: the other loop takes over
            rounds_in_lds(a, b, h, kk + 1, rounds, tail_rounds, r, mb, reply, spin_limit, status, near, part, red, fin9,
                          lds3, &r_shared);
            return;
        }
        // Bind the leading variable, x[j] <- x[j] + r (x[j + h] - x[j]), in place: a thread folds exactly
        // the four entries of each table (of two neighbouring groups) that its share of the next
        // coefficients is made of, and accumulates them right away: one pass over the tables and one
        // reduction per round, while the host hashes.  h > 4096 here, so there is always such a round.
        {
            const uint64_t h2 = h >> 1, q2 = h >> 2;
            Quad3 qd;
            clear(qd);
            for (uint64_t i = 2 * (uint64_t)tid; i < q2; i += 2 * kRoundsBlock) {
                const uint64_t j[4] = {i, i + q2, i + h2, i + h2 + q2};
                v2u64 xl[4], xu[4], yl[4], yu[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    xl[e] = pair_at(a + j[e]);
                    xu[e] = pair_at(a + j[e] + h);
                    yl[e] = pair_at(b + j[e]);
                    yu[e] = pair_at(b + j[e] + h);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    xl[e].x = gl::add(xl[e].x, gl::mul(r, gl::sub(xu[e].x, xl[e].x)));
                    xl[e].y = gl::add(xl[e].y, gl::mul(r, gl::sub(xu[e].y, xl[e].y)));
                    yl[e].x = gl::add(yl[e].x, gl::mul(r, gl::sub(yu[e].x, yl[e].x)));
                    yl[e].y = gl::add(yl[e].y, gl::mul(r, gl::sub(yu[e].y, yl[e].y)));
                    pair_to(a + j[e], xl[e].x, xl[e].y);
                    pair_to(b + j[e], yl[e].x, yl[e].y);
                }
                accumulate(qd, xl[0].x, xl[1].x, xl[2].x, xl[3].x, yl[0].x, yl[1].x, yl[2].x, yl[3].x);
                accumulate(qd, xl[0].y, xl[1].y, xl[2].y, xl[3].y, yl[0].y, yl[1].y, yl[2].y, yl[3].y);
            }
            quad_block_sum(qd, waves_for(q2 / 2), red, fin9);  // its barriers also publish the folded entries
        }
        L = h;
    }
    if (tid == 0) {
        mail_post(&mb->fin[0], a[0]);
        mail_post(&mb->fin[1], b[0]);
        status[0] = 0;
    }
}

#ifndef IMM_MAX_ROUND_BLOCKS
#define IMM_MAX_ROUND_BLOCKS 512  // two blocks per CU: mixed read/write streams run best with few, long-lived blocks
#endif
constexpr uint32_t kMaxRoundBlocks = IMM_MAX_ROUND_BLOCKS;
constexpr uint64_t kRoundStreamMinL = 1ull << 24;  // two tables of 128 MiB each: beyond the 256 MB cache
constexpr uint64_t kRoundWideMin = 1ull << 14;  // items from which the two-items-per-thread kernel is used

uint32_t round_blocks(uint64_t items) {
    if (items <= 8192) return 1;  // small tables: one block writes the result itself, no second launch
    const uint64_t threads = items >= kRoundWideMin ? items / 2 : items;
    uint64_t nb = (threads + kBlock - 1) / kBlock;
    if (nb < 1) nb = 1;
    if (nb > kMaxRoundBlocks) nb = kMaxRoundBlocks;
    return (uint32_t)nb;
}

}  // namespace

// ------------------------------------------------------------------ wrappers
hipError_t encode(hipStream_t stream, const void* src, int dtype, uint64_t count, uint64_t* dst) {
    switch (dtype) {
    case IMM_I8: return launch_encode<int8_t>(stream, src, count, dst);
    case IMM_I16: return launch_encode<int16_t>(stream, src, count, dst);
    case IMM_I64: return launch_encode<int64_t>(stream, src, count, dst);
    default: return hipErrorInvalidValue;
    }
}

hipError_t front(hipStream_t stream, const int16_t* A, uint64_t countA, uint64_t* dstA, const int8_t* B, uint64_t countB,
                 uint64_t* dstB, const Point& ptA, int tA, uint64_t* eqA, const Point& ptB, int tB, uint64_t* eqB) {
    FrontArgs f{};
    bool va, vb;
    f.srcA = A; f.dstA = dstA; f.countA = countA;
    f.srcB = B; f.dstB = dstB; f.countB = countB;
    f.eqA = eqA; f.eqB = eqB; f.tA = tA; f.tB = tB;
    f.blocks_eq = (uint32_t)(((1ull << tA) + (1ull << tB) + kBlock - 1) / kBlock);
    f.blocks_A = encode_blocks<int16_t>(A, dstA, countA, &va);
    f.blocks_B = countB ? encode_blocks<int8_t>(B, dstB, countB, &vb) : 0;
    if (!countB) vb = true;
    const dim3 grid(f.blocks_eq + f.blocks_A + f.blocks_B);
    if (va && vb) hipLaunchKernelGGL((front_kernel<true, true>), grid, dim3(kBlock), 0, stream, f, ptA, ptB);
    else if (va) hipLaunchKernelGGL((front_kernel<true, false>), grid, dim3(kBlock), 0, stream, f, ptA, ptB);
    else if (vb) hipLaunchKernelGGL((front_kernel<false, true>), grid, dim3(kBlock), 0, stream, f, ptA, ptB);
    else hipLaunchKernelGGL((front_kernel<false, false>), grid, dim3(kBlock), 0, stream, f, ptA, ptB);
    return hipGetLastError();
}

hipError_t eq_build2(hipStream_t stream, const Point& ptA, int tA, uint64_t* outA, const Point& ptB, int tB,
                     uint64_t* outB, uint32_t* planesB) {
    const uint64_t total = (1ull << tA) + (1ull << tB);
    hipLaunchKernelGGL(eq_build2_kernel, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream, ptA,
                       tA, outA, ptB, tB, outB, planesB);
    return hipGetLastError();
}

hipError_t eq_build2_gated(hipStream_t stream, const Gate* gate, uint64_t spin_limit, int tA, uint64_t* outA, int tB,
                           uint64_t* outB, uint32_t* planesB) {
    const uint64_t total = (1ull << tA) + (1ull << tB);
    hipLaunchKernelGGL(eq_build2_gated_kernel, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream, gate,
                       spin_limit, tA, outA, tB, outB, planesB);
    return hipGetLastError();
}

Split plan_over_rows(uint64_t rows, uint64_t cols) {
    // Aim at 512 blocks of 256 lanes (two per CU; one lane owns two columns), at least 32 rows per block.
    // A block should live long: on a table of 16384 x 4096 field elements blocks of 256 or 512 rows
    // stream at 6.2 to 6.4 TB/s, blocks of 128 rows (twice as many, half as long-lived) at 5.0 TB/s.
    const uint64_t col_blocks = ((cols + 1) / 2 + kBlock - 1) / kBlock;
    uint64_t want = (512 + col_blocks - 1) / col_blocks;
    uint64_t per = (rows + want - 1) / want;
    if (per < 32) per = 32;
    per = (per + kRowsUnroll - 1) / kRowsUnroll * kRowsUnroll;
    if (per > rows) per = rows;
    Split sp;
    sp.per_split = per;
    sp.nsplit = (uint32_t)((rows + per - 1) / per);
    return sp;
}

#ifndef IMM_BESIDE_DIV
#define IMM_BESIDE_DIV 512
#endif
#ifndef IMM_BESIDE_MIN_KB
#define IMM_BESIDE_MIN_KB 128u
#endif
Split plan_over_rows_beside(uint64_t rows, uint64_t cols, size_t elem_bytes, uint64_t other_bytes) {
    // Beside a larger reduction that fills the machine on its own, few long-lived workgroups stream best:
    // each takes about as many bytes as half a CU's share of the other table, at least 128 KiB.
    uint64_t target = other_bytes / IMM_BESIDE_DIV;
    if (target < (IMM_BESIDE_MIN_KB << 10)) target = IMM_BESIDE_MIN_KB << 10;
    const uint64_t block_cols = elem_bytes == 2 ? kI16BlockCols : 2 * kBlock;  // columns of a workgroup
    const uint64_t width = cols < block_cols ? cols : block_cols;
    uint64_t per = target / (width * elem_bytes);
    if (per < 32) per = 32;
    per = (per + kRowsUnroll - 1) / kRowsUnroll * kRowsUnroll;
    if (elem_bytes == 2 && per > kI16MaxSplit) per = kI16MaxSplit;
    if ((rows + per - 1) / per > kHandoverMaxSplits) {  // keep the summing workgroup's share small
        per = (rows + kHandoverMaxSplits - 1) / kHandoverMaxSplits;
        per = (per + kRowsUnroll - 1) / kRowsUnroll * kRowsUnroll;
    }
    if (per > rows) per = rows;
    Split sp;
    sp.per_split = per;
    sp.nsplit = (uint32_t)((rows + per - 1) / per);
    return sp;
}

Split plan_over_cols(uint64_t rows, uint64_t cols, int dtype) {
    Split sp;
    if (dtype == IMM_I8 && i8_fast_shape(cols)) {
        // blocks of kI8Rows rows; split the columns (whole block passes) until there are >= 1024 blocks
        const uint64_t row_blocks = (rows + kI8Rows - 1) / kI8Rows;
        uint64_t want = (IMM_I8_MIN_BLOCKS + row_blocks - 1) / row_blocks;
        uint64_t per = (cols + want - 1) / want;
        per = (per + kI8ColsPerPass - 1) / kI8ColsPerPass * kI8ColsPerPass;
        if (per > kI8MaxSplit) per = kI8MaxSplit;
        sp.per_split = per;
        sp.nsplit = (uint32_t)((cols + per - 1) / per);
        return sp;
    }
    // a block covers kRowsPerBlock rows; split the columns until there are >= 2048 blocks,
    // but keep at least 2048 columns (4 pairs per lane) per split
    const uint64_t row_blocks = (rows + kRowsPerBlock - 1) / kRowsPerBlock;
    uint64_t want = (2048 + row_blocks - 1) / row_blocks;
    uint64_t per = (cols + want - 1) / want;
    if (per < 2048) per = 2048;
    per = (per + 511) / 512 * 512;  // whole block passes, and even
    if (per >= cols) per = (cols + 1) / 2 * 2;
    sp.per_split = per;
    sp.nsplit = (uint32_t)((cols + per - 1) / per);
    return sp;
}

hipError_t reduce_over_rows(hipStream_t stream, const void* T, int dtype, uint64_t rows, uint64_t cols, uint64_t ld,
                            const uint64_t* eq_rows, uint64_t* partial, Split sp) {
    switch (dtype) {
    case IMM_I8: return launch_over_rows<int8_t>(stream, T, rows, cols, ld, eq_rows, partial, sp);
    case IMM_I16:
        if (i16_fast_shape(T, cols, ld) && sp.per_split <= kI16MaxSplit) {
            dim3 grid((unsigned)((cols + kI16BlockCols - 1) / kI16BlockCols), sp.nsplit);
            hipLaunchKernelGGL(reduce_over_rows_i16_kernel, grid, dim3(kBlock), 0, stream, static_cast<const int16_t*>(T),
                               ld, rows, cols, eq_rows, partial, sp.per_split);
            return hipGetLastError();
        }
        return launch_over_rows<int16_t>(stream, T, rows, cols, ld, eq_rows, partial, sp);
    case IMM_I64: return launch_over_rows<int64_t>(stream, T, rows, cols, ld, eq_rows, partial, sp);
    case IMM_F64P: return launch_over_rows<uint64_t>(stream, T, rows, cols, ld, eq_rows, partial, sp);
    default: return hipErrorInvalidValue;
    }
}

static bool i8_fast_launch(const void* T, uint64_t cols, uint64_t ld, const void* planes, Split sp) {
    return planes != nullptr && i8_fast_shape(cols) && sp.per_split % kI8ColsPerPass == 0 && sp.per_split <= kI8MaxSplit &&
           reinterpret_cast<uintptr_t>(T) % 16 == 0 && ld % 16 == 0 && reinterpret_cast<uintptr_t>(planes) % 16 == 0;
}

hipError_t reduce_over_cols(hipStream_t stream, const void* T, int dtype, uint64_t rows, uint64_t cols, uint64_t ld,
                            const uint64_t* eq_cols, const uint32_t* eq_planes, uint64_t* partial, Split sp) {
    switch (dtype) {
    case IMM_I8:
        if (i8_fast_launch(T, cols, ld, eq_planes, sp)) {
            dim3 grid((unsigned)((rows + kI8Rows - 1) / kI8Rows), sp.nsplit);
            hipLaunchKernelGGL(reduce_over_cols_i8_kernel, grid, dim3(kBlock), 0, stream,
                               static_cast<const int8_t*>(T), ld, rows, cols, eq_planes, partial, sp.per_split);
            return hipGetLastError();
        }
        return launch_over_cols<int8_t>(stream, T, rows, cols, ld, eq_cols, partial, sp);
    case IMM_I16: return launch_over_cols<int16_t>(stream, T, rows, cols, ld, eq_cols, partial, sp);
    case IMM_I64: return launch_over_cols<int64_t>(stream, T, rows, cols, ld, eq_cols, partial, sp);
    case IMM_F64P: return launch_over_cols<uint64_t>(stream, T, rows, cols, ld, eq_cols, partial, sp);
    default: return hipErrorInvalidValue;
    }
}

hipError_t reduce_both(hipStream_t stream, const void* A, int dtA, uint64_t rowsA, uint64_t colsA, uint64_t ldA,
                       const uint64_t* eq_rows, uint64_t* partA, Split spA, uint32_t* countersA, uint64_t paddedA,
                       uint64_t* outA, const void* B, int dtB, uint64_t rowsB, uint64_t colsB, uint64_t ldB,
                       const uint64_t* eq_cols, const uint32_t* eq_planes, uint64_t* partB, Split spB, bool* done) {
    *done = false;
    const size_t sa = dtA == IMM_F64P ? 8 : dtA == IMM_I16 ? 2 : 0;
    if (!sa || reinterpret_cast<uintptr_t>(A) % (2 * sa) != 0 || ldA % 2 != 0) return hipSuccess;
    const bool b_wide = dtB == IMM_F64P && reinterpret_cast<uintptr_t>(B) % 16 == 0 && ldB % 2 == 0 &&
                        spB.per_split % 2 == 0 && reinterpret_cast<uintptr_t>(eq_cols) % 16 == 0;
    const bool b_i8 = dtB == IMM_I8 && dtA == IMM_I16 && i8_fast_launch(B, colsB, ldB, eq_planes, spB);
    if (!b_wide && !b_i8) return hipSuccess;
    const bool a_i16 = dtA == IMM_I16 && i16_fast_shape(A, colsA, ldA) && spA.per_split <= kI16MaxSplit;
    const uint64_t block_colsA = a_i16 ? kI16BlockCols : 2 * kBlock;
    ReduceArgs a{A, ldA, rowsA, colsA, eq_rows, partA, spA.per_split,
                 (uint32_t)((colsA + block_colsA - 1) / block_colsA), spA.nsplit};
    if (a.grid_x > kHandoverBlocks) return hipSuccess;
    ReduceArgs b{B, ldB, rowsB, colsB, b_i8 ? static_cast<const void*>(eq_planes) : static_cast<const void*>(eq_cols), partB,
                 spB.per_split,
                 (uint32_t)(b_i8 ? (rowsB + kI8Rows - 1) / kI8Rows : (rowsB + kRowsPerBlock - 1) / kRowsPerBlock),
                 spB.nsplit};
    const Handover ha{countersA, outA, paddedA};
    const uint64_t blocks = (uint64_t)a.grid_x * a.grid_y + (uint64_t)b.grid_x * b.grid_y;
    if (blocks > 0x7FFFFFFFull) return hipSuccess;
    const dim3 grid((unsigned)blocks);
    if (b_i8 && a_i16)
        hipLaunchKernelGGL((reduce_both_kernel<int16_t, int8_t, true, true>), grid, dim3(kBlock), 0, stream, a, ha, b);
    else if (b_i8)
        hipLaunchKernelGGL((reduce_both_kernel<int16_t, int8_t, false, true>), grid, dim3(kBlock), 0, stream, a, ha, b);
    else if (dtA == IMM_F64P)
        hipLaunchKernelGGL((reduce_both_kernel<uint64_t, uint64_t, false, false>), grid, dim3(kBlock), 0, stream, a, ha, b);
    else if (a_i16)
        hipLaunchKernelGGL((reduce_both_kernel<int16_t, uint64_t, true, false>), grid, dim3(kBlock), 0, stream, a, ha, b);
    else
        hipLaunchKernelGGL((reduce_both_kernel<int16_t, uint64_t, false, false>), grid, dim3(kBlock), 0, stream, a, ha, b);
    *done = true;
    return hipGetLastError();
}

hipError_t fill_words(hipStream_t stream, uint64_t* words, uint64_t count, uint64_t value) {
    if (!count) return hipSuccess;
    uint64_t blocks = (count + kBlock - 1) / kBlock;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(fill_words_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, stream, words, count, value);
    return hipGetLastError();
}

hipError_t reduce_over_cols_and_combine(hipStream_t stream, const uint64_t* T, uint64_t rows, uint64_t cols, uint64_t ld,
                                        const uint64_t* eq_cols, uint64_t* out_rows, const uint64_t* cpartial,
                                        uint32_t cnsplit, uint64_t clen, uint64_t cpadded, uint64_t* cout) {
    const bool vec = (reinterpret_cast<uintptr_t>(T) % 16 == 0) && (ld % 2 == 0) && (cols % 2 == 0) &&
                     (reinterpret_cast<uintptr_t>(eq_cols) % 16 == 0);
    const uint32_t cblocks = (uint32_t)((cpadded + 63) / 64);
    const CombineArgs c{cpartial, cnsplit, clen, cpadded, cout};
    dim3 grid((unsigned)((rows + kRowsPerBlock - 1) / kRowsPerBlock) + cblocks);
    if (vec)
        hipLaunchKernelGGL((reduce_over_cols_and_combine_kernel<uint64_t, kRowsPerBlock, kColsUnroll, true>), grid,
                           dim3(kBlock), 0, stream, T, ld, rows, cols, eq_cols, out_rows, c, cblocks);
    else
        hipLaunchKernelGGL((reduce_over_cols_and_combine_kernel<uint64_t, kRowsPerBlock, kColsUnroll, false>), grid,
                           dim3(kBlock), 0, stream, T, ld, rows, cols, eq_cols, out_rows, c, cblocks);
    return hipGetLastError();
}

hipError_t combine(hipStream_t stream, const uint64_t* partial, uint32_t nsplit, uint64_t len, uint64_t padded,
                   uint64_t* out) {
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)((padded + 63) / 64)), dim3(kBlock), 0, stream, partial, nsplit,
                       len, padded, out);
    return hipGetLastError();
}

hipError_t dot(hipStream_t stream, const uint64_t* x, const uint64_t* y, uint64_t len, uint64_t* out) {
    hipLaunchKernelGGL(dot_kernel, dim3(1), dim3(kBlock), 0, stream, x, y, len, out);
    return hipGetLastError();
}

uint64_t round_scratch_words(uint64_t) { return 3ull * kMaxRoundBlocks; }

hipError_t round(hipStream_t stream, uint64_t* a, uint64_t* b, uint64_t L, bool fold, uint64_t r, uint64_t* out3,
                 uint64_t* scratch) {
    if (fold && L == 2) {
        hipLaunchKernelGGL(fold_last_kernel, dim3(1), dim3(64), 0, stream, a, b, r, out3);
        return hipGetLastError();
    }
    const uint64_t items = fold ? L / 4 : L / 2;
    const uint32_t nb = round_blocks(items);
    uint64_t* dst = nb == 1 ? out3 : scratch;
    const bool wide = items >= kRoundWideMin && reinterpret_cast<uintptr_t>(a) % 16 == 0 &&
                      reinterpret_cast<uintptr_t>(b) % 16 == 0;
    const bool streaming = L >= kRoundStreamMinL;
    if (wide && fold && streaming)
        hipLaunchKernelGGL((round_wide_kernel<true, true>), dim3(nb), dim3(kBlock), 0, stream, a, b, L, r, dst);
    else if (wide && fold)
        hipLaunchKernelGGL((round_wide_kernel<true, false>), dim3(nb), dim3(kBlock), 0, stream, a, b, L, r, dst);
    else if (wide && streaming)
        hipLaunchKernelGGL((round_wide_kernel<false, true>), dim3(nb), dim3(kBlock), 0, stream, a, b, L, r, dst);
    else if (wide)
        hipLaunchKernelGGL((round_wide_kernel<false, false>), dim3(nb), dim3(kBlock), 0, stream, a, b, L, r, dst);
    else if (fold)
        hipLaunchKernelGGL((round_kernel<true>), dim3(nb), dim3(kBlock), 0, stream, a, b, L, r, dst);
    else
        hipLaunchKernelGGL((round_kernel<false>), dim3(nb), dim3(kBlock), 0, stream, a, b, L, r, dst);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || nb == 1) return e;
    hipLaunchKernelGGL(round_finish_kernel, dim3(1), dim3(kBlock), 0, stream, scratch, nb, out3);
    return hipGetLastError();
}

hipError_t rounds(hipStream_t stream, uint64_t* a, uint64_t* b, uint64_t L, int nrounds, int first_k, bool absorb_claim,
                  const uint32_t state_in[8], uint64_t* words, uint32_t* state_out) {
    sha::State st;
    for (int i = 0; i < 8; ++i) st.h[i] = state_in[i];
    hipLaunchKernelGGL(rounds_kernel, dim3(1), dim3(kRoundsBlock), 0, stream, a, b, L, nrounds, first_k,
                       absorb_claim ? 1 : 0, st, words, state_out);
    return hipGetLastError();
}

hipError_t challenge_once(hipStream_t stream, const uint32_t state_in[8], uint64_t* value, uint32_t* state_out) {
    sha::State st;
    for (int i = 0; i < 8; ++i) st.h[i] = state_in[i];
    hipLaunchKernelGGL(challenge_kernel, dim3(1), dim3(64), 0, stream, st, value, state_out);
    return hipGetLastError();
}

hipError_t rounds_mailbox(hipStream_t stream, const RoundsJobs& jobs, int count, Mailbox* mailboxes,
                          const uint64_t* replies, uint64_t spin_limit, uint64_t* status) {
    hipLaunchKernelGGL(rounds_mailbox_kernel, dim3((unsigned)count), dim3(kRoundsBlock), 0, stream, jobs, mailboxes,
                       replies, spin_limit, status);
    return hipGetLastError();
}

}  // namespace k
}  // namespace imm
