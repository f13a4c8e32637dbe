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
// eq_build2(ptA .. eqB), encode(A -> dstA) and, unless countB is 0, encode(B -> dstB) in one launch (countA >= 1).
hipError_t front(hipStream_t stream, const int16_t* A, uint64_t countA, uint64_t* dstA, const int8_t* B, uint64_t countB,
                 uint64_t* dstB, const Point& ptA, int tA, uint64_t* eqA, const Point& ptB, int tB, uint64_t* eqB);

// planesB (nullable, 2^tB x 8 bytes): the second vector once more, cut into bytes -- for every four
// neighbouring entries eight words, word k holding byte k of each of the four -- which is the form the
// reduction of an int8 table along its rows takes it in.
hipError_t eq_build2(hipStream_t stream, const Point& ptA, int tA, uint64_t* outA, const Point& ptB, int tB,
                     uint64_t* outB, uint32_t* planesB);

// The same vectors from points that the host hands over after the launch: the kernel waits, at most
// `spin_limit` polls per word, until the words rx[0..tA), ry[0..tB) of `gate` (device-visible memory,
// preset to kMailEmpty by the host) hold canonical elements.  kMailAbort in a needed word, or a wait that
// runs out, makes the kernel end without writing.
struct Gate {
    uint64_t rx[IMM_MAX_ROUNDS];
    uint64_t ry[IMM_MAX_ROUNDS];
};
hipError_t eq_build2_gated(hipStream_t stream, const Gate* gate, uint64_t spin_limit, int tA, uint64_t* outA, int tB,
                           uint64_t* outB, uint32_t* planesB);

// Geometry of a split reduction: how many partial vectors a launch writes.
struct Split {
    uint32_t nsplit;      // number of partial vectors
    uint64_t per_split;   // rows (or columns) covered by one partial vector
};
Split plan_over_rows(uint64_t rows, uint64_t cols);
// the same for a reduction that shares its launch with a larger one that streams `other_bytes`
Split plan_over_rows_beside(uint64_t rows, uint64_t cols, size_t elem_bytes, uint64_t other_bytes);
Split plan_over_cols(uint64_t rows, uint64_t cols, int dtype);

// partial[s][j] = sum over the rows i of split s of eq[i] * T[i][j]   (j < cols)
hipError_t reduce_over_rows(hipStream_t stream, const void* T, int dtype, uint64_t rows, uint64_t cols, uint64_t ld,
                            const uint64_t* eq_rows, uint64_t* partial, Split sp);

// partial[s][i] = sum over the columns j of split s of eq[j] * T[i][j]   (i < rows)
// eq_planes (nullable): the byte planes of eq_cols as eq_build2 writes them; with them an aligned int8
// table takes the kernel that reads it as stored.
hipError_t reduce_over_cols(hipStream_t stream, const void* T, int dtype, uint64_t rows, uint64_t cols, uint64_t ld,
                            const uint64_t* eq_cols, const uint32_t* eq_planes, uint64_t* partial, Split sp);

// Both reductions of one statement in a single launch, A's workgroups first.  B's part is
// reduce_over_cols(B ...) as above.  A's part writes its partial vectors into partA and the workgroup
// that finishes a block of columns last sums them into outA[0 .. colsA) (outA[colsA .. paddedA) is
// zeroed), so no launch has to follow for A.  For that hand-over partA must hold kNoValue in every word
// and countersA (kHandoverBlocks words) zeros when the launch starts; it leaves both that way.  Covers
// the aligned forms of widened A with widened B, int16 A with widened B and int16 A with int8 B; for
// anything else nothing is launched and *done is false.
constexpr uint32_t kHandoverBlocks = 1024;  // column blocks of A at most
constexpr uint64_t kNoValue = 0xFFFFFFFFFFFFFFFFull;  // an empty word of a partial vector: not a canonical element
hipError_t reduce_both(hipStream_t stream, const void* A, int dtA, uint64_t rowsA, uint64_t colsA, uint64_t ldA,
                       const uint64_t* eq_rows, uint64_t* partA, Split spA, uint32_t* countersA, uint64_t paddedA,
                       uint64_t* outA, const void* B, int dtB, uint64_t rowsB, uint64_t colsB, uint64_t ldB,
                       const uint64_t* eq_cols, const uint32_t* eq_planes, uint64_t* partB, Split spB, bool* done);

// words[0 .. count) = value
hipError_t fill_words(hipStream_t stream, uint64_t* words, uint64_t count, uint64_t value);

// out[j] = sum_s partial[s][j] for j < len, 0 for len <= j < padded
// reduce_over_cols of a table of field elements with a single column split (out_rows[i] for i < rows),
// and in the same launch combine(cpartial, cnsplit, clen, cpadded, cout) of an earlier reduction.
hipError_t reduce_over_cols_and_combine(hipStream_t stream, const uint64_t* T, uint64_t rows, uint64_t cols, uint64_t ld,
                                        const uint64_t* eq_cols, uint64_t* out_rows, const uint64_t* cpartial,
                                        uint32_t cnsplit, uint64_t clen, uint64_t cpadded, uint64_t* cout);

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

// Layout of the device-side proof word buffer written by rounds().
constexpr int kWordC0 = 0, kWordVA = 1, kWordVB = 2, kWordG = 3, kWordR = 3 + 3 * IMM_MAX_ROUNDS;
constexpr int kWordCount = kWordR + IMM_MAX_ROUNDS;
constexpr uint64_t kRoundsMaxL = 1ull << 15;  // longest table the single-workgroup round loop takes

// Run `nrounds` sumcheck rounds (numbered first_k .. first_k + nrounds - 1, 0-based) in one launch
// on tables of length L = 2^nrounds <= kRoundsMaxL, hashing the transcript on the device.
//   state_in : transcript state before the first absorbed message, as the eight big-endian words
//   absorb_claim: the launch also derives c0 = g(0) + g(1), stores it and absorbs it ("clmC")
//   words    : device buffer of kWordCount words (c0, vA, vB, g[], r[])
//   state_out: device buffer of 8 words, the state after the "fin " message
hipError_t rounds(hipStream_t stream, uint64_t* a, uint64_t* b, uint64_t L, int nrounds, int first_k, bool absorb_claim,
                  const uint32_t state_in[8], uint64_t* words, uint32_t* state_out);

// One transcript challenge on the device: value[0] and state_out[0..8) (big-endian words) from state_in.
hipError_t challenge_once(hipStream_t stream, const uint32_t state_in[8], uint64_t* value, uint32_t* state_out);

// Mailbox in pinned, coherent host memory shared by rounds_mailbox() and the host thread that
// hashes the transcript.  Every slot holds kMailEmpty until its owner writes it.
constexpr uint64_t kMailEmpty = 0xFFFFFFFFFFFFFFFFull;  // not a canonical field element
constexpr uint64_t kMailAbort = 0xFFFFFFFFFFFFFFFEull;  // host -> device: stop waiting
constexpr uint64_t kMailFail = 0xFFFFFFFFFFFFFFFDull;   // device -> host, in place of g_1: the tables are not canonical
constexpr int kTailMaxLog2 = IMM_HOST_TAIL_MAX;  // longest tables (2^10 entries) that the device hands to the host to finish
struct Mailbox {
    uint64_t g[IMM_MAX_ROUNDS][4];  // device -> host: g_k(0), g_k(1), g_k(2), unused
    uint64_t r[IMM_MAX_ROUNDS];     // host -> device: r_k
    uint64_t fin[4];                // device -> host: a[0], b[0] after the last fold
    uint64_t tail[2][1 << kTailMaxLog2];  // device -> host: the tables a, b once they are short (see RoundsJob)
};

// The same rounds as rounds(), for up to kRoundsMaxJobs independent proofs in one launch (one
// workgroup each), with the host supplying the challenges: job p talks through mailboxes[p] (a
// device-visible pointer to pinned host memory, slots preset to kMailEmpty).  tables of job p:
// L = 2^rounds <= kRoundsMaxL entries each, folded in place.  Lane 0 of a workgroup waits at most
// `spin_limit` polls per round; status[p] (device memory) becomes 0 on completion and 1 if a wait
// ran out or the host posted kMailAbort.  If `replies` is not null, job p reads r_k from
// replies[p * IMM_MAX_ROUNDS + k] (device memory that the host writes into directly, preset to
// kMailEmpty) instead of from its mailbox: polling local memory costs a fraction of a read over PCIe.
constexpr int kRoundsMaxJobs = 16;
struct RoundsJob {
    uint64_t* a;
    uint64_t* b;
    uint64_t L;
    int rounds;
    // 0: the kernel runs all rounds and posts fin[].  t > 0 (at most kTailMaxLog2, at most rounds - 2): it
    // runs the first rounds - t of them; having bound r_(rounds - t) it has already posted the message of
    // the round after, as always, and now posts the tables, 2^t entries each, into tail[][] and ends: the
    // last t rounds work on tables so short that the host computes them faster than a message goes there
    // and back.
    int tail_rounds;
};
struct RoundsJobs {
    RoundsJob job[kRoundsMaxJobs];
};
hipError_t rounds_mailbox(hipStream_t stream, const RoundsJobs& jobs, int count, Mailbox* mailboxes,
                          const uint64_t* replies, uint64_t spin_limit, uint64_t* status);

}  // namespace k
}  // namespace imm
