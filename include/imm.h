/* imm.h -- C ABI of the MI355X matmul-sumcheck prover.
 *
 * What it proves.  The audit step of the paper (section 5.2, item 2 of the VC
 * statement; the call F_theta* inside the VC algorithm of the appendix) has to
 * show that the reference model's continuous transformations -- in practice its
 * matrix products -- were computed from the committed operands.  The paper
 * leaves the (Prove, Vrfy) pair abstract (section 2.2) and uses hash commitments
 * (section 2.1).  This library instantiates Prove for one statement "C = A.B"
 * as a Fiat-Shamir sumcheck over the Goldilocks field p = 2^64 - 2^32 + 1:
 *
 *   C~(rx, ry) = sum_{j in {0,1}^delta} A~(rx, j) * B~(j, ry)
 *
 * A is m x d (int16 activations), B is d x n (int8 weights), C is m x n (int64),
 * all row-major.  mu, delta, nu = ceil(log2) of m, d, n; dimensions are padded
 * to powers of two by virtual zeros.  T~ is the multilinear extension with the
 * FIRST variable bound to the MOST significant index bit.  Signed integers are
 * mapped to x mod p.  Every field element that crosses this interface is the
 * canonical residue in [0, p), stored as a little-endian uint64_t.
 *
 * Transcript (SHA-256): a 32-byte state s.
 *   init      s = SHA256("IMM-FS-v1")
 *   absorb    s = SHA256(s || tag[4] || u64le(len) || data)
 *   challenge for ctr = 0,1,..: h = SHA256(s || "chal" || u32le(ctr));
 *             v = u64le(h[0..8)); accept when v < p and set s = h.
 * Proof schedule: absorb "shap" (m,d,n as 3 x u64le), "comA", "comB", "comC"
 * (the three digests); squeeze rx[mu] then ry[nu]; absorb "clmC" (c0); for each
 * round k = 1..delta absorb "rnd " (g_k(0), g_k(1), g_k(2)) and squeeze r_k;
 * absorb "fin " (vA, vB).
 *
 * Pointers are marked HOST or DEVICE.  The caller owns every buffer it passes;
 * inputs are never modified.  The library allocates device memory only inside an
 * imm_ctx and frees it in imm_ctx_destroy.  `stream` is a hipStream_t passed as
 * void* (NULL = the default stream).  No exception or abort crosses this ABI:
 * every call returns an int, 0 for success / ACCEPT, negative for a usage or
 * runtime error, positive (imm_verify only) for a REJECT reason.
 */
#ifndef IMM_H
#define IMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define IMM_MAX_ROUNDS 32     /* largest supported ceil(log2(dimension)) */
#define IMM_PROOF_VERSION 1u

/* element types of a table handed to the library */
typedef enum imm_dtype {
    IMM_I8 = 1,    /* int8_t  */
    IMM_I16 = 2,   /* int16_t */
    IMM_I64 = 3,   /* int64_t */
    IMM_F64P = 4   /* uint64_t, canonical Goldilocks residue (already encoded) */
} imm_dtype;

/* error codes (negative) */
#define IMM_OK 0
#define IMM_E_NULL (-1)    /* a required pointer is NULL */
#define IMM_E_SHAPE (-2)   /* zero dimension, dimension > 2^IMM_MAX_ROUNDS, ld < cols, bad count */
#define IMM_E_DTYPE (-3)   /* dtype not valid for this argument */
#define IMM_E_NOMEM (-4)   /* device or host allocation failed */
#define IMM_E_HIP (-5)     /* a HIP runtime call failed; see imm_last_error() */
#define IMM_E_STATE (-6)   /* nothing to fetch / context not in the required state */

/* reject reasons (positive, imm_verify only) -- the paper's "output bottom" */
#define IMM_REJ_ROUND_SUM 1  /* g_k(0) + g_k(1) != running claim; round in *fail_round (1-based) */
#define IMM_REJ_FINAL 2      /* last claim != vA * vB */
#define IMM_REJ_OPEN_A 3     /* vA != A~(rx || r) recomputed from the supplied A */
#define IMM_REJ_OPEN_B 4     /* vB != B~(r || ry) */
#define IMM_REJ_OPEN_C 5     /* c0 != C~(rx || ry) */
#define IMM_REJ_COMMIT 6     /* a supplied matrix does not hash to its committed digest */
#define IMM_REJ_FORMAT 7     /* header does not match the shapes, or a word >= p */
#define IMM_REJ_UNOPENED 8   /* no check failed, but A, B or C was not supplied: c0, vA and vB are then not
                                tied to the commitments and a prover could have chosen them freely */

/* Hash commitment of one matrix (paper section 2.1: c = Hash(m); no blinding salt).
 * digest = SHA256("IMM-COMMIT-v1" || u32le(dtype) || u64le(rows) || u64le(cols)
 *                 || leaf_0 || leaf_1 || ...),
 * leaf_t = SHA256 of the t-th 1 MiB slice of the raw row-major little-endian bytes. */
typedef struct imm_commit1 {
    uint8_t digest[32];
    uint64_t rows, cols;
    uint32_t dtype;   /* imm_dtype of the committed raw integers */
    uint32_t _pad;
} imm_commit1;

typedef struct imm_commit {
    imm_commit1 A, B, C;
} imm_commit;

/* One proof.  g[3*(k-1)+t] = g_k(t) for round k = 1..delta, t = 0,1,2; unused
 * entries are zero.  c0 = claimed C~(rx, ry); vA = A~(rx, r); vB = B~(r, ry). */
typedef struct imm_proof {
    uint32_t version, mu, delta, nu;
    uint64_t c0;
    uint64_t vA, vB;
    uint64_t g[3 * IMM_MAX_ROUNDS];
} imm_proof;

/* One statement of a batch (see imm_sumcheck_matmul_prove_batch). */
typedef struct imm_matmul_desc {
    const void* A_dev;  /* DEVICE, m x d row-major, dtype dtA (IMM_I16 or IMM_F64P) */
    const void* B_dev;  /* DEVICE, d x n row-major, dtype dtB (IMM_I8 or IMM_F64P) */
    uint32_t dtA, dtB;
    uint64_t m, d, n;
    const imm_commit* com; /* HOST */
} imm_matmul_desc;

typedef struct imm_ctx imm_ctx; /* opaque; owns device scratch, a pinned staging page, events */

/* Create a context on HIP device `device`.  `scratch_bytes` is a hint: that much
 * device memory is reserved up front (0 = grow on demand; buffers grow, never
 * shrink, so a warm-up call with the largest shapes makes later calls
 * allocation-free).  Errors: IMM_E_NULL, IMM_E_HIP, IMM_E_NOMEM. */
int imm_ctx_create(imm_ctx** out, int device, size_t scratch_bytes);
int imm_ctx_destroy(imm_ctx* ctx);

/* Text of the last HIP/runtime error seen by the calling thread ("" if none). */
const char* imm_last_error(void);

/* Write the initial transcript state SHA256("IMM-FS-v1") into state[32] (HOST). */
int imm_fs_init(uint8_t state[32]);

/* Hash-commit the three matrices of a statement (paper section 2.1 and the model
 * commitment of section 5.4 "Setup").  A, B, C are HOST pointers to row-major
 * int16 / int8 / int64 arrays; any of them may be NULL, in which case that entry
 * of *out is left untouched.  CPU only; not part of the timed prover.
 * Errors: IMM_E_NULL (out), IMM_E_SHAPE. */
int imm_commit_matmul(const int16_t* A, const int8_t* B, const int64_t* C,
                      uint64_t m, uint64_t d, uint64_t n, imm_commit* out);

/* One table to commit from device memory: rows x cols raw integers of type dtype (IMM_I8, IMM_I16
 * or IMM_I64), row-major without gaps between rows, at a 4-byte aligned DEVICE address. */
typedef struct imm_table_desc {
    const void* table_dev;
    uint32_t dtype;
    uint32_t _pad;
    uint64_t rows, cols;
} imm_table_desc;

/* The same commitments as imm_commit_matmul (paper section 2.1; same bytes), for `count` tables that
 * live in device memory: every 1 MiB leaf of every table is hashed by one GPU lane, all in one
 * launch on `stream`; the leaf digests come back to the host, which hashes each table's header and
 * leaf digests into out_host[t] (HOST, count entries).  A hash chain is sequential, so the launch
 * takes about 28 ms however few leaves there are, and as long as they fit the chip's 65536 lanes:
 * it pays from roughly five hundred leaves (half a GiB) on, e.g. the activations and products of
 * all statements of a request at once; for single matrices imm_commit_matmul on the host is faster.
 * Synchronises `stream`.  Errors: IMM_E_NULL, IMM_E_SHAPE (count < 0, a zero or too large
 * dimension, a misaligned address, more than 2^22 leaves in all), IMM_E_DTYPE, IMM_E_NOMEM, IMM_E_HIP. */
int imm_commit_tables_device(imm_ctx* ctx, void* stream, int count, const imm_table_desc* tables,
                             imm_commit1* out_host);

/* Field-encoding pass: dst[i] = src[i] mod p for `count` elements.
 * src: DEVICE, dtype IMM_I8 / IMM_I16 / IMM_I64.  dst: DEVICE, count x uint64_t.
 * Asynchronous on `stream`.  Used to widen weights once at deployment so that
 * proofs can take them as IMM_F64P.  Errors: IMM_E_NULL, IMM_E_DTYPE, IMM_E_HIP. */
int imm_encode(imm_ctx* ctx, void* stream, const void* src_dev, imm_dtype dtype,
               uint64_t count, uint64_t* dst_dev);

/* Multilinear-extension evaluation T~(pt_rows || pt_cols) of a rows x cols table
 * with leading dimension ld (elements).  table_dev: DEVICE, any imm_dtype.
 * pt_rows: HOST, ceil(log2(rows)) canonical field elements (first = row MSB);
 * pt_cols: HOST, ceil(log2(cols)) elements; either may be NULL when its count is 0.
 * *out_host (HOST) receives the canonical value; the call synchronises `stream`.
 * Errors: IMM_E_NULL, IMM_E_SHAPE, IMM_E_DTYPE, IMM_E_NOMEM, IMM_E_HIP. */
int imm_mle_eval(imm_ctx* ctx, void* stream, const void* table_dev, imm_dtype dt,
                 uint64_t rows, uint64_t cols, uint64_t ld,
                 const uint64_t* pt_rows, const uint64_t* pt_cols, uint64_t* out_host);

/* imm_mle_eval for callers that cannot allocate device memory: code under HIP stream capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same value, but no context and no allocation of
 * any kind: the working memory (both eq vectors, the partial evaluations, the per-split partial
 * vectors) is an array of IMM_STATIC_SCRATCH_BYTES that is part of the library's device image, one
 * copy per device, held until the process ends.  Runs on the calling thread's current HIP device,
 * asynchronously on `stream`; the result goes to *out_dev (DEVICE, one word) in stream order and
 * nothing is synchronised.  pt_rows, pt_cols: HOST, read before the call returns.
 * A table whose working memory exceeds the array -- roughly 8 bytes x (2^ceil(log2 rows) +
 * 2^ceil(log2 cols) + 3 x the longer dimension) -- is refused with IMM_E_SHAPE and a text in
 * imm_last_error(); imm_mle_eval takes any size.  All calls on one device share the array: two
 * calls that overlap in time on the same device (different streams or threads) race and must be
 * ordered by the caller.  The array's address is looked up when a context is created on the
 * device, or else by the first call there (which should then come before any stream capture).
 * Errors: IMM_E_NULL, IMM_E_SHAPE, IMM_E_DTYPE, IMM_E_HIP. */
#define IMM_STATIC_SCRATCH_BYTES (8u << 20)
int imm_mle_eval_static(void* stream, const void* table_dev, imm_dtype dt,
                        uint64_t rows, uint64_t cols, uint64_t ld,
                        const uint64_t* pt_rows, const uint64_t* pt_cols, uint64_t* out_dev);

/* Prove C = A.B for one statement (the schedule at the top of this file).
 * A_dev: DEVICE m x d, IMM_I16 or IMM_F64P.  B_dev: DEVICE d x n, IMM_I8 or
 * IMM_F64P.  Raw integer operands are widened into context scratch by the
 * encoding pass first; IMM_F64P operands are streamed as they are.
 * com: HOST, the statement's commitments (only the digests are read).
 * transcript_state: HOST, 32 bytes, in = chained state (imm_fs_init for a fresh
 * transcript), out = state after this proof.  out_host: HOST.
 * c0 is computed as sum_j a[j] b[j], which equals C~(rx, ry) iff C = A.B.
 * Synchronous with respect to out_host; kernels run on `stream`.
 * Errors: IMM_E_NULL, IMM_E_SHAPE, IMM_E_DTYPE, IMM_E_NOMEM, IMM_E_HIP. */
int imm_sumcheck_matmul_prove(imm_ctx* ctx, void* stream,
                              const void* A_dev, imm_dtype dtA,
                              const void* B_dev, imm_dtype dtB,
                              uint64_t m, uint64_t d, uint64_t n,
                              const imm_commit* com,
                              uint8_t transcript_state[32], imm_proof* out_host);

/* `count` proofs in order.  chained = 1: one transcript threads through all of
 * them (proof t+1 starts from the state after proof t), as for the layers of one
 * audited request.  chained = 0: every proof starts from the incoming state, as
 * for independent experts; on return transcript_state holds the state after the
 * LAST proof, and states_out (HOST, count x 32 bytes, may be NULL) receives the
 * state after each proof.  A desc with a zero dimension is IMM_E_SHAPE. */
int imm_sumcheck_matmul_prove_batch(imm_ctx* ctx, void* stream, int count,
                                    const imm_matmul_desc* descs, int chained,
                                    uint8_t transcript_state[32], imm_proof* outs_host,
                                    uint8_t* states_out);

/* One pass of the per-round kernel on caller-owned tables (also the unit that the
 * prover runs delta times).  a_dev, b_dev: DEVICE, L canonical field elements each,
 * L a power of two >= 2, modified in place.  If fold_r is non-NULL (HOST, one field
 * element) the leading variable is first bound to *fold_r:
 *   x[i] <- x[i] + r (x[i + L/2] - x[i]),  i < L/2,
 * and the round polynomial is evaluated on the folded tables of length L/2;
 * otherwise it is evaluated on the tables of length L.  g_host (HOST, 3 words)
 * receives g(0), g(1), g(2); when the evaluated length is 1 it receives
 * (a[0], b[0], 0) instead.  Synchronises `stream`. */
int imm_round_fold_eval(imm_ctx* ctx, void* stream, uint64_t* a_dev, uint64_t* b_dev,
                        uint64_t L, const uint64_t* fold_r, uint64_t g_host[3]);

/* Verify one proof -- CPU only (the paper's Vrfy; anything but 0 is its "bottom").
 * com: HOST; the shapes m, d, n are taken from it.  transcript_in: HOST 32 bytes.
 * A, B, C: HOST raw matrices.  The digests are recomputed and the three openings c0 = C~(rx || ry),
 * vA = A~(rx || r), vB = B~(r || ry) are checked by direct evaluation (this stands in for a
 * polynomial-commitment opening, which hash commitments do not provide).  Returns IMM_OK (ACCEPT) only
 * when all three matrices were supplied and every check passed.  A matrix may be NULL: its digest and
 * opening are then skipped, and when nothing else fails the call returns IMM_REJ_UNOPENED, not
 * ACCEPT -- the sumcheck transcript is consistent, but the skipped openings have to be established by
 * other means (e.g. imm_mle_eval on the device at the points that imm_verify_points returns) before
 * the proof means anything.  transcript_out (HOST, nullable) receives the state after the proof on
 * IMM_OK and on IMM_REJ_UNOPENED; *fail_round (nullable) the failing round of IMM_REJ_ROUND_SUM.
 * Errors: IMM_E_NULL, IMM_E_SHAPE / IMM_E_DTYPE (commitments that do not describe an int16 x int8 ->
 * int64 statement), IMM_E_NOMEM. */
int imm_verify(const imm_commit* com, const uint8_t transcript_in[32], const imm_proof* proof,
               const int16_t* A, const int8_t* B, const int64_t* C,
               uint8_t transcript_out[32], int* fail_round);

/* The points at which a proof's three values are openings, replayed from the transcript (no check
 * of the proof's arithmetic): rx[mu], ry[nu], r[delta] (HOST, IMM_MAX_ROUNDS words each, any may be
 * NULL).  c0 = C~(rx || ry), vA = A~(rx || r), vB = B~(r || ry).  Errors: as imm_verify; a proof whose
 * header or words are malformed gives IMM_REJ_FORMAT. */
int imm_verify_points(const imm_commit* com, const uint8_t transcript_in[32], const imm_proof* proof,
                      uint64_t* rx, uint64_t* ry, uint64_t* r);

/* One challenge squeezed from a transcript state (the rule at the top of this file): state (HOST,
 * 32 bytes) is replaced by the accepted hash, *out (HOST) receives the canonical value. */
int imm_transcript_challenge(uint8_t state[32], uint64_t* out);

/* ---- Logit distances of the audited decision steps ------------------------------------------
 * Beside the matrix products, the audit proof reports how far the deployed logits l_i of each
 * discrete decision step were from the reference logits l*_i (paper section 4.3, logit distance
 * distribution; section 5.3, per-request statistic p(t1); appendix "Optimization: Verification of
 * Top-K", top-K distance).  These calls compute those numbers for T steps over a vocabulary of n
 * entries; logits are float32, row-major with leading dimension ld (elements), resident on the
 * device.  Exponentials are evaluated in float32, every sum is accumulated in float64, results are
 * float64.  Logits must be finite (a masked entry is a large negative number, not -inf).  All three
 * are asynchronous on `stream` except where a HOST result is returned.  They use working memory of
 * the context: calls on one context must not overlap, also not on different streams. */

#define IMM_TOPK_MAX 64 /* largest supported K of imm_topk_distance */

/* tv_out_dev[i] = 1/2 sum_j |p_j - q_j| and kl_out_dev[i] = sum_j p_j (log p_j - log q_j) with
 * p = softmax(logits row i) (deployed) and q = softmax(ref row i) (reference).  Either output may
 * be NULL.  logits_dev, ref_dev: DEVICE float32 T x n; outputs: DEVICE float64[T].
 * Rows that are 16-byte aligned with n a multiple of four take the fast path.
 * Errors: IMM_E_NULL (also: both outputs NULL), IMM_E_SHAPE (T or n zero, ld < n, T >= 2^31,
 * n > 2^30), IMM_E_NOMEM, IMM_E_HIP. */
int imm_ldd_tv_kl(imm_ctx* ctx, void* stream, const float* logits_dev, const float* ref_dev,
                  uint64_t T, uint64_t n, uint64_t ld, double* tv_out_dev, double* kl_out_dev);

/* out_dev[i] = min over l' with Top_K(l') = I_i of ||l' - l_i||_1: the smallest L1 change of row i
 * of logits_dev after which the K recorded indices idx_dev[i*K .. i*K+K) are a valid top-K set
 * (0 iff they already are).  idx_dev: DEVICE int32 T x K, 1 <= K <= IMM_TOPK_MAX, K < n; the
 * indices of a row must be distinct and inside [0, n) -- a row that violates this yields NaN.
 * out_dev: DEVICE float64[T].  Errors: IMM_E_NULL, IMM_E_SHAPE, IMM_E_HIP. */
int imm_topk_distance(imm_ctx* ctx, void* stream, const float* logits_dev, uint64_t T, uint64_t n,
                      uint64_t ld, const int32_t* idx_dev, uint32_t K, double* out_dev);

/* *out_host = |{i < T : dist_dev[i] > t1}| / T, the per-request tail density p(t1).
 * dist_dev: DEVICE float64[T].  Synchronises `stream`.  Errors: IMM_E_NULL, IMM_E_SHAPE, IMM_E_HIP. */
int imm_tail_density(imm_ctx* ctx, void* stream, const double* dist_dev, uint64_t T, double t1,
                     double* out_host);

/* Test/diagnostic access to the intermediates of the most recent single proof of
 * this context: which = 0 eqx (2^mu), 1 eqy (2^nu), 2 a = A~(rx, .) (2^delta),
 * 3 b = B~(., ry) (2^delta), 4 rx, 5 ry, 6 r (the round challenges).  Copies at
 * most `capacity` words to out_host and stores the available count in *count.
 * a and b are snapshots taken before the first fold.  Needs IMM_OPT_DEBUG_SNAPSHOTS
 * set before the proof; IMM_E_STATE otherwise. */
int imm_debug_fetch(imm_ctx* ctx, int which, uint64_t* out_host, uint64_t capacity, uint64_t* count);

/* Test/diagnostic: the same challenge derivation as imm_transcript_challenge, run by one lane of the
 * device (the routine the round kernel uses when the device hashes the transcript).  state: HOST, 32
 * bytes, in/out; *out_host the value.  Synchronises `stream`. */
int imm_debug_device_challenge(imm_ctx* ctx, void* stream, uint8_t state[32], uint64_t* out_host);

/* Context options. */
#define IMM_OPT_DEBUG_SNAPSHOTS 1 /* value != 0: keep the intermediates imm_debug_fetch serves (default 0) */
#define IMM_OPT_WIDEN 2           /* value != 0 (default): raw int8/int16 operands of a proof go through the
                                     encoding pass and are streamed as 8-byte field elements; value 0: the
                                     reductions read the narrow integers directly and encode in registers */
#define IMM_OPT_TRANSCRIPT 3      /* who hashes the round messages while the round kernel runs (default
                                     IMM_TRANSCRIPT_HOST).  IMM_TRANSCRIPT_DEVICE: lane 0 of the round kernel (no host involvement
                                     until the final copy); IMM_TRANSCRIPT_HOST: the calling thread, which
                                     exchanges g_k / r_k with the running kernel through a mailbox in pinned
                                     host memory (lower latency per round; both sides wait with a bound) */
#define IMM_TRANSCRIPT_DEVICE 0
#define IMM_TRANSCRIPT_HOST 1
#define IMM_OPT_SPIN_LIMIT 4      /* host-transcript mode: polls the kernel spends per round waiting for r_k
                                     before it gives up and exits (default 2^21, about four seconds).
                                     imm_ldd_tv_kl: polls a workgroup spends waiting for the merged statistics
                                     of its row (at most 2^15 are used) before it works them out itself; the
                                     results do not depend on it, 0 makes every workgroup do so */
#define IMM_OPT_HOST_WAIT_MS 5    /* host-transcript mode: milliseconds the host waits for a mailbox slot
                                     before it aborts the kernel and returns IMM_E_HIP (default 30000) */
#define IMM_OPT_REPLY_IN_DEVICE_MEMORY 6 /* host-transcript mode: 1 (default) the host writes r_k straight into device
                                     memory, where the kernel polls it locally (needs the device memory mapped
                                     into the host's address space; otherwise, and with 0, r_k goes through the
                                     mailbox in pinned host memory) */
#define IMM_OPT_FUSE_REDUCTIONS 7 /* 1 (default): in narrow-read mode the partial evaluations of A and of B run in
                                     one launch where the operand forms allow it (the workgroup of A's part that
                                     finishes last sums its partial vectors); with widened tables the sum of A's
                                     partial vectors rides in the launch of B's reduction and the widening of two
                                     raw operands shares a launch with the eq vectors; 0: one launch each */
#define IMM_OPT_ENCODE_AHEAD 8    /* 1 (default): in a batch proved one proof after the other, the raw operands of
                                     up to three proofs beyond the current one are widened (IMM_OPT_WIDEN) on a
                                     second stream of the library's own while the current one runs, into a ring
                                     of four pairs of scratch tables; that stream starts after everything queued
                                     on the caller's stream up to that point, so operands only have to be ready
                                     in the caller's stream order, as without it, and no table outlives the call.
                                     0: every proof widens its own operands */
#define IMM_OPT_TIMELINE 9        /* value != 0: the host notes the time (CLOCK_MONOTONIC, ns) at which a proof
                                     passes the points IMM_T_* below; imm_debug_timeline returns the notes of
                                     the most recent proof (default 0) */
#define IMM_OPT_HOST_TAIL 10      /* host-transcript mode: t = value (0..IMM_HOST_TAIL_MAX, default
                                     IMM_HOST_TAIL_DEFAULT).  The round kernel runs the rounds on tables longer than
                                     2^t entries; once a fold leaves 2^t entries it hands the two tables to the host
                                     (2^(t+4) bytes through the mailbox) and ends, and the host, which hashes every
                                     round's message anyway, computes the last t rounds itself: on tables that short
                                     a round's arithmetic takes less time than one message to the device and back.
                                     Same proof bytes for every value; 0: the kernel runs every round.  Statements
                                     with fewer than t + 2 rounds are not split, and where k independent proofs share
                                     a launch (their workgroups side by side, one host thread serving them in turn) t
                                     is lowered by ceil(log2 k).  IMM_E_SHAPE outside the range */
#define IMM_OPT_QUEUE_AHEAD 11    /* chained batches in host-transcript mode: 1 (default) = the kernels of proof p + 1
                                     are queued while the host still serves the round loop of proof p; its eq kernel
                                     waits on the device (bounded by IMM_OPT_SPIN_LIMIT) for the points, which the
                                     host writes to it the moment proof p is finished.  0 = every proof is launched
                                     after the one before it has returned.  Same proof bytes either way.  Not used
                                     while debug snapshots, time marks or kernel profiling are on */
#define IMM_HOST_TAIL_DEFAULT 9
#define IMM_HOST_TAIL_MAX 10
int imm_ctx_set_option(imm_ctx* ctx, int option, int64_t value);

/* Points of a proof on the host's side (IMM_OPT_TIMELINE). */
#define IMM_T_ENTRY 0                /* the call has validated its arguments */
#define IMM_T_HEAD_HASHED 1          /* shapes and commitments absorbed, rx and ry squeezed */
#define IMM_T_FRONT_LAUNCHED 2       /* eq vectors (and the widening, where it shares their launch) queued */
#define IMM_T_REDUCTIONS_LAUNCHED 3  /* both partial evaluations queued */
#define IMM_T_ROUNDS_LAUNCHED 4      /* round kernel queued */
#define IMM_T_FIRST_MESSAGE 5        /* g_1 has arrived in the mailbox */
#define IMM_T_FIRST_CHALLENGE 6      /* r_1 posted */
#define IMM_T_LAST_CHALLENGE 7       /* r_delta posted */
#define IMM_T_FINAL_VALUES 8         /* vA, vB have arrived */
#define IMM_T_EXIT 9                 /* the call is about to return */
#define IMM_T_COUNT 10
/* Copies at most `capacity` notes (ids[i], ns[i]; either may be NULL) of the most recent proof of this
 * context and stores their number in *count.  IMM_E_STATE unless IMM_OPT_TIMELINE is set. */
int imm_debug_timeline(imm_ctx* ctx, uint32_t* ids, uint64_t* ns, uint32_t capacity, uint32_t* count);

/* Per-kernel timing with HIP events on the launch stream.  Kernel ids: */
#define IMM_K_ENCODE_A 0
#define IMM_K_ENCODE_B 1
#define IMM_K_EQ 2
#define IMM_K_REDUCE_A 3   /* partial MLE of A over its rows (column-wise reduction) */
#define IMM_K_REDUCE_B 4   /* partial MLE of B over its columns (row-wise reduction) */
#define IMM_K_ROUND 5      /* evaluate g_k(0,1,2) + fold */
#define IMM_K_COMBINE 6    /* sum of per-split partial vectors */
#define IMM_K_LDD 7        /* TV / KL distances of the logits */
#define IMM_K_TOPK 8       /* top-K distance */
#define IMM_K_COMMIT 9     /* leaf hashing of imm_commit_tables_device */
#define IMM_K_COUNT 10
/* mask: bit k set = time kernel id k (0 = profiling off). */
int imm_ctx_set_profiling(imm_ctx* ctx, uint32_t mask);
/* Sum of durations (ms) and number of launches since the last reset. */
int imm_ctx_kernel_time(imm_ctx* ctx, int kernel_id, uint64_t* launches, double* total_ms);
int imm_ctx_reset_profiling(imm_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* IMM_H */
