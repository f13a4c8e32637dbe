// Host orchestration of the prover: context, scratch buffers, launch sequence,
// transcript glue and proof assembly.  The arithmetic runs in kernels.hip; the
// host only hashes and moves a few words per round.
#include <hip/hip_runtime.h>
#include <mutex>
#include <new>
#include <stdexcept>
#include <emmintrin.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstddef>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/imm.h"
#include "host_field.h"
#include "internal.h"
#include "kernels.h"
#include "commit_leaves.h"
#include "ldd.h"
#include "sha256.h"
#include "transcript.h"

namespace imm {

static thread_local std::string g_last_error;

void set_last_error(const char* text) { g_last_error = text; }

int fail_hip(hipError_t e, const char* what) {
    g_last_error = std::string(what) + ": " + hipGetErrorString(e);
    return IMM_E_HIP;
}

#define IMM_HIP(call)                                       \
    do {                                                    \
        hipError_t e_ = (call);                             \
        if (e_ != hipSuccess) return fail_hip(e_, #call);   \
    } while (0)

// While kernels are queued that wait for this thread (the round loop of one proof with the kernels of
// the next proof behind it), a buffer that has to grow must not be freed on the spot: the kernels in
// flight may still use it, and hipFree waits for the device, which waits for this thread.  Buffers
// that are outgrown meanwhile are parked here and freed once the stream has drained.
static thread_local std::vector<void*>* g_parked = nullptr;

// A device buffer that only grows.
struct DevBuf {
    void* p = nullptr;
    size_t bytes = 0;
    int ensure(size_t need) {
        if (need <= bytes) return IMM_OK;
        if (p && g_parked) {
            g_parked->push_back(p);
            p = nullptr;
            bytes = 0;
        }
        if (p) {
            hipError_t e = hipFree(p);
            p = nullptr;
            bytes = 0;
            if (e != hipSuccess) return fail_hip(e, "hipFree");
        }
        size_t rounded = (need + 255) & ~size_t(255);
        hipError_t e = hipMalloc(&p, rounded);
        if (e != hipSuccess) {
            p = nullptr;
            (void)hipGetLastError();
            g_last_error = "hipMalloc failed";
            return e == hipErrorOutOfMemory ? IMM_E_NOMEM : fail_hip(e, "hipMalloc");
        }
        bytes = rounded;
        return IMM_OK;
    }
    void release() {
        if (p) (void)hipFree(p);
        p = nullptr;
        bytes = 0;
    }
    uint64_t* u64() const { return static_cast<uint64_t*>(p); }
};

struct Profiler {
    static constexpr size_t kPool = 1024;  // event pairs
    uint32_t mask = 0;
    std::vector<hipEvent_t> ev;
    struct Rec { int id; size_t first; bool closed; };  // closed: the second event of the pair is recorded
    std::vector<Rec> recs;
    double total_ms[IMM_K_COUNT] = {};
    uint64_t launches[IMM_K_COUNT] = {};

    bool wants(int id) const { return (mask >> id) & 1u; }
    int begin(int id, hipStream_t s) {
        if (!wants(id)) return IMM_OK;
        if (ev.empty()) {
            ev.resize(2 * kPool);
            // timing only: nothing on the host reads what the kernels wrote when it reads these events, so
            // recording one need not push the caches out to system scope
            for (auto& e : ev) IMM_HIP(hipEventCreateWithFlags(&e, hipEventDisableSystemFence));
        }
        if (recs.size() >= kPool) {
            int rc = flush();
            if (rc) return rc;
        }
        size_t first = 2 * recs.size();
        recs.push_back({id, first, false});
        IMM_HIP(hipEventRecord(ev[first], s));
        return IMM_OK;
    }
    int end(int id, hipStream_t s) {
        if (!wants(id) || recs.empty() || recs.back().id != id) return IMM_OK;
        IMM_HIP(hipEventRecord(ev[recs.back().first + 1], s));
        recs.back().closed = true;
        return IMM_OK;
    }
    void cancel(int id) {  // drops the pair opened by the last begin(id): nothing was launched after all
        if (wants(id) && !recs.empty()) recs.pop_back();
    }
    // Adds up the pairs recorded so far and empties the list, whatever happens: a pair that a failed
    // call left open, or whose events the runtime will not read, is dropped, not kept for the next flush.
    int flush() {
        hipError_t bad = hipSuccess;
        for (const Rec& r : recs) {
            if (!r.closed) continue;
            float ms = 0.f;
            hipError_t e = hipEventSynchronize(ev[r.first + 1]);
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev[r.first], ev[r.first + 1]);
            if (e != hipSuccess) {
                bad = e;
                continue;
            }
            total_ms[r.id] += ms;
            launches[r.id] += 1;
        }
        recs.clear();
        if (bad != hipSuccess) {
            (void)hipGetLastError();
            return fail_hip(bad, "reading the profiling events");
        }
        return IMM_OK;
    }
    void reset() {
        recs.clear();
        for (int i = 0; i < IMM_K_COUNT; ++i) { total_ms[i] = 0; launches[i] = 0; }
    }
    void destroy() {
        for (auto& e : ev) (void)hipEventDestroy(e);
        ev.clear();
    }
};

// Reply slots that the host writes and the round kernel polls: fine-grained device memory, reachable
// from the host through the PCIe aperture when the whole device memory is mapped there.  Blocks are
// handed from context to context and never given back to the runtime while the process lives.
constexpr size_t kGateCount = 2;  // proofs whose points may be outstanding: the one after the current
constexpr size_t kReplyWords = (size_t)k::kRoundsMaxJobs * IMM_MAX_ROUNDS + kGateCount * sizeof(k::Gate) / sizeof(uint64_t);
static std::mutex g_reply_mutex;
static std::vector<std::pair<int, uint64_t*>> g_reply_pool;  // (device, block)

static uint64_t* reply_block_take(int device) {
    {
        std::lock_guard<std::mutex> lock(g_reply_mutex);
        for (size_t i = 0; i < g_reply_pool.size(); ++i)
            if (g_reply_pool[i].first == device) {
                uint64_t* p = g_reply_pool[i].second;
                g_reply_pool.erase(g_reply_pool.begin() + (long)i);
                return p;
            }
    }
    int large_bar = 0;
    if (hipDeviceGetAttribute(&large_bar, hipDeviceAttributeIsLargeBar, device) != hipSuccess || large_bar != 1) {
        (void)hipGetLastError();
        return nullptr;
    }
    void* p = nullptr;
    if (hipExtMallocWithFlags(&p, kReplyWords * sizeof(uint64_t), hipDeviceMallocFinegrained) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    return static_cast<uint64_t*>(p);
}
static void reply_block_give(int device, uint64_t* p) {
    if (!p) return;
    std::lock_guard<std::mutex> lock(g_reply_mutex);
    g_reply_pool.emplace_back(device, p);
}
// A store into device memory from the host: through the aperture, pushed out of the write buffers.
static inline void reply_store(uint64_t* slot, uint64_t v) {
    *reinterpret_cast<volatile uint64_t*>(slot) = v;
    _mm_sfence();
}

}  // namespace imm

struct imm_ctx {
    int device = 0;
    imm::DevBuf eqx, eqy, eqy_planes, a, b, partA, partB, handA, hand_counters, round_scratch, words, snapA, snapB,
        group_tables, ldd_partial, ldd_post, ldd_sum, ldd_arrive, commit_leaves, commit_digests;
    uint64_t* pinned = nullptr;  // host staging, 4 KiB
    imm::k::Mailbox* mailbox = nullptr;  // pinned + coherent, kRoundsMaxJobs of them: g_k out, r_k in
    uint64_t* replies = nullptr;         // host-writable device memory for r_k, or null (then the mailbox carries them)
    imm::k::Gate* gates_pinned = nullptr; // behind the mailboxes: where the points of a proof queued ahead arrive
    bool queue_ahead = true;             // IMM_OPT_QUEUE_AHEAD
    bool reply_in_device_memory = true;
    int transcript_mode = IMM_TRANSCRIPT_HOST;
    uint64_t spin_limit = 1ull << 21;    // device polls per round before giving up (about 2 us each)
    int64_t host_wait_ms = 30000;        // host patience per mailbox slot
    int host_tail = IMM_HOST_TAIL_DEFAULT;  // IMM_OPT_HOST_TAIL: the host computes the rounds on tables of at most 2^9 entries
    imm::Profiler prof;
    bool debug = false;
    bool widen = true;
    bool fuse_reductions = true;
    // Widening of the operands of the proofs to come while the current proof runs (sequences of proofs
    // only): a ring of table pairs, a stream for the encode kernels, one event that lets them start
    // and one per pair that says its tables are written.
    static constexpr int kAheadDepth = 3;  // proofs beyond the current one whose tables may be queued
    static constexpr int kTableSets = kAheadDepth + 1;
    bool encode_ahead = true;
    imm::DevBuf encA[kTableSets], encB[kTableSets];
    int set = 0;                           // the pair the current proof reads
    hipStream_t ahead_stream = nullptr;
    hipEvent_t ahead_go = nullptr, ahead_done[kTableSets] = {};
    struct Ahead {
        imm_matmul_desc ds;
        bool hasA, hasB;
        int set;
    } ahead[kAheadDepth];                  // in proof order; ahead[0] belongs to the proof after the current one
    int ahead_count = 0;
    // host-side time marks of the last proof (IMM_OPT_TIMELINE)
    bool timeline = false;
    int marks = 0;
    uint64_t mark_ns[IMM_T_COUNT * 2] = {};
    uint32_t mark_id[IMM_T_COUNT * 2] = {};
    void mark(uint32_t id) {
        if (!timeline || marks >= IMM_T_COUNT * 2) return;
        mark_ns[marks] = (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
                             std::chrono::steady_clock::now().time_since_epoch()).count();
        mark_id[marks++] = id;
    }
    // intermediates of the last single proof (debug)
    int dbg_mu = -1, dbg_delta = -1, dbg_nu = -1;
    uint64_t dbg_rx[IMM_MAX_ROUNDS], dbg_ry[IMM_MAX_ROUNDS], dbg_r[IMM_MAX_ROUNDS];
};

namespace imm {

// proof words and challenges, the 32-byte state, one status word per concurrent round loop
constexpr size_t kWordsDev = k::kWordCount + 4 + k::kRoundsMaxJobs;

static bool dim_ok(uint64_t v) { return v >= 1 && v <= (1ull << IMM_MAX_ROUNDS); }

static int fetch_words(imm_ctx* ctx, hipStream_t s, const uint64_t* dev, size_t count, uint64_t* host_out) {
    IMM_HIP(hipMemcpyAsync(ctx->pinned, dev, count * sizeof(uint64_t), hipMemcpyDeviceToHost, s));
    IMM_HIP(hipStreamSynchronize(s));
    std::memcpy(host_out, ctx->pinned, count * sizeof(uint64_t));
    return IMM_OK;
}

// eq vectors for the row point (tR coordinates) and the column point (tC); with `planes` the column
// vector also in the byte-plane form the int8 reduction reads (ctx->eqy_planes).
// With `gate` the points are not known yet: the kernel waits for them to arrive there (gate_open).
static int build_eq(imm_ctx* ctx, hipStream_t s, const uint64_t* pr, int tR, const uint64_t* pc, int tC,
                    bool planes = false, const k::Gate* gate = nullptr) {
    int rc;
    if ((rc = ctx->eqx.ensure(sizeof(uint64_t) << tR))) return rc;
    if ((rc = ctx->eqy.ensure(sizeof(uint64_t) << tC))) return rc;
    if (planes && (rc = ctx->eqy_planes.ensure(sizeof(uint64_t) << tC))) return rc;
    uint32_t* planes_dev = planes ? static_cast<uint32_t*>(ctx->eqy_planes.p) : nullptr;
    if ((rc = ctx->prof.begin(IMM_K_EQ, s))) return rc;
    if (gate) {
        IMM_HIP(k::eq_build2_gated(s, gate, ctx->spin_limit, tR, ctx->eqx.u64(), tC, ctx->eqy.u64(), planes_dev));
    } else {
        k::Point a{}, b{};
        for (int i = 0; i < tR; ++i) a.v[i] = pr[i];
        for (int i = 0; i < tC; ++i) b.v[i] = pc[i];
        IMM_HIP(k::eq_build2(s, a, tR, ctx->eqx.u64(), b, tC, ctx->eqy.u64(), planes_dev));
    }
    return ctx->prof.end(IMM_K_EQ, s);
}

// The gate of pipeline slot `slot`: in device memory that the host writes into where there is such
// memory, else in pinned host memory.  Closed = every word kMailEmpty.
static k::Gate* gate_of(imm_ctx* ctx, int slot) {
    if (ctx->reply_in_device_memory && ctx->replies)
        return reinterpret_cast<k::Gate*>(ctx->replies + (size_t)k::kRoundsMaxJobs * IMM_MAX_ROUNDS) + slot;
    return ctx->gates_pinned + slot;
}
static void gate_fill(k::Gate* g, uint64_t value) {
    volatile uint64_t* w = reinterpret_cast<volatile uint64_t*>(g);
    for (size_t i = 0; i < sizeof(k::Gate) / sizeof(uint64_t); ++i) w[i] = value;
    _mm_sfence();
}
static void gate_open(k::Gate* g, const uint64_t* rx, int mu, const uint64_t* ry, int nu) {
    volatile uint64_t* wx = g->rx;
    volatile uint64_t* wy = g->ry;
    for (int i = 0; i < mu; ++i) wx[i] = rx[i];
    for (int i = 0; i < nu; ++i) wy[i] = ry[i];
    _mm_sfence();
}

// Whether the reduction of a table along its rows can read it as int8 (then the eq vector's byte planes are needed).
static bool wants_planes(int dt, uint64_t cols) { return dt == IMM_I8 && cols % 16 == 0; }

// The memory of the hand-over between the workgroups of A's reduction (k::reduce_both): `words` words
// of partial vectors, all holding k::kNoValue, and zeroed counters.  Launches leave it as they found it,
// so it is only written here when it is (re)allocated.
static int ensure_handover(imm_ctx* ctx, hipStream_t s, uint64_t words) {
    int rc;
    if (ctx->handA.bytes < words * sizeof(uint64_t)) {
        if ((rc = ctx->handA.ensure(words * sizeof(uint64_t)))) return rc;
        IMM_HIP(k::fill_words(s, ctx->handA.u64(), ctx->handA.bytes / sizeof(uint64_t), k::kNoValue));
    }
    if (!ctx->hand_counters.p) {
        if ((rc = ctx->hand_counters.ensure(sizeof(uint64_t) * (k::kHandoverBlocks / 2)))) return rc;
        IMM_HIP(k::fill_words(s, ctx->hand_counters.u64(), k::kHandoverBlocks / 2, 0));
    }
    return IMM_OK;
}

// Sum the per-split partial vectors into out[0..len) and zero out[len..padded).  When the
// reduction ran as a single split it already wrote out[0..len) and only the padding is left.
static int finish_partial(imm_ctx* ctx, hipStream_t s, bool direct, DevBuf& part, uint32_t nsplit, uint64_t len,
                          uint64_t padded, uint64_t* out) {
    int rc;
    if (direct && len == padded) return IMM_OK;
    if ((rc = ctx->prof.begin(IMM_K_COMBINE, s))) return rc;
    if (direct)
        IMM_HIP(k::combine(s, nullptr, 0, 0, padded - len, out + len));
    else
        IMM_HIP(k::combine(s, part.u64(), nsplit, len, padded, out));
    return ctx->prof.end(IMM_K_COMBINE, s);
}

// a[j] = sum_i eqx[i] T[i][j] for j < cols, zero up to `padded`.
static int partial_over_rows(imm_ctx* ctx, hipStream_t s, int kid, const void* T, int dt, uint64_t rows, uint64_t cols,
                             uint64_t ld, const uint64_t* eq, uint64_t padded, DevBuf& part, uint64_t* out) {
    int rc;
    k::Split sp = k::plan_over_rows(rows, cols);
    const bool direct = sp.nsplit == 1;  // a single split writes the result vector itself
    if (!direct && (rc = part.ensure(sizeof(uint64_t) * sp.nsplit * cols))) return rc;
    if ((rc = ctx->prof.begin(kid, s))) return rc;
    IMM_HIP(k::reduce_over_rows(s, T, dt, rows, cols, ld, eq, direct ? out : part.u64(), sp));
    if ((rc = ctx->prof.end(kid, s))) return rc;
    return finish_partial(ctx, s, direct, part, sp.nsplit, cols, padded, out);
}

// b[i] = sum_j eqy[j] T[i][j] for i < rows, zero up to `padded`.
static int partial_over_cols(imm_ctx* ctx, hipStream_t s, int kid, const void* T, int dt, uint64_t rows, uint64_t cols,
                             uint64_t ld, const uint64_t* eq, uint64_t padded, DevBuf& part, uint64_t* out) {
    int rc;
    k::Split sp = k::plan_over_cols(rows, cols, dt);
    const bool direct = sp.nsplit == 1;
    if (!direct && (rc = part.ensure(sizeof(uint64_t) * sp.nsplit * rows))) return rc;
    if ((rc = ctx->prof.begin(kid, s))) return rc;
    IMM_HIP(k::reduce_over_cols(s, T, dt, rows, cols, ld, eq,
                                wants_planes(dt, cols) ? static_cast<const uint32_t*>(ctx->eqy_planes.p) : nullptr,
                                direct ? out : part.u64(), sp));
    if ((rc = ctx->prof.end(kid, s))) return rc;
    return finish_partial(ctx, s, direct, part, sp.nsplit, rows, padded, out);
}

static int run_round(imm_ctx* ctx, hipStream_t s, uint64_t* a, uint64_t* b, uint64_t L, bool fold, uint64_t r,
                     uint64_t* out3_dev, uint64_t* host3) {
    int rc;
    if ((rc = ctx->round_scratch.ensure(sizeof(uint64_t) * k::round_scratch_words(L)))) return rc;
    if ((rc = ctx->prof.begin(IMM_K_ROUND, s))) return rc;
    IMM_HIP(k::round(s, a, b, L, fold, r, out3_dev, ctx->round_scratch.u64()));
    if ((rc = ctx->prof.end(IMM_K_ROUND, s))) return rc;
    return fetch_words(ctx, s, out3_dev, 3, host3);
}

// Wait until a mailbox slot written by the device leaves the empty state.
static bool mail_wait(const uint64_t* slot, int64_t patience_ms, uint64_t* value) {
    const volatile uint64_t* p = slot;
    std::chrono::steady_clock::time_point t0;
    for (uint64_t spin = 0;; ++spin) {
        uint64_t v = *p;
        if (v != k::kMailEmpty) {
            std::atomic_thread_fence(std::memory_order_acquire);
            *value = v;
            return true;
        }
        if (spin == 0) t0 = std::chrono::steady_clock::now();  // a word that is there already costs no look at the clock
        if ((spin & 0xFFF) == 0xFFF) {
            auto dt = std::chrono::steady_clock::now() - t0;
            if (std::chrono::duration_cast<std::chrono::milliseconds>(dt).count() > patience_ms) return false;
        }
        __builtin_ia32_pause();
    }
}

// One statement on its way through the prover.
struct Job {
    const imm_matmul_desc* ds = nullptr;
    imm_proof* out = nullptr;
    int mu = 0, delta = 0, nu = 0;
    uint64_t D = 1;
    Transcript tr;
    uint64_t rx[IMM_MAX_ROUNDS] = {}, ry[IMM_MAX_ROUNDS] = {}, rr[IMM_MAX_ROUNDS] = {};
    uint64_t* a = nullptr;  // device tables of length D
    uint64_t* b = nullptr;
    uint64_t L = 1;         // current table length
    int kk = 0;             // rounds already done
    bool claim_absorbed = false;
    explicit Job(const uint8_t state[32]) : tr(state) {}
};

static int check_desc(const imm_matmul_desc& ds) {
    if (!ds.A_dev || !ds.B_dev || !ds.com) return IMM_E_NULL;
    if (!dim_ok(ds.m) || !dim_ok(ds.d) || !dim_ok(ds.n)) return IMM_E_SHAPE;
    if (ds.dtA != IMM_I16 && ds.dtA != IMM_F64P) return IMM_E_DTYPE;
    if (ds.dtB != IMM_I8 && ds.dtB != IMM_F64P) return IMM_E_DTYPE;
    // the commitments must be those of this statement: the verifier takes the shapes from them
    const imm_commit& c = *ds.com;
    if (c.A.rows != ds.m || c.A.cols != ds.d || c.B.rows != ds.d || c.B.cols != ds.n || c.C.rows != ds.m ||
        c.C.cols != ds.n) {
        g_last_error = "the shapes recorded in the commitments differ from m, d, n";
        return IMM_E_SHAPE;
    }
    if (c.A.dtype != IMM_I16 || c.B.dtype != IMM_I8 || c.C.dtype != IMM_I64) {
        g_last_error = "the commitments are not those of an int16 x int8 -> int64 statement";
        return IMM_E_DTYPE;
    }
    return IMM_OK;
}

// a0..a4: transcript head on the host, then eq vectors, encoding and the two streaming partial
// evaluations on the stream; leaves a[], b[] (zero-padded to D) in job.a / job.b.
static bool same_operands(const imm_matmul_desc& p, const imm_matmul_desc& q) {
    return p.A_dev == q.A_dev && p.B_dev == q.B_dev && p.dtA == q.dtA && p.dtB == q.dtB && p.m == q.m && p.d == q.d &&
           p.n == q.n;
}

// Forgets the tables queued ahead of time: the stream that writes them drains first, so that
// whatever uses the buffers next finds them idle.  Every sequence ends with this, also when it ends
// early: tables never outlive the call they were queued in, whose operands may change afterwards.
static int ahead_drop(imm_ctx* ctx) {
    if (!ctx->ahead_count) return IMM_OK;
    ctx->ahead_count = 0;
    IMM_HIP(hipStreamSynchronize(ctx->ahead_stream));
    return IMM_OK;
}

// Queues the widening of the raw operands of the proofs that follow the current one (look[0] is the
// next), as far as the ring reaches, each into a pair of tables that neither the current proof nor
// a queued one uses: the proofs that read those pairs before have returned.  The encode kernels run
// on a stream of their own, which starts once everything queued on s so far (the current proof's
// streaming kernels) is done: they share the machine with round loops, which leave the memory
// system idle, and with the streaming kernels of later proofs only as far as they fall behind.
static int ahead_queue(imm_ctx* ctx, hipStream_t s, const imm_matmul_desc* look, int count) {
    if (count > imm_ctx::kAheadDepth) count = imm_ctx::kAheadDepth;
    if (ctx->ahead_count >= count) return IMM_OK;
    int rc;
    if (!ctx->ahead_stream) {
        IMM_HIP(hipStreamCreateWithFlags(&ctx->ahead_stream, hipStreamNonBlocking));
        IMM_HIP(hipEventCreateWithFlags(&ctx->ahead_go, hipEventDisableTiming));
        for (hipEvent_t& e : ctx->ahead_done) IMM_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    }
    hipStream_t t = ctx->ahead_stream;
    IMM_HIP(hipEventRecord(ctx->ahead_go, s));
    IMM_HIP(hipStreamWaitEvent(t, ctx->ahead_go, 0));
    for (int i = ctx->ahead_count; i < count; ++i) {
        const imm_matmul_desc& next = look[i];
        imm_ctx::Ahead& q = ctx->ahead[i];
        q.ds = next;
        q.hasA = next.dtA != IMM_F64P;
        q.hasB = next.dtB != IMM_F64P;
        q.set = (ctx->set + 1 + i) % imm_ctx::kTableSets;
        const uint64_t m = next.m, d = next.d, n = next.n;
        if (q.hasA) {
            if ((rc = ctx->encA[q.set].ensure(sizeof(uint64_t) * m * d))) return rc;
            if ((rc = ctx->prof.begin(IMM_K_ENCODE_A, t))) return rc;
            IMM_HIP(k::encode(t, next.A_dev, (int)next.dtA, m * d, ctx->encA[q.set].u64()));
            if ((rc = ctx->prof.end(IMM_K_ENCODE_A, t))) return rc;
        }
        if (q.hasB) {
            if ((rc = ctx->encB[q.set].ensure(sizeof(uint64_t) * d * n))) return rc;
            if ((rc = ctx->prof.begin(IMM_K_ENCODE_B, t))) return rc;
            IMM_HIP(k::encode(t, next.B_dev, (int)next.dtB, d * n, ctx->encB[q.set].u64()));
            if ((rc = ctx->prof.end(IMM_K_ENCODE_B, t))) return rc;
        }
        IMM_HIP(hipEventRecord(ctx->ahead_done[q.set], t));
        ctx->ahead_count = i + 1;
    }
    return IMM_OK;
}

// look[0..look_count) are the proofs that follow this one on the same context in the same call:
// their raw operands are widened while this proof and the ones between run.
// With `gate` the proof before this one in a chain is not finished yet: the head of the transcript is
// left out here, and the eq kernel waits at the gate for the points.
static int stream_phase(imm_ctx* ctx, hipStream_t s, Job& job, const imm_matmul_desc* look = nullptr,
                        int look_count = 0, const k::Gate* gate = nullptr) {
    const imm_matmul_desc& ds = *job.ds;
    const uint64_t m = ds.m, d = ds.d, n = ds.n;
    job.mu = hf::ceil_log2(m);
    job.delta = hf::ceil_log2(d);
    job.nu = hf::ceil_log2(n);
    job.D = 1ull << job.delta;
    job.L = job.D;
    const uint64_t D = job.D;
    int rc;
    // a1 for A and B comes first: each operand is widened into scratch (skipped for pre-encoded tables
    // or in narrow-read mode).  The widening does not depend on the transcript: where it has launches
    // of its own they go out before the host hashes the head of the transcript, and everything else
    // is queued behind them while they run.
    const void* Ap = ds.A_dev;
    const void* Bp = ds.B_dev;
    int dtA = (int)ds.dtA, dtB = (int)ds.dtB;
    bool taken_over = false;
    if (ctx->ahead_count) {
        if (ctx->widen && same_operands(ctx->ahead[0].ds, ds)) {
            // the tables were queued while the proofs before this one ran: take them over
            const imm_ctx::Ahead q = ctx->ahead[0];
            for (int i = 1; i < ctx->ahead_count; ++i) ctx->ahead[i - 1] = ctx->ahead[i];
            ctx->ahead_count -= 1;
            ctx->set = q.set;
            taken_over = true;
            if (q.hasA) {
                Ap = ctx->encA[q.set].p;
                dtA = IMM_F64P;
            }
            if (q.hasB) {
                Bp = ctx->encB[q.set].p;
                dtB = IMM_F64P;
            }
        } else if ((rc = ahead_drop(ctx))) {
            return rc;
        }
    }
    imm::DevBuf& encA = ctx->encA[ctx->set];
    imm::DevBuf& encB = ctx->encB[ctx->set];
    bool eq_done = false;
    if (!gate && ctx->widen && ctx->fuse_reductions && !taken_over && dtA == IMM_I16 && (dtB == IMM_I8 || dtB == IMM_F64P)) {
        // A raw, B raw or widened beforehand: the widening and the eq vectors (a0 + a1 + a2) go out as one launch
        const bool rawB = dtB == IMM_I8;
        job.tr.head(m, d, n, ds.com->A.digest, ds.com->B.digest, ds.com->C.digest, job.mu, job.nu, job.rx, job.ry);
        ctx->mark(IMM_T_HEAD_HASHED);
        if ((rc = ctx->eqx.ensure(sizeof(uint64_t) << job.mu))) return rc;
        if ((rc = ctx->eqy.ensure(sizeof(uint64_t) << job.nu))) return rc;
        if ((rc = encA.ensure(sizeof(uint64_t) * m * d))) return rc;
        if (rawB && (rc = encB.ensure(sizeof(uint64_t) * d * n))) return rc;
        k::Point px{}, py{};
        for (int i = 0; i < job.mu; ++i) px.v[i] = job.rx[i];
        for (int i = 0; i < job.nu; ++i) py.v[i] = job.ry[i];
        if ((rc = ctx->prof.begin(IMM_K_ENCODE_B, s))) return rc;
        IMM_HIP(k::front(s, static_cast<const int16_t*>(Ap), m * d, encA.u64(), rawB ? static_cast<const int8_t*>(Bp) : nullptr,
                         rawB ? d * n : 0, rawB ? encB.u64() : nullptr, px, job.mu, ctx->eqx.u64(), py, job.nu,
                         ctx->eqy.u64()));
        if ((rc = ctx->prof.end(IMM_K_ENCODE_B, s))) return rc;
        Ap = encA.p;
        if (rawB) Bp = encB.p;
        dtA = dtB = IMM_F64P;
        eq_done = true;
        ctx->mark(IMM_T_FRONT_LAUNCHED);
    }
    if (ctx->widen && dtA != IMM_F64P) {
        if ((rc = encA.ensure(sizeof(uint64_t) * m * d))) return rc;
        if ((rc = ctx->prof.begin(IMM_K_ENCODE_A, s))) return rc;
        IMM_HIP(k::encode(s, Ap, dtA, m * d, encA.u64()));
        if ((rc = ctx->prof.end(IMM_K_ENCODE_A, s))) return rc;
        Ap = encA.p;
        dtA = IMM_F64P;
    }
    if (ctx->widen && dtB != IMM_F64P) {
        if ((rc = encB.ensure(sizeof(uint64_t) * d * n))) return rc;
        if ((rc = ctx->prof.begin(IMM_K_ENCODE_B, s))) return rc;
        IMM_HIP(k::encode(s, Bp, dtB, d * n, encB.u64()));
        if ((rc = ctx->prof.end(IMM_K_ENCODE_B, s))) return rc;
        Bp = encB.p;
        dtB = IMM_F64P;
    }
    // a0 + a2: the points from the transcript, and their eq vectors
    if (gate) {
        if ((rc = build_eq(ctx, s, nullptr, job.mu, nullptr, job.nu, wants_planes(dtB, n), gate))) return rc;
    } else if (!eq_done) {
        job.tr.head(m, d, n, ds.com->A.digest, ds.com->B.digest, ds.com->C.digest, job.mu, job.nu, job.rx, job.ry);
        ctx->mark(IMM_T_HEAD_HASHED);
        if ((rc = build_eq(ctx, s, job.rx, job.mu, job.ry, job.nu, wants_planes(dtB, n)))) return rc;
        ctx->mark(IMM_T_FRONT_LAUNCHED);
    }
    if (taken_over) IMM_HIP(hipStreamWaitEvent(s, ctx->ahead_done[ctx->set], 0));  // the tables are written

    // a3 + a4: in narrow-read mode both reductions in one launch where the operand forms allow it: the
    // table of A is read beside B's instead of filling and draining the machine on its own, and the
    // workgroup of A's reduction that finishes a block of columns last sums its partial vectors, so no
    // launch stands between the reductions and the round kernel.
    bool both = false;
    // Raw int16 activations also share the launch of weights that the caller widened beforehand
    // (narrow-read mode with pre-encoded B): A's 2 bytes per entry are a thirtieth of the launch's traffic.
    // (A widened table of A beside a widened B gains nothing: both stream from HBM at its rate, so A's
    // bytes take their time either way, and the hand-over costs more than the launch it saves.)
    if (ctx->fuse_reductions && ((dtB == IMM_I8 && (dtA == IMM_I16 || dtA == IMM_F64P)) ||
                                 (dtB == IMM_F64P && dtA == IMM_I16))) {
        const size_t elemA = dtA == IMM_F64P ? 8 : 2, elemB = dtB == IMM_F64P ? 8 : 1;
        const k::Split spA = k::plan_over_rows_beside(m, d, elemA, d * n * elemB), spB = k::plan_over_cols(d, n, dtB);
        const bool directB = spB.nsplit == 1;
        if ((rc = ensure_handover(ctx, s, (uint64_t)spA.nsplit * d))) return rc;
        if (!directB && (rc = ctx->partB.ensure(sizeof(uint64_t) * spB.nsplit * d))) return rc;
        if ((rc = ctx->prof.begin(IMM_K_REDUCE_B, s))) return rc;
        IMM_HIP(k::reduce_both(s, Ap, dtA, m, d, d, ctx->eqx.u64(), ctx->handA.u64(), spA,
                               static_cast<uint32_t*>(ctx->hand_counters.p), D, job.a, Bp, dtB, d, n, n, ctx->eqy.u64(),
                               wants_planes(dtB, n) ? static_cast<const uint32_t*>(ctx->eqy_planes.p) : nullptr,
                               directB ? job.b : ctx->partB.u64(), spB, &both));
        if (both) {
            if ((rc = ctx->prof.end(IMM_K_REDUCE_B, s))) return rc;
            if ((rc = finish_partial(ctx, s, directB, ctx->partB, spB.nsplit, d, D, job.b))) return rc;
        } else {
            ctx->prof.cancel(IMM_K_REDUCE_B);
        }
    }
    if (!both) {
        // Widened tables: when B's reduction writes b itself (a single column split), the sum of A's
        // partial vectors rides in its launch instead of taking one of its own between the two.
        const k::Split spA = k::plan_over_rows(m, d), spB = k::plan_over_cols(d, n, dtB);
        const bool directA = spA.nsplit == 1;
        if (ctx->fuse_reductions && dtB == IMM_F64P && spB.nsplit == 1 && !(directA && d == D)) {
            if (!directA && (rc = ctx->partA.ensure(sizeof(uint64_t) * spA.nsplit * d))) return rc;
            if ((rc = ctx->prof.begin(IMM_K_REDUCE_A, s))) return rc;
            IMM_HIP(k::reduce_over_rows(s, Ap, dtA, m, d, d, ctx->eqx.u64(), directA ? job.a : ctx->partA.u64(), spA));
            if ((rc = ctx->prof.end(IMM_K_REDUCE_A, s))) return rc;
            if ((rc = ctx->prof.begin(IMM_K_REDUCE_B, s))) return rc;
            if (directA)  // only the padding of a is left
                IMM_HIP(k::reduce_over_cols_and_combine(s, static_cast<const uint64_t*>(Bp), d, n, n, ctx->eqy.u64(), job.b,
                                                        nullptr, 0, 0, D - d, job.a + d));
            else
                IMM_HIP(k::reduce_over_cols_and_combine(s, static_cast<const uint64_t*>(Bp), d, n, n, ctx->eqy.u64(), job.b,
                                                        ctx->partA.u64(), spA.nsplit, d, D, job.a));
            if ((rc = ctx->prof.end(IMM_K_REDUCE_B, s))) return rc;
            if ((rc = finish_partial(ctx, s, true, ctx->partB, 1, d, D, job.b))) return rc;
        } else {
            if ((rc = partial_over_rows(ctx, s, IMM_K_REDUCE_A, Ap, dtA, m, d, d, ctx->eqx.u64(), D, ctx->partA, job.a)))
                return rc;
            if ((rc = partial_over_cols(ctx, s, IMM_K_REDUCE_B, Bp, dtB, d, n, n, ctx->eqy.u64(), D, ctx->partB, job.b)))
                return rc;
        }
    }
    ctx->mark(IMM_T_REDUCTIONS_LAUNCHED);
    if (look_count > 0 && ctx->widen && ctx->encode_ahead && (rc = ahead_queue(ctx, s, look, look_count))) return rc;

    std::memset(job.out, 0, sizeof(*job.out));
    job.out->version = IMM_PROOF_VERSION;
    job.out->mu = (uint32_t)job.mu;
    job.out->delta = (uint32_t)job.delta;
    job.out->nu = (uint32_t)job.nu;
    return IMM_OK;
}

// delta == 0: a single shared index, the claim is the product of the two table entries.
static int finish_without_rounds(imm_ctx* ctx, hipStream_t s, Job& job) {
    int rc;
    uint64_t av, bv;
    if ((rc = fetch_words(ctx, s, job.a, 1, &av))) return rc;
    if ((rc = fetch_words(ctx, s, job.b, 1, &bv))) return rc;
    job.out->c0 = hf::mul(av, bv);
    job.tr.absorb_words("clmC", &job.out->c0, 1);
    job.out->vA = av;
    job.out->vB = bv;
    const uint64_t fin[2] = {av, bv};
    job.tr.absorb_words("fin ", fin, 2);
    return IMM_OK;
}

// Tables longer than the single-workgroup limit are first shortened with one launch and one
// host round-trip per round.
static int long_table_prefix(imm_ctx* ctx, hipStream_t s, Job& job) {
    if (job.L <= k::kRoundsMaxL) return IMM_OK;
    int rc;
    uint64_t* words = ctx->words.u64();
    uint64_t g[3];
    if ((rc = run_round(ctx, s, job.a, job.b, job.L, false, 0, words + k::kWordG, g))) return rc;
    job.out->c0 = hf::add(g[0], g[1]);
    job.tr.absorb_words("clmC", &job.out->c0, 1);
    job.claim_absorbed = true;
    for (; job.L > k::kRoundsMaxL; ++job.kk) {
        job.out->g[3 * job.kk] = g[0];
        job.out->g[3 * job.kk + 1] = g[1];
        job.out->g[3 * job.kk + 2] = g[2];
        job.tr.absorb_words("rnd ", g, 3);
        job.rr[job.kk] = job.tr.challenge();
        if ((rc = run_round(ctx, s, job.a, job.b, job.L, true, job.rr[job.kk], words + k::kWordG, g))) return rc;
        job.L >>= 1;
    }
    return IMM_OK;
}

// a5..a8 for up to kRoundsMaxJobs proofs at once: the round kernel (one workgroup per proof) runs
// on the device while this thread hashes.  For every proof in turn the kernel posts g_k, the host
// absorbs it, squeezes r_k and posts it back; independent proofs overlap their waits.
struct RoundsLaunch {
    k::RoundsJobs rj{};
    int max_rounds = 0;
    int slot = 0;  // first of the `count` mailboxes (and reply rows, status words) that the launch uses
};
static int rounds_launch(imm_ctx* ctx, hipStream_t s, Job** jobs, int count, int slot, RoundsLaunch& rl) {
    k::Mailbox* mb = ctx->mailbox + slot;
    rl.slot = slot;
    uint64_t* replies = ctx->reply_in_device_memory && ctx->replies ? ctx->replies + (size_t)slot * IMM_MAX_ROUNDS : nullptr;
    k::RoundsJobs& rj = rl.rj;
    int& max_rounds = rl.max_rounds;
    for (int p = 0; p < count; ++p) {
        rj.job[p].a = jobs[p]->a;
        rj.job[p].b = jobs[p]->b;
        rj.job[p].L = jobs[p]->L;
        rj.job[p].rounds = jobs[p]->delta - jobs[p]->kk;
        // the kernel reads tables that do not fit into LDS with 16-byte accesses; they are buffers of the context
        if ((reinterpret_cast<uintptr_t>(jobs[p]->a) | reinterpret_cast<uintptr_t>(jobs[p]->b)) % 16 != 0) {
            g_last_error = "round tables are not 16-byte aligned";
            return IMM_E_STATE;
        }
        // The last rounds, on tables of at most 2^host_tail entries, are the host's: it computes them in
        // less time than one message takes to the device and back (the kernel needs two rounds of its own).
        // One host thread serves the proofs of a launch in turn while their workgroups work side by side,
        // so with `count` proofs the host's rounds must be that much shorter to beat the device's.
        const int tail = std::max(0, ctx->host_tail - hf::ceil_log2((uint64_t)count));
        rj.job[p].tail_rounds = rj.job[p].rounds >= tail + 2 ? tail : 0;
        if (rj.job[p].rounds > max_rounds) max_rounds = rj.job[p].rounds;
        // every slot that the kernel will write starts out empty
        std::memset(&mb[p], 0xFF, offsetof(k::Mailbox, tail));
        for (int t = 0; t < 2 && rj.job[p].tail_rounds; ++t) std::memset(mb[p].tail[t], 0xFF, sizeof(uint64_t) << rj.job[p].tail_rounds);
    }
    std::atomic_thread_fence(std::memory_order_seq_cst);
    if (replies) {  // ahead of the launch on the same path to the device, so the kernel finds them empty
        for (int p = 0; p < count; ++p)
            for (int t = 0; t < rj.job[p].rounds; ++t)
                *reinterpret_cast<volatile uint64_t*>(replies + (size_t)p * IMM_MAX_ROUNDS + t) = k::kMailEmpty;
        _mm_sfence();
    }
    int rc;
    uint64_t* status_dev = ctx->words.u64() + k::kWordCount + 4 + slot;
    if ((rc = ctx->prof.begin(IMM_K_ROUND, s))) return rc;
    IMM_HIP(k::rounds_mailbox(s, rj, count, mb, replies, ctx->spin_limit, status_dev));
    if ((rc = ctx->prof.end(IMM_K_ROUND, s))) return rc;
    ctx->mark(IMM_T_ROUNDS_LAUNCHED);
    return IMM_OK;
}

// The host's side of the loop that rounds_launch started.  On failure the kernel's waits have been
// released (abort values in every reply slot); the caller lets the stream drain.
static int rounds_serve(imm_ctx* ctx, Job** jobs, int count, const RoundsLaunch& rl) {
    k::Mailbox* mb = ctx->mailbox + rl.slot;
    uint64_t* replies = ctx->reply_in_device_memory && ctx->replies ? ctx->replies + (size_t)rl.slot * IMM_MAX_ROUNDS : nullptr;
    const k::RoundsJobs& rj = rl.rj;
    const int max_rounds = rl.max_rounds;
    bool ok = true, bad_tables = false;
    // tables of the proofs whose last rounds the host computes (filled when the device hands them over)
    std::vector<uint64_t> tail((size_t)count * 2 << k::kTailMaxLog2);
    for (int slot = 0; slot < max_rounds && ok; ++slot) {
        for (int p = 0; p < count && ok; ++p) {
            Job& job = *jobs[p];
            if (slot >= rj.job[p].rounds) continue;
            const int kk = job.kk + slot;
            const int dev_rounds = rj.job[p].rounds - rj.job[p].tail_rounds;  // challenges that the kernel binds
            uint64_t* ta = tail.data() + ((size_t)p * 2 << k::kTailMaxLog2);
            uint64_t* tb = ta + (size_t(1) << k::kTailMaxLog2);
            uint64_t g[3];
            if (!rj.job[p].tail_rounds || slot <= dev_rounds) {  // the kernel's messages: one more than it binds challenges
                for (int t = 0; t < 3 && ok; ++t) ok = mail_wait(&mb[p].g[slot][t], ctx->host_wait_ms, &g[t]);
                if (!ok) break;
                if (g[0] >= hf::P || g[1] >= hf::P || g[2] >= hf::P) {  // k::kMailFail: the tables were not canonical
                    ok = false;
                    bad_tables = true;
                    break;
                }
            } else {
                hf::round_evals(ta, tb, 1ull << (rj.job[p].rounds - slot), g);
            }
            if (slot == 0 && p == 0) ctx->mark(IMM_T_FIRST_MESSAGE);
            if (!job.claim_absorbed) {
                job.out->c0 = hf::add(g[0], g[1]);
                job.tr.absorb_words("clmC", &job.out->c0, 1);
                job.claim_absorbed = true;
            }
            job.out->g[3 * kk] = g[0];
            job.out->g[3 * kk + 1] = g[1];
            job.out->g[3 * kk + 2] = g[2];
            job.tr.absorb_words("rnd ", g, 3);
            job.rr[kk] = job.tr.challenge();
            if (!rj.job[p].tail_rounds || slot < dev_rounds) {
                if (replies)
                    reply_store(replies + (size_t)p * IMM_MAX_ROUNDS + slot, job.rr[kk]);
                else
                    __atomic_store_n(&mb[p].r[slot], job.rr[kk], __ATOMIC_RELEASE);
            } else {
                const uint64_t len = 1ull << (rj.job[p].rounds - slot);  // table length before this round's fold
                if (slot == dev_rounds)  // the kernel has bound its last challenge: its tables are on their way
                    for (uint64_t i = 0; i < len && ok; ++i)
                        ok = mail_wait(&mb[p].tail[0][i], ctx->host_wait_ms, &ta[i]) &&
                             mail_wait(&mb[p].tail[1][i], ctx->host_wait_ms, &tb[i]);
                if (!ok) break;
                hf::fold(ta, len, job.rr[kk]);
                hf::fold(tb, len, job.rr[kk]);
            }
            if (p == 0 && (slot == 0 || slot == rj.job[0].rounds - 1))
                ctx->mark(slot == 0 ? IMM_T_FIRST_CHALLENGE : IMM_T_LAST_CHALLENGE);
        }
    }
    for (int p = 0; p < count && ok; ++p) {
        uint64_t fin[2] = {0, 0};
        if (rj.job[p].tail_rounds) {
            fin[0] = tail[(size_t)p * 2 << k::kTailMaxLog2];
            fin[1] = tail[((size_t)p * 2 + 1) << k::kTailMaxLog2];
        } else {
            ok = mail_wait(&mb[p].fin[0], ctx->host_wait_ms, &fin[0]) && mail_wait(&mb[p].fin[1], ctx->host_wait_ms, &fin[1]);
            if (!ok) break;
        }
        jobs[p]->out->vA = fin[0];
        jobs[p]->out->vB = fin[1];
        jobs[p]->tr.absorb_words("fin ", fin, 2);
        if (p == 0) ctx->mark(IMM_T_FINAL_VALUES);
    }
    if (!ok) {
        // release every workgroup from whatever wait it is in, then let the kernel drain
        for (int p = 0; p < count; ++p)
            for (int t = 0; t < IMM_MAX_ROUNDS; ++t) {
                __atomic_store_n(&mb[p].r[t], k::kMailAbort, __ATOMIC_RELEASE);
                if (replies) reply_store(replies + (size_t)p * IMM_MAX_ROUNDS + t, k::kMailAbort);
            }
        g_last_error = bad_tables ? "the reductions did not deliver canonical field elements (a hand-over between workgroups ran out)"
                                  : "round kernel and host transcript lost contact (mailbox wait ran out)";
        return IMM_E_HIP;
    }
    // No stream synchronisation here: posting fin[] is a workgroup's last access to its mailbox
    // and tables, every result is already on the host, and whatever is launched next on this
    // stream is ordered behind the kernel's last instructions anyway.
    return IMM_OK;
}

static int rounds_with_host_transcript(imm_ctx* ctx, hipStream_t s, Job** jobs, int count) {
    RoundsLaunch rl;
    int rc = rounds_launch(ctx, s, jobs, count, 0, rl);
    if (rc) return rc;
    rc = rounds_serve(ctx, jobs, count, rl);
    if (rc) (void)hipStreamSynchronize(s);
    return rc;
}

// a5..a8 in one launch that also hashes the transcript on the device; one copy at the end brings
// back the proof words, the challenges and the new state.
static int rounds_with_device_transcript(imm_ctx* ctx, hipStream_t s, Job& job) {
    int rc;
    uint64_t* words = ctx->words.u64();
    const uint8_t* st = job.tr.s;
    uint32_t st_in[8];
    for (int i = 0; i < 8; ++i)
        st_in[i] = (uint32_t)st[4 * i] << 24 | (uint32_t)st[4 * i + 1] << 16 | (uint32_t)st[4 * i + 2] << 8 |
                   (uint32_t)st[4 * i + 3];
    uint32_t* st_dev = reinterpret_cast<uint32_t*>(words + k::kWordCount);
    if ((rc = ctx->prof.begin(IMM_K_ROUND, s))) return rc;
    IMM_HIP(k::rounds(s, job.a, job.b, job.L, job.delta - job.kk, job.kk, !job.claim_absorbed, st_in, words, st_dev));
    if ((rc = ctx->prof.end(IMM_K_ROUND, s))) return rc;
    uint64_t hw[k::kWordCount + 4];
    if ((rc = fetch_words(ctx, s, words, k::kWordCount + 4, hw))) return rc;
    imm_proof* out = job.out;
    if (!job.claim_absorbed) out->c0 = hw[k::kWordC0];
    for (int t = job.kk; t < job.delta; ++t) {
        out->g[3 * t] = hw[k::kWordG + 3 * t];
        out->g[3 * t + 1] = hw[k::kWordG + 3 * t + 1];
        out->g[3 * t + 2] = hw[k::kWordG + 3 * t + 2];
        job.rr[t] = hw[k::kWordR + t];
    }
    out->vA = hw[k::kWordVA];
    out->vB = hw[k::kWordVB];
    const uint32_t* st_out = reinterpret_cast<const uint32_t*>(hw + k::kWordCount);
    for (int i = 0; i < 8; ++i) {
        job.tr.s[4 * i] = (uint8_t)(st_out[i] >> 24);
        job.tr.s[4 * i + 1] = (uint8_t)(st_out[i] >> 16);
        job.tr.s[4 * i + 2] = (uint8_t)(st_out[i] >> 8);
        job.tr.s[4 * i + 3] = (uint8_t)st_out[i];
    }
    return IMM_OK;
}

// Everything after the streaming phase for one proof; leaves the new state in job.tr.
static int finish_one(imm_ctx* ctx, hipStream_t s, Job& job) {
    int rc;
    if (job.delta == 0) return finish_without_rounds(ctx, s, job);
    if ((rc = long_table_prefix(ctx, s, job))) return rc;
    if (ctx->transcript_mode == IMM_TRANSCRIPT_HOST) {
        Job* one = &job;
        return rounds_with_host_transcript(ctx, s, &one, 1);
    }
    return rounds_with_device_transcript(ctx, s, job);
}

static int prove_one(imm_ctx* ctx, hipStream_t s, const imm_matmul_desc& ds, uint8_t state[32], imm_proof* out,
                     const imm_matmul_desc* look = nullptr, int look_count = 0) {
    if (!state || !out) return IMM_E_NULL;
    int rc;
    if ((rc = check_desc(ds))) return rc;
    ctx->marks = 0;
    ctx->mark(IMM_T_ENTRY);
    Job job(state);
    job.ds = &ds;
    job.out = out;
    const uint64_t D = 1ull << hf::ceil_log2(ds.d);
    if ((rc = ctx->a.ensure(sizeof(uint64_t) * D))) return rc;
    if ((rc = ctx->b.ensure(sizeof(uint64_t) * D))) return rc;
    if ((rc = ctx->words.ensure(sizeof(uint64_t) * kWordsDev))) return rc;
    job.a = ctx->a.u64();
    job.b = ctx->b.u64();
    if ((rc = stream_phase(ctx, s, job, look, look_count))) return rc;
    if (ctx->debug) {
        if ((rc = ctx->snapA.ensure(sizeof(uint64_t) * D))) return rc;
        if ((rc = ctx->snapB.ensure(sizeof(uint64_t) * D))) return rc;
        IMM_HIP(hipMemcpyAsync(ctx->snapA.p, job.a, sizeof(uint64_t) * D, hipMemcpyDeviceToDevice, s));
        IMM_HIP(hipMemcpyAsync(ctx->snapB.p, job.b, sizeof(uint64_t) * D, hipMemcpyDeviceToDevice, s));
    }
    if ((rc = finish_one(ctx, s, job))) return rc;
    std::memcpy(state, job.tr.s, 32);
    if (ctx->debug) {
        ctx->dbg_mu = job.mu; ctx->dbg_delta = job.delta; ctx->dbg_nu = job.nu;
        std::memcpy(ctx->dbg_rx, job.rx, sizeof(job.rx));
        std::memcpy(ctx->dbg_ry, job.ry, sizeof(job.ry));
        std::memcpy(ctx->dbg_r, job.rr, sizeof(job.rr));
    }
    ctx->mark(IMM_T_EXIT);
    return ctx->prof.mask ? ctx->prof.flush() : IMM_OK;
}

// A chain of proofs (each starts from the state the one before it leaves) with the kernels of proof
// p + 1 queued while the host still serves the round loop of proof p.  The state that proof p + 1
// starts from is not known then, so its eq kernel is launched without the points and waits for them at
// a gate; everything behind it in the stream (reductions, round kernel) needs no value from the host
// to be launched.  When proof p is finished the host hashes the head of proof p + 1 and writes the
// points through the gate: the device goes on within a microsecond or two, where a launch after the
// fact costs the hashing, the launch calls and the start of a kernel on an idle queue (about 10 us per
// proof).  Proofs that the round kernel does not take (no rounds, very long tables) are proven the
// plain way, with nothing queued across them.
static bool queueable(const imm_matmul_desc& ds) {
    const int delta = hf::ceil_log2(ds.d);
    return delta >= 1 && (1ull << delta) <= k::kRoundsMaxL;
}

static int prove_chain(imm_ctx* ctx, hipStream_t s, int count, const imm_matmul_desc* descs, uint8_t state[32],
                       imm_proof* outs, uint8_t* states_out) {
    int rc;
    uint64_t Dmax = 1;
    for (int p = 0; p < count; ++p) Dmax = std::max<uint64_t>(Dmax, uint64_t(1) << hf::ceil_log2(descs[p].d));
    if ((rc = ctx->a.ensure(sizeof(uint64_t) * Dmax))) return rc;
    if ((rc = ctx->b.ensure(sizeof(uint64_t) * Dmax))) return rc;
    if ((rc = ctx->words.ensure(sizeof(uint64_t) * kWordsDev))) return rc;

    std::vector<void*> parked;
    struct Parking {  // buffers outgrown while kernels are queued are freed when the stream has drained
        std::vector<void*>& list;
        hipStream_t s;
        explicit Parking(std::vector<void*>& l, hipStream_t st) : list(l), s(st) { g_parked = &list; }
        ~Parking() {
            g_parked = nullptr;
            if (list.empty()) return;
            (void)hipStreamSynchronize(s);
            for (void* q : list) (void)hipFree(q);
        }
    } parking(parked, s);

    Job job[2] = {Job(state), Job(state)};
    RoundsLaunch rl[2];
    bool in_loop[2] = {false, false};  // its round kernel is launched and waits to be served
    auto set_up = [&](int p, int sl) {
        job[sl] = Job(state);
        job[sl].ds = &descs[p];
        job[sl].out = &outs[p];
        job[sl].a = ctx->a.u64();
        job[sl].b = ctx->b.u64();
    };
    // proof p from the known state: plain launch; its round loop is left to be served if the kernel takes it
    auto start_plain = [&](int p, int sl) -> int {
        set_up(p, sl);
        int r;
        if ((r = stream_phase(ctx, s, job[sl], descs + p + 1, count - p - 1))) return r;
        in_loop[sl] = queueable(descs[p]);
        if (in_loop[sl]) {
            Job* one = &job[sl];
            return rounds_launch(ctx, s, &one, 1, sl, rl[sl]);
        }
        return finish_one(ctx, s, job[sl]);
    };
    auto give_up = [&](int r) -> int {
        // release whatever waits for this thread, in both slots, then let everything drain
        for (int sl = 0; sl < 2; ++sl) {
            gate_fill(gate_of(ctx, sl), k::kMailAbort);
            uint64_t* replies = ctx->reply_in_device_memory && ctx->replies ? ctx->replies + (size_t)sl * IMM_MAX_ROUNDS : nullptr;
            for (int t = 0; t < IMM_MAX_ROUNDS; ++t) {
                __atomic_store_n(&ctx->mailbox[sl].r[t], k::kMailAbort, __ATOMIC_RELEASE);
                if (replies) reply_store(replies + t, k::kMailAbort);
            }
        }
        (void)hipStreamSynchronize(s);
        (void)ahead_drop(ctx);
        return r;
    };

    if ((rc = start_plain(0, 0))) return give_up(rc);
    for (int p = 0; p < count; ++p) {
        const int sl = p & 1, nsl = sl ^ 1;
        bool queued = false;
        k::Gate* gate = gate_of(ctx, nsl);
        if (in_loop[sl] && p + 1 < count && queueable(descs[p + 1])) {
            set_up(p + 1, nsl);
            gate_fill(gate, k::kMailEmpty);
            if ((rc = stream_phase(ctx, s, job[nsl], descs + p + 2, count - p - 2, gate))) return give_up(rc);
            Job* one = &job[nsl];
            if ((rc = rounds_launch(ctx, s, &one, 1, nsl, rl[nsl]))) return give_up(rc);
            in_loop[nsl] = true;
            queued = true;
        }
        if (in_loop[sl]) {
            Job* one = &job[sl];
            if ((rc = rounds_serve(ctx, &one, 1, rl[sl]))) return give_up(rc);
            in_loop[sl] = false;
        }
        std::memcpy(state, job[sl].tr.s, 32);
        if (states_out) std::memcpy(states_out + 32 * (size_t)p, state, 32);
        if (queued) {
            Job& jn = job[nsl];
            const imm_matmul_desc& ds = descs[p + 1];
            jn.tr = Transcript(state);
            jn.tr.head(ds.m, ds.d, ds.n, ds.com->A.digest, ds.com->B.digest, ds.com->C.digest, jn.mu, jn.nu, jn.rx, jn.ry);
            gate_open(gate, jn.rx, jn.mu, jn.ry, jn.nu);
        } else if (p + 1 < count) {
            if ((rc = start_plain(p + 1, nsl))) return give_up(rc);
        }
    }
    return IMM_OK;
}

// Independent proofs (every one starts from `start`): the streaming phases are queued back to
// back, each into its own pair of tables, and the round loops of a whole group then run in one
// launch.  A statement that needs a different path (no rounds, very long tables) is proven on its
// own.  states_out[p] receives the state after proof p.
static int prove_independent(imm_ctx* ctx, hipStream_t s, int count, const imm_matmul_desc* descs,
                             const uint8_t start[32], imm_proof* outs, uint8_t* states) {
    int rc;
    if ((rc = ctx->words.ensure(sizeof(uint64_t) * kWordsDev))) return rc;
    for (int g0 = 0; g0 < count; g0 += k::kRoundsMaxJobs) {
        const int g1 = g0 + k::kRoundsMaxJobs < count ? g0 + k::kRoundsMaxJobs : count;
        uint64_t words_needed = 0;
        for (int p = g0; p < g1; ++p) words_needed += 2ull << hf::ceil_log2(descs[p].d);
        if ((rc = ctx->group_tables.ensure(sizeof(uint64_t) * words_needed))) return rc;
        std::vector<Job> jobs;
        jobs.reserve((size_t)(g1 - g0));
        std::vector<Job*> grouped;
        uint64_t* next = ctx->group_tables.u64();
        for (int p = g0; p < g1; ++p) {
            jobs.emplace_back(start);
            Job& job = jobs.back();
            job.ds = &descs[p];
            job.out = &outs[p];
            const uint64_t D = 1ull << hf::ceil_log2(descs[p].d);
            job.a = next;
            job.b = next + D;
            next += 2 * D;
            if ((rc = stream_phase(ctx, s, job))) return rc;
            if (job.delta == 0 || job.L > k::kRoundsMaxL) {
                if ((rc = finish_one(ctx, s, job))) return rc;
            } else {
                grouped.push_back(&job);
            }
        }
        if (!grouped.empty() && (rc = rounds_with_host_transcript(ctx, s, grouped.data(), (int)grouped.size())))
            return rc;
        for (int p = g0; p < g1; ++p) std::memcpy(states + 32 * (size_t)p, jobs[(size_t)(p - g0)].tr.s, 32);
    }
    return ctx->prof.mask ? ctx->prof.flush() : IMM_OK;
}

}  // namespace imm

using namespace imm;

// No exception crosses the C ABI: host allocations that fail (vectors of jobs, leaves, events) and
// anything else the standard library throws become error codes.
template <typename F>
static int guarded(F&& body) {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        g_last_error = "host allocation failed";
        return IMM_E_NOMEM;
    } catch (const std::exception& e) {
        g_last_error = e.what();
        return IMM_E_STATE;
    } catch (...) {
        g_last_error = "unknown exception";
        return IMM_E_STATE;
    }
}

extern "C" const char* imm_last_error(void) { return g_last_error.c_str(); }

extern "C" int imm_ctx_create(imm_ctx** out, int device, size_t scratch_bytes) {
    return guarded([&]() -> int {
        if (!out) return IMM_E_NULL;
        *out = nullptr;
        int count = 0;
        IMM_HIP(hipGetDeviceCount(&count));
        if (device < 0 || device >= count) {
            g_last_error = "no such HIP device";
            return IMM_E_HIP;
        }
        IMM_HIP(hipSetDevice(device));
        imm_ctx* ctx = new (std::nothrow) imm_ctx();
        if (!ctx) return IMM_E_NOMEM;
        ctx->device = device;
        hipError_t e = hipHostMalloc(reinterpret_cast<void**>(&ctx->pinned), 4096, hipHostMallocDefault);
        if (e != hipSuccess) {
            delete ctx;
            return fail_hip(e, "hipHostMalloc");
        }
        e = hipHostMalloc(reinterpret_cast<void**>(&ctx->mailbox),
                          sizeof(k::Mailbox) * k::kRoundsMaxJobs + sizeof(k::Gate) * kGateCount,
                          hipHostMallocMapped | hipHostMallocCoherent);
        if (e != hipSuccess) {
            (void)hipHostFree(ctx->pinned);
            delete ctx;
            return fail_hip(e, "hipHostMalloc(mailbox)");
        }
        ctx->gates_pinned = reinterpret_cast<k::Gate*>(ctx->mailbox + k::kRoundsMaxJobs);
        ctx->replies = reply_block_take(device);  // may be null: then the mailbox carries the challenges
        if (int rc = static_scratch_prepare(device)) {
            (void)hipHostFree(ctx->pinned);
            (void)hipHostFree(ctx->mailbox);
            reply_block_give(device, ctx->replies);
            delete ctx;
            return rc;
        }
        if (scratch_bytes) {
            // the hint goes to the widened weight table, by far the largest scratch buffer
            int rc = ctx->encB[0].ensure(scratch_bytes);
            if (rc) {
                (void)hipHostFree(ctx->pinned);
                (void)hipHostFree(ctx->mailbox);
                delete ctx;
                return rc;
            }
        }
        *out = ctx;
        return IMM_OK;
    });
}

extern "C" int imm_ctx_destroy(imm_ctx* ctx) {
    if (!ctx) return IMM_E_NULL;
    (void)hipSetDevice(ctx->device);
    (void)hipDeviceSynchronize();
    if (ctx->ahead_stream) {
        (void)hipEventDestroy(ctx->ahead_go);
        for (hipEvent_t e : ctx->ahead_done) (void)hipEventDestroy(e);
        (void)hipStreamDestroy(ctx->ahead_stream);
    }
    for (DevBuf& bf : ctx->encA) bf.release();
    for (DevBuf& bf : ctx->encB) bf.release();
    for (DevBuf* bf : {&ctx->eqx, &ctx->eqy, &ctx->eqy_planes, &ctx->a, &ctx->b, &ctx->partA, &ctx->partB, &ctx->handA,
                       &ctx->hand_counters,
                       &ctx->round_scratch, &ctx->words, &ctx->snapA, &ctx->snapB, &ctx->group_tables,
                       &ctx->ldd_partial, &ctx->ldd_post, &ctx->ldd_sum, &ctx->ldd_arrive, &ctx->commit_leaves,
                       &ctx->commit_digests})
        bf->release();
    ctx->prof.destroy();
    reply_block_give(ctx->device, ctx->replies);
    if (ctx->pinned) (void)hipHostFree(ctx->pinned);
    if (ctx->mailbox) (void)hipHostFree(ctx->mailbox);
    delete ctx;
    return IMM_OK;
}

extern "C" int imm_ctx_set_option(imm_ctx* ctx, int option, int64_t value) {
    if (!ctx) return IMM_E_NULL;
    switch (option) {
    case IMM_OPT_DEBUG_SNAPSHOTS: ctx->debug = value != 0; return IMM_OK;
    case IMM_OPT_WIDEN: ctx->widen = value != 0; return IMM_OK;
    case IMM_OPT_FUSE_REDUCTIONS: ctx->fuse_reductions = value != 0; return IMM_OK;
    case IMM_OPT_ENCODE_AHEAD: ctx->encode_ahead = value != 0; return IMM_OK;
    case IMM_OPT_TIMELINE: ctx->timeline = value != 0; ctx->marks = 0; return IMM_OK;
    case IMM_OPT_QUEUE_AHEAD: ctx->queue_ahead = value != 0; return IMM_OK;
    case IMM_OPT_HOST_TAIL:
        if (value < 0 || value > k::kTailMaxLog2) return IMM_E_SHAPE;
        ctx->host_tail = (int)value;
        return IMM_OK;
    case IMM_OPT_REPLY_IN_DEVICE_MEMORY: ctx->reply_in_device_memory = value != 0; return IMM_OK;
    case IMM_OPT_TRANSCRIPT:
        if (value != IMM_TRANSCRIPT_DEVICE && value != IMM_TRANSCRIPT_HOST) return IMM_E_SHAPE;
        ctx->transcript_mode = (int)value;
        return IMM_OK;
    case IMM_OPT_SPIN_LIMIT:
        if (value < 0) return IMM_E_SHAPE;
        ctx->spin_limit = (uint64_t)value;
        return IMM_OK;
    case IMM_OPT_HOST_WAIT_MS:
        if (value < 1) return IMM_E_SHAPE;
        ctx->host_wait_ms = value;
        return IMM_OK;
    default: return IMM_E_STATE;
    }
}

extern "C" int imm_ctx_set_profiling(imm_ctx* ctx, uint32_t mask) {
    return guarded([&]() -> int {
        if (!ctx) return IMM_E_NULL;
        IMM_HIP(hipSetDevice(ctx->device));
        if (ctx->prof.mask) {
            int rc = ctx->prof.flush();
            if (rc) return rc;
        }
        ctx->prof.mask = mask & ((1u << IMM_K_COUNT) - 1);
        return IMM_OK;
    });
}

extern "C" int imm_ctx_kernel_time(imm_ctx* ctx, int kernel_id, uint64_t* launches, double* total_ms) {
    return guarded([&]() -> int {
        if (!ctx) return IMM_E_NULL;
        if (kernel_id < 0 || kernel_id >= IMM_K_COUNT) return IMM_E_SHAPE;
        IMM_HIP(hipSetDevice(ctx->device));
        int rc = ctx->prof.flush();
        if (rc) return rc;
        if (launches) *launches = ctx->prof.launches[kernel_id];
        if (total_ms) *total_ms = ctx->prof.total_ms[kernel_id];
        return IMM_OK;
    });
}

extern "C" int imm_ctx_reset_profiling(imm_ctx* ctx) {
    return guarded([&]() -> int {
        if (!ctx) return IMM_E_NULL;
        IMM_HIP(hipSetDevice(ctx->device));
        int rc = ctx->prof.flush();
        ctx->prof.reset();
        return rc;
    });
}

extern "C" int imm_encode(imm_ctx* ctx, void* stream, const void* src_dev, imm_dtype dtype, uint64_t count,
                          uint64_t* dst_dev) {
    return guarded([&]() -> int {
        if (!ctx || (count && (!src_dev || !dst_dev))) return IMM_E_NULL;
        if (dtype != IMM_I8 && dtype != IMM_I16 && dtype != IMM_I64) return IMM_E_DTYPE;
        IMM_HIP(hipSetDevice(ctx->device));
        hipStream_t s = static_cast<hipStream_t>(stream);
        int rc;
        if ((rc = ctx->prof.begin(IMM_K_ENCODE_B, s))) return rc;
        IMM_HIP(k::encode(s, src_dev, dtype, count, dst_dev));
        return ctx->prof.end(IMM_K_ENCODE_B, s);
    });
}

extern "C" int imm_mle_eval(imm_ctx* ctx, void* stream, const void* table_dev, imm_dtype dt, uint64_t rows,
                            uint64_t cols, uint64_t ld, const uint64_t* pt_rows, const uint64_t* pt_cols,
                            uint64_t* out_host) {
    return guarded([&]() -> int {
        if (!ctx || !table_dev || !out_host) return IMM_E_NULL;
        if (!dim_ok(rows) || !dim_ok(cols) || ld < cols) return IMM_E_SHAPE;
        if (dt < IMM_I8 || dt > IMM_F64P) return IMM_E_DTYPE;
        const int tR = hf::ceil_log2(rows), tC = hf::ceil_log2(cols);
        if ((tR && !pt_rows) || (tC && !pt_cols)) return IMM_E_NULL;
        for (int i = 0; i < tR; ++i)
            if (pt_rows[i] >= hf::P) return IMM_E_SHAPE;
        for (int i = 0; i < tC; ++i)
            if (pt_cols[i] >= hf::P) return IMM_E_SHAPE;
        IMM_HIP(hipSetDevice(ctx->device));
        hipStream_t s = static_cast<hipStream_t>(stream);
        int rc;
        if ((rc = build_eq(ctx, s, pt_rows, tR, pt_cols, tC, cols >= 256 && wants_planes((int)dt, cols)))) return rc;
        if ((rc = ctx->words.ensure(sizeof(uint64_t) * kWordsDev))) return rc;
        if (cols >= 256) {
            // wide table: reduce along the rows first, then one dot product with the row weights
            if ((rc = ctx->a.ensure(sizeof(uint64_t) * rows))) return rc;
            if ((rc = partial_over_cols(ctx, s, IMM_K_REDUCE_B, table_dev, dt, rows, cols, ld, ctx->eqy.u64(), rows,
                                        ctx->partB, ctx->a.u64())))
                return rc;
            IMM_HIP(k::dot(s, ctx->a.u64(), ctx->eqx.u64(), rows, ctx->words.u64()));
        } else {
            if ((rc = ctx->a.ensure(sizeof(uint64_t) * cols))) return rc;
            if ((rc = partial_over_rows(ctx, s, IMM_K_REDUCE_A, table_dev, dt, rows, cols, ld, ctx->eqx.u64(), cols,
                                        ctx->partA, ctx->a.u64())))
                return rc;
            IMM_HIP(k::dot(s, ctx->a.u64(), ctx->eqy.u64(), cols, ctx->words.u64()));
        }
        if ((rc = fetch_words(ctx, s, ctx->words.u64(), 1, out_host))) return rc;
        return ctx->prof.mask ? ctx->prof.flush() : IMM_OK;
    });
}

extern "C" int imm_sumcheck_matmul_prove(imm_ctx* ctx, void* stream, const void* A_dev, imm_dtype dtA,
                                         const void* B_dev, imm_dtype dtB, uint64_t m, uint64_t d, uint64_t n,
                                         const imm_commit* com, uint8_t transcript_state[32], imm_proof* out_host) {
    return guarded([&]() -> int {
        if (!ctx) return IMM_E_NULL;
        IMM_HIP(hipSetDevice(ctx->device));
        imm_matmul_desc ds;
        ds.A_dev = A_dev; ds.B_dev = B_dev;
        ds.dtA = (uint32_t)dtA; ds.dtB = (uint32_t)dtB;
        ds.m = m; ds.d = d; ds.n = n;
        ds.com = com;
        return prove_one(ctx, static_cast<hipStream_t>(stream), ds, transcript_state, out_host);
    });
}

extern "C" int imm_sumcheck_matmul_prove_batch(imm_ctx* ctx, void* stream, int count, const imm_matmul_desc* descs,
                                               int chained, uint8_t transcript_state[32], imm_proof* outs_host,
                                               uint8_t* states_out) {
    return guarded([&]() -> int {
        if (!ctx || !transcript_state || (count > 0 && (!descs || !outs_host))) return IMM_E_NULL;
        if (count < 0) return IMM_E_SHAPE;
        IMM_HIP(hipSetDevice(ctx->device));
        hipStream_t s = static_cast<hipStream_t>(stream);
        // validate everything before the first launch
        for (int t = 0; t < count; ++t) {
            int rc = check_desc(descs[t]);
            if (rc) return rc;
        }
        uint8_t start[32], cur[32];
        std::memcpy(start, transcript_state, 32);
        std::memcpy(cur, transcript_state, 32);
        if (!chained && count > 1 && ctx->transcript_mode == IMM_TRANSCRIPT_HOST && !ctx->debug) {
            std::vector<uint8_t> states((size_t)count * 32);
            int rc = prove_independent(ctx, s, count, descs, start, outs_host, states.data());
            if (rc) return rc;
            if (states_out) std::memcpy(states_out, states.data(), states.size());
            std::memcpy(transcript_state, states.data() + 32 * (size_t)(count - 1), 32);
            return IMM_OK;
        }
        if (chained && count > 1 && ctx->queue_ahead && ctx->transcript_mode == IMM_TRANSCRIPT_HOST && !ctx->debug &&
            !ctx->timeline && !ctx->prof.mask) {
            int rc = prove_chain(ctx, s, count, descs, cur, outs_host, states_out);
            if (rc) return rc;
            std::memcpy(transcript_state, cur, 32);
            return IMM_OK;
        }
        for (int t = 0; t < count; ++t) {
            if (!chained) std::memcpy(cur, start, 32);
            int rc = prove_one(ctx, s, descs[t], cur, &outs_host[t], descs + t + 1, count - t - 1);
            if (rc) {
                (void)ahead_drop(ctx);
                return rc;
            }
            if (states_out) std::memcpy(states_out + 32 * (size_t)t, cur, 32);
        }
        std::memcpy(transcript_state, cur, 32);
        return IMM_OK;
    });
}

extern "C" int imm_round_fold_eval(imm_ctx* ctx, void* stream, uint64_t* a_dev, uint64_t* b_dev, uint64_t L,
                                   const uint64_t* fold_r, uint64_t g_host[3]) {
    return guarded([&]() -> int {
        if (!ctx || !a_dev || !b_dev || !g_host) return IMM_E_NULL;
        if (L < 2 || (L & (L - 1)) || L > (1ull << IMM_MAX_ROUNDS)) return IMM_E_SHAPE;
        if (fold_r && *fold_r >= hf::P) return IMM_E_SHAPE;
        IMM_HIP(hipSetDevice(ctx->device));
        hipStream_t s = static_cast<hipStream_t>(stream);
        int rc;
        if ((rc = ctx->words.ensure(sizeof(uint64_t) * kWordsDev))) return rc;
        if ((rc = run_round(ctx, s, a_dev, b_dev, L, fold_r != nullptr, fold_r ? *fold_r : 0, ctx->words.u64(), g_host)))
            return rc;
        return ctx->prof.mask ? ctx->prof.flush() : IMM_OK;
    });
}

extern "C" int imm_debug_fetch(imm_ctx* ctx, int which, uint64_t* out_host, uint64_t capacity, uint64_t* count) {
    return guarded([&]() -> int {
        if (!ctx || !count) return IMM_E_NULL;
        if (!ctx->debug || ctx->dbg_delta < 0) return IMM_E_STATE;
        IMM_HIP(hipSetDevice(ctx->device));
        const uint64_t* host_src = nullptr;
        const void* dev_src = nullptr;
        uint64_t avail = 0;
        switch (which) {
        case 0: dev_src = ctx->eqx.p; avail = 1ull << ctx->dbg_mu; break;
        case 1: dev_src = ctx->eqy.p; avail = 1ull << ctx->dbg_nu; break;
        case 2: dev_src = ctx->snapA.p; avail = 1ull << ctx->dbg_delta; break;
        case 3: dev_src = ctx->snapB.p; avail = 1ull << ctx->dbg_delta; break;
        case 4: host_src = ctx->dbg_rx; avail = (uint64_t)ctx->dbg_mu; break;
        case 5: host_src = ctx->dbg_ry; avail = (uint64_t)ctx->dbg_nu; break;
        case 6: host_src = ctx->dbg_r; avail = (uint64_t)ctx->dbg_delta; break;
        default: return IMM_E_SHAPE;
        }
        *count = avail;
        uint64_t ncopy = avail < capacity ? avail : capacity;
        if (!ncopy) return IMM_OK;
        if (!out_host) return IMM_E_NULL;
        if (host_src) {
            std::memcpy(out_host, host_src, ncopy * sizeof(uint64_t));
        } else {
            IMM_HIP(hipDeviceSynchronize());
            IMM_HIP(hipMemcpy(out_host, dev_src, ncopy * sizeof(uint64_t), hipMemcpyDeviceToHost));
        }
        return IMM_OK;
    });
}

extern "C" int imm_debug_timeline(imm_ctx* ctx, uint32_t* ids, uint64_t* ns, uint32_t capacity, uint32_t* count) {
    if (!ctx || !count) return IMM_E_NULL;
    if (!ctx->timeline) return IMM_E_STATE;
    *count = (uint32_t)ctx->marks;
    for (int i = 0; i < ctx->marks && (uint32_t)i < capacity; ++i) {
        if (ids) ids[i] = ctx->mark_id[i];
        if (ns) ns[i] = ctx->mark_ns[i];
    }
    return IMM_OK;
}

extern "C" int imm_debug_device_challenge(imm_ctx* ctx, void* stream, uint8_t state[32], uint64_t* out_host) {
    return guarded([&]() -> int {
        if (!ctx || !state || !out_host) return IMM_E_NULL;
        IMM_HIP(hipSetDevice(ctx->device));
        hipStream_t s = static_cast<hipStream_t>(stream);
        int rc;
        if ((rc = ctx->words.ensure(sizeof(uint64_t) * kWordsDev))) return rc;
        uint32_t st_in[8];
        for (int i = 0; i < 8; ++i)
            st_in[i] = (uint32_t)state[4 * i] << 24 | (uint32_t)state[4 * i + 1] << 16 | (uint32_t)state[4 * i + 2] << 8 |
                       (uint32_t)state[4 * i + 3];
        uint64_t* words = ctx->words.u64();
        IMM_HIP(k::challenge_once(s, st_in, words, reinterpret_cast<uint32_t*>(words + 1)));
        uint64_t hw[5];
        if ((rc = fetch_words(ctx, s, words, 5, hw))) return rc;
        *out_host = hw[0];
        const uint32_t* st_out = reinterpret_cast<const uint32_t*>(hw + 1);
        for (int i = 0; i < 8; ++i) {
            state[4 * i] = (uint8_t)(st_out[i] >> 24);
            state[4 * i + 1] = (uint8_t)(st_out[i] >> 16);
            state[4 * i + 2] = (uint8_t)(st_out[i] >> 8);
            state[4 * i + 3] = (uint8_t)st_out[i];
        }
        return IMM_OK;
    });
}

extern "C" int imm_ldd_tv_kl(imm_ctx* ctx, void* stream, const float* logits_dev, const float* ref_dev, uint64_t T,
                             uint64_t n, uint64_t ld, double* tv_out_dev, double* kl_out_dev) {
    return guarded([&]() -> int {
        if (!ctx || !logits_dev || !ref_dev || (!tv_out_dev && !kl_out_dev)) return IMM_E_NULL;
        if (T == 0 || n == 0 || ld < n || T > 0x7FFFFFFFull || n > (1ull << 30)) return IMM_E_SHAPE;
        IMM_HIP(hipSetDevice(ctx->device));
        hipStream_t s = static_cast<hipStream_t>(stream);
        int rc;
        if (ctx->ldd_partial.bytes < k::ldd_slot_bytes(T, n) || ctx->ldd_post.bytes < k::ldd_post_bytes(T) ||
            ctx->ldd_sum.bytes < k::ldd_sum_bytes(T) || ctx->ldd_arrive.bytes < k::ldd_counter_bytes(T)) {
            if ((rc = ctx->ldd_partial.ensure(k::ldd_slot_bytes(T, n)))) return rc;
            if ((rc = ctx->ldd_post.ensure(k::ldd_post_bytes(T)))) return rc;
            if ((rc = ctx->ldd_sum.ensure(k::ldd_sum_bytes(T)))) return rc;
            if ((rc = ctx->ldd_arrive.ensure(k::ldd_counter_bytes(T)))) return rc;
            IMM_HIP(k::ldd_init_sync(s, ctx->ldd_partial.u64(), ctx->ldd_partial.bytes, ctx->ldd_post.u64(),
                                     ctx->ldd_post.bytes, ctx->ldd_sum.u64(), ctx->ldd_sum.bytes,
                                     static_cast<uint32_t*>(ctx->ldd_arrive.p), ctx->ldd_arrive.bytes));
        }
        // a workgroup whose wait runs out finishes on its own, so the bound can be short: about 50 ms
        const uint64_t wait_polls = ctx->spin_limit < (1ull << 15) ? ctx->spin_limit : (1ull << 15);
        if ((rc = ctx->prof.begin(IMM_K_LDD, s))) return rc;
        IMM_HIP(k::ldd_tv_kl(s, logits_dev, ref_dev, T, n, ld, ctx->ldd_partial.u64(), ctx->ldd_post.u64(),
                             ctx->ldd_sum.u64(), static_cast<uint32_t*>(ctx->ldd_arrive.p), wait_polls, tv_out_dev, kl_out_dev));
        return ctx->prof.end(IMM_K_LDD, s);
    });
}

extern "C" int imm_topk_distance(imm_ctx* ctx, void* stream, const float* logits_dev, uint64_t T, uint64_t n,
                                 uint64_t ld, const int32_t* idx_dev, uint32_t K, double* out_dev) {
    return guarded([&]() -> int {
        if (!ctx || !logits_dev || !idx_dev || !out_dev) return IMM_E_NULL;
        if (T == 0 || n == 0 || ld < n || T > 0x7FFFFFFFull || n > 0x7FFFFFFFull) return IMM_E_SHAPE;
        if (K < 1 || K > IMM_TOPK_MAX || K >= n) return IMM_E_SHAPE;
        IMM_HIP(hipSetDevice(ctx->device));
        hipStream_t s = static_cast<hipStream_t>(stream);
        int rc;
        if ((rc = ctx->prof.begin(IMM_K_TOPK, s))) return rc;
        IMM_HIP(k::topk_distance(s, logits_dev, T, n, ld, idx_dev, K, out_dev));
        return ctx->prof.end(IMM_K_TOPK, s);
    });
}

extern "C" int imm_tail_density(imm_ctx* ctx, void* stream, const double* dist_dev, uint64_t T, double t1,
                                double* out_host) {
    return guarded([&]() -> int {
        if (!ctx || !dist_dev || !out_host) return IMM_E_NULL;
        if (T == 0) return IMM_E_SHAPE;
        IMM_HIP(hipSetDevice(ctx->device));
        hipStream_t s = static_cast<hipStream_t>(stream);
        int rc;
        if ((rc = ctx->words.ensure(sizeof(uint64_t) * kWordsDev))) return rc;
        unsigned long long* count_dev = reinterpret_cast<unsigned long long*>(ctx->words.u64());
        IMM_HIP(k::tail_count(s, dist_dev, T, t1, count_dev));
        uint64_t count = 0;
        if ((rc = fetch_words(ctx, s, ctx->words.u64(), 1, &count))) return rc;
        *out_host = (double)count / (double)T;
        return IMM_OK;
    });
}

// ------------------------------------------------------------------ commitments from device memory
extern "C" int imm_commit_tables_device(imm_ctx* ctx, void* stream, int count, const imm_table_desc* tables,
                                        imm_commit1* out_host) {
    return guarded([&]() -> int {
        using namespace imm;
        if (!ctx || (count > 0 && (!tables || !out_host))) return IMM_E_NULL;
        if (count < 0) return IMM_E_SHAPE;
        if (count == 0) return IMM_OK;
        constexpr uint64_t kLeafBytes = 1ull << 20, kMaxLeaves = 1ull << 22;
        const uint64_t lim = 1ull << IMM_MAX_ROUNDS;
        std::vector<k::LeafDesc> leaves;
        std::vector<uint64_t> first(count + 1, 0);  // first[t]: index of table t's first leaf
        bool aligned16 = true;
        for (int t = 0; t < count; ++t) {
            const imm_table_desc& d = tables[t];
            if (!d.table_dev) return IMM_E_NULL;
            if (d.rows == 0 || d.cols == 0 || d.rows > lim || d.cols > lim) return IMM_E_SHAPE;
            const uint64_t elem = d.dtype == IMM_I8 ? 1 : d.dtype == IMM_I16 ? 2 : d.dtype == IMM_I64 ? 8 : 0;
            if (!elem) return IMM_E_DTYPE;
            const uintptr_t addr = reinterpret_cast<uintptr_t>(d.table_dev);
            if (addr % 4) return IMM_E_SHAPE;
            aligned16 = aligned16 && addr % 16 == 0;
            const uint64_t bytes = d.rows * d.cols * elem;  // < 2^53
            const uint64_t n = (bytes + kLeafBytes - 1) / kLeafBytes;
            first[t + 1] = first[t] + n;
            if (first[t + 1] > kMaxLeaves) return IMM_E_SHAPE;
            for (uint64_t i = 0; i < n; ++i)
                leaves.push_back({static_cast<const uint8_t*>(d.table_dev) + i * kLeafBytes,
                                  std::min(kLeafBytes, bytes - i * kLeafBytes)});
        }
        IMM_HIP(hipSetDevice(ctx->device));
        hipStream_t s = static_cast<hipStream_t>(stream);
        int rc;
        const size_t total = leaves.size();
        if ((rc = ctx->commit_leaves.ensure(sizeof(k::LeafDesc) * total))) return rc;
        if ((rc = ctx->commit_digests.ensure(32 * total))) return rc;
        // (the descriptors are in pageable memory: the copy has left `leaves` when the call returns)
        IMM_HIP(hipMemcpyAsync(ctx->commit_leaves.p, leaves.data(), sizeof(k::LeafDesc) * total, hipMemcpyHostToDevice, s));
        if ((rc = ctx->prof.begin(IMM_K_COMMIT, s))) return rc;
        IMM_HIP(k::commit_leaves(s, static_cast<const k::LeafDesc*>(ctx->commit_leaves.p), (uint32_t)total, aligned16,
                                 static_cast<uint8_t*>(ctx->commit_digests.p)));
        if ((rc = ctx->prof.end(IMM_K_COMMIT, s))) return rc;
        std::vector<uint8_t> digests(32 * total);
        IMM_HIP(hipMemcpyAsync(digests.data(), ctx->commit_digests.p, digests.size(), hipMemcpyDeviceToHost, s));
        IMM_HIP(hipStreamSynchronize(s));
        for (int t = 0; t < count; ++t) {
            const imm_table_desc& d = tables[t];
            Sha256 top;
            uint8_t hdr[13 + 4 + 8 + 8];
            std::memcpy(hdr, "IMM-COMMIT-v1", 13);
            for (int i = 0; i < 4; ++i) hdr[13 + i] = (uint8_t)(d.dtype >> (8 * i));
            for (int i = 0; i < 8; ++i) hdr[17 + i] = (uint8_t)(d.rows >> (8 * i));
            for (int i = 0; i < 8; ++i) hdr[25 + i] = (uint8_t)(d.cols >> (8 * i));
            top.update(hdr, sizeof(hdr));
            top.update(digests.data() + 32 * first[t], 32 * (size_t)(first[t + 1] - first[t]));
            top.finish(out_host[t].digest);
            out_host[t].rows = d.rows;
            out_host[t].cols = d.cols;
            out_host[t].dtype = d.dtype;
            out_host[t]._pad = 0;
        }
        return ctx->prof.mask ? ctx->prof.flush() : IMM_OK;
    });
}
