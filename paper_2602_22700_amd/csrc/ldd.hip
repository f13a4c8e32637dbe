// gfx950 kernels for the logit-distance step of the audit: total-variation and KL distance of
// two softmax distributions (paper section 4.3), the top-K distance (paper appendix on the
// verification of top-K) and the tail density p(t1) (section 5.3).
//
// A row of a 128k vocabulary is 512 KiB per operand and every logit is needed once, so all of these
// are streaming reductions bound by HBM.  The softmax distances cut a row into chunks, one workgroup
// per chunk, which hold their part of both rows in registers until the row's statistics are known;
// the top-K distance takes one workgroup of 1024 threads per row and finds the few largest logits
// without a sort.  Each logit is read from memory once.
#include "ldd.h"

#include <math.h>

namespace imm {
namespace k {
namespace {

constexpr int kLddBlock = 1024;

typedef float v4f __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------ TV and KL
// A row pair of a 128k vocabulary is 1 MiB and a few hundred workgroups are resident at a time, so
// with a workgroup per row far more than the caches hold is in flight, and every further pass over
// a row comes from HBM again.  Here a row is cut into chunks of 16384 logits, one workgroup per
// chunk, and a workgroup keeps its part of both rows in registers from the first load to the end,
// so each logit is read from memory once:
//
//   1. chunk maxima mx_c, my_c, then Z_c = sum e^(x - mx_c), Z'_c = sum e^(y - my_c) and
//      W_c = sum e^(x - mx_c) (x - y), written to the slot of (row, chunk); the workgroup counts
//      itself in on the row (TV only).
//   2. merge, one chunk per lane: mx = max mx_c, Z = sum Z_c e^(mx_c - mx), likewise Z', W, and
//      KL = W/Z - (mx + log Z) + (my + log Z').  For the KL that is returned this is done by a small
//      second kernel, one wave per row; if only KL is wanted, steps 1 and 2 are all there is, and the
//      first kernel is a plain streaming pass.
//   3. if TV is wanted, the workgroup that counted in last on a row merges as well, right away, and
//      posts mx, my, 1/Z, 1/Z' for the row; the other workgroups of the row wait for that post.  By
//      then the registers hold e^(x - mx_c) and e^(y - my_c) in place of the logits, so a workgroup
//      only scales them by alpha_c = e^(mx_c - mx)/Z and beta_c = e^(my_c - my)/Z' and sums
//      |alpha_c e^(x - mx_c) - beta_c e^(y - my_c)|.  The parts of a row are added up as fixed-point
//      numbers by one integer atomic add each (integer addition gives the same total in any order)
//      that nobody waits for; the second kernel turns the total into TV and leaves slots, counters,
//      sums and posts as they were found, for the next call.
//
// The wait in step 3 is bounded.  The chunks of a row have neighbouring workgroup ids, the hardware
// starts workgroups in id order, and none of them waits before it has counted in, so the post
// normally arrives within microseconds.  A workgroup whose wait runs out stops depending on the
// others: it works out the slots of all other chunks of its row itself and merges for itself (the
// same arithmetic on the same data gives the same bits, so writing them again is harmless).  Every
// workgroup therefore ends whatever the others do.
//
// Slots, counters and posts are written with agent-scope atomic stores (they go through to the
// level all XCDs share) and read with agent-scope atomic loads.  Nothing relies on the order in
// which such stores become visible: an empty word of a slot or a post is kNoPost, which no result
// can be, so every word says for itself whether it is there, and the workgroup that merges a row
// looks again until all words of all slots are (the count only tells it that they are on their
// way).  No cache-wide write-back or invalidate is involved, which is what a device-wide fence
// would cost here, tens of thousands of times per launch.
//
// Arithmetic: e^d for d <= 0 is the hardware base-2 exponential of d * log2(e), all in fp32:
// relative error at most about 2^-24 (2.3 |d| + 4) per term (rounding of d, of the product, of the
// constant, and of the exponential).  Four neighbouring terms are added in fp32, everything beyond
// that is accumulated in fp64, so the error of a sum stays that of its terms.  The factors
// e^(mx_c - mx) of the merge come from the same fp32 exponential where the result feeds TV (the
// fp64 library routine needs more registers than a workgroup that still holds its chunk can spare)
// and from the fp64 routine where it feeds KL.
constexpr float kLog2e = 1.44269504088896340736f;
// Few threads with many registers each: what a CU holds of the rows while its workgroups wait for
// their posts is what keeps HBM busy, and a thread's fixed register cost is paid once per thread.
constexpr int kTvBlock = 256;
constexpr int kTvWaves = kTvBlock / 64;
constexpr int kPerThreadVec = 64;     // logits of each row held by a thread: aligned rows (16-byte loads) ..
constexpr int kPerThreadScalar = 16;  // .. and the others (4-byte loads, one address each)
constexpr int kTvWavesPerSimd = 3;    // register budget of the aligned kernels: 512 / 3 per thread
constexpr float kAbsent = -3.402823466e38f;                 // stands in for positions past the row's end
constexpr int kXcds = 8;
constexpr uint64_t kNoPost = ~0ull;                         // "not there yet": a NaN pattern that no result takes
constexpr double kTvFixedOne = 4611686018427387904.0;       // 2^62

__device__ __forceinline__ float exp_nonpos(float d) { return __builtin_amdgcn_exp2f(d * kLog2e); }

// |ex/Z - ey/Z'| with both products rounded on their own (no fused multiply-add of one into the
// other), so that identical rows give exactly zero.
__device__ __forceinline__ float prob_gap(float ex, float izx, float ey, float izy) {
#pragma clang fp contract(off)
    const float px = ex * izx, py = ey * izy;
    return fabsf(px - py);
}

// The thread's PER logits of the chunk of row x that starts at logit `first` and has `len`
// (1 .. kTvBlock * PER) logits.  VEC (rows of a multiple of four logits, 16-byte aligned): groups of
// four neighbours, groups kTvBlock apart; otherwise single logits kTvBlock apart.  Positions >= len
// read as kAbsent.  Addresses are the row pointer plus a 32-bit byte offset (rows of at most 2^30
// logits).  The loads are streaming: nobody reads the data again.
template <bool VEC, int PER>
__device__ __forceinline__ void load_chunk(const float* __restrict__ x, uint32_t first, uint32_t len, uint32_t tid,
                                           float (&v)[PER]) {
    const char* bytes = reinterpret_cast<const char*>(x);
    if (VEC) {
        if (len == kTvBlock * PER) {  // the same for the whole workgroup
#pragma unroll
            for (int j = 0; j < PER / 4; ++j) {
                const uint32_t i = 4 * (tid + kTvBlock * j);
                const v4f q = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(bytes + (first + i) * 4u));
                v[4 * j] = q.x; v[4 * j + 1] = q.y; v[4 * j + 2] = q.z; v[4 * j + 3] = q.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < PER / 4; ++j) {
                const uint32_t i = 4 * (tid + kTvBlock * j);
                const bool ok = i < len;  // len is a multiple of four
                const v4f q = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(bytes + (ok ? (first + i) * 4u : 0u)));
                v[4 * j] = ok ? q.x : kAbsent; v[4 * j + 1] = ok ? q.y : kAbsent;
                v[4 * j + 2] = ok ? q.z : kAbsent; v[4 * j + 3] = ok ? q.w : kAbsent;
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const uint32_t i = tid + kTvBlock * j;
            const bool ok = i < len;
            const float t = __builtin_nontemporal_load(reinterpret_cast<const float*>(bytes + (ok ? (first + i) * 4u : 0u)));
            v[j] = ok ? t : kAbsent;
        }
    }
}

__device__ __forceinline__ float wave_all_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ double wave_all_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// One slot per (row, chunk), 32 bytes: zx, zy, w as fp64 bit patterns, mx | my << 32 as fp32 bit patterns.
constexpr int kSlotWords = 4;
// One post per row: mx | my << 32, then 1/Z | 1/Z' << 32, fp32 bit patterns; kNoPost when empty.
constexpr int kPostWords = 2;

__device__ __forceinline__ void put(uint64_t* p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t peek(const uint64_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t never_empty(uint64_t v) { return v == kNoPost ? v - 1 : v; }  // still a NaN
__device__ __forceinline__ uint64_t bits(double v) { return never_empty((uint64_t)__double_as_longlong(v)); }
__device__ __forceinline__ double real(uint64_t v) { return __longlong_as_double((long long)v); }
__device__ __forceinline__ uint64_t pair(float lo, float hi) {
    return never_empty((uint64_t)__float_as_uint(lo) | ((uint64_t)__float_as_uint(hi) << 32));
}
__device__ __forceinline__ float lo_of(uint64_t v) { return __uint_as_float((uint32_t)v); }
__device__ __forceinline__ float hi_of(uint64_t v) { return __uint_as_float((uint32_t)(v >> 32)); }

// The count goes up; returns the old count.  The count is not ordered against the stores to the slot:
// whoever reads slots because of a count checks that every word is there.
__device__ __forceinline__ uint32_t count_in(uint32_t* counter) {
    return __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct TvShared {
    float wave_max[kTvWaves][2];
    double wave_sum[kTvWaves][3];
    uint64_t post[kPostWords];
};

// Step 1 for the chunk held in (a, b): every thread returns the chunk maxima, wave 0 returns the
// three sums in all its lanes, and with KEEP a, b are left holding e^(a - mx), e^(b - my).  Groups
// of four neighbouring terms are added in fp32; from there on the sums are fp64.  Two barriers.
template <bool KEEP, int PER>
__device__ __forceinline__ void chunk_stats(float (&a)[PER], float (&b)[PER], TvShared& sh, uint32_t lane, uint32_t wave,
                                            float& mx, float& my, double& zx, double& zy, double& w) {
    mx = a[0]; my = b[0];
#pragma unroll
    for (int j = 1; j < PER; ++j) { mx = fmaxf(mx, a[j]); my = fmaxf(my, b[j]); }
    mx = wave_all_max(mx);
    my = wave_all_max(my);
    if (lane == 0) { sh.wave_max[wave][0] = mx; sh.wave_max[wave][1] = my; }
    __syncthreads();
#pragma unroll
    for (int v = 0; v < kTvWaves; ++v) { mx = fmaxf(mx, sh.wave_max[v][0]); my = fmaxf(my, sh.wave_max[v][1]); }
    zx = 0; zy = 0; w = 0;
#pragma unroll
    for (int j = 0; j < PER; j += 4) {
        float sx = 0.f, sy = 0.f, sw = 0.f;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float ex = exp_nonpos(a[j + c] - mx), ey = exp_nonpos(b[j + c] - my);
            sx += ex; sy += ey; sw += ex * (a[j + c] - b[j + c]);   // absent positions: 0 * 0
            if (KEEP) { a[j + c] = ex; b[j + c] = ey; }
        }
        zx += sx; zy += sy; w += sw;
    }
    zx = wave_all_sum(zx);
    zy = wave_all_sum(zy);
    w = wave_all_sum(w);
    if (lane == 0) { sh.wave_sum[wave][0] = zx; sh.wave_sum[wave][1] = zy; sh.wave_sum[wave][2] = w; }
    __syncthreads();
    if (wave == 0) {
        const uint32_t src = lane < kTvWaves ? lane : 0;
        const double keep = lane < kTvWaves ? 1.0 : 0.0;
        zx = wave_all_sum(keep * sh.wave_sum[src][0]);
        zy = wave_all_sum(keep * sh.wave_sum[src][1]);
        w = wave_all_sum(keep * sh.wave_sum[src][2]);
    }
}

__device__ __forceinline__ void put_stats(uint64_t* slot, float mx, float my, double zx, double zy, double w) {
    put(slot + 0, bits(zx));
    put(slot + 1, bits(zy));
    put(slot + 2, bits(w));
    put(slot + 3, pair(mx, my));
}

// Step 2, by one wave: lane c takes chunk c (then c + 64, ... for rows of more than 64 chunks, merging
// as it goes), then the lanes merge.  All loads of a chunk's slot are issued together.  EXACT takes the
// factors e^(mx_c - mx) from the fp64 library exponential, otherwise from the fp32 one.
template <bool EXACT>
__device__ __forceinline__ double merge_factor(float d) {
    return EXACT ? exp((double)d) : (double)exp_nonpos(d);
}
// Returns whether every word of every slot of the row was there (the same answer in all lanes).
template <bool EXACT>
__device__ __forceinline__ bool merge_row(const uint64_t* slots, uint32_t S, uint32_t lane, float& gx, float& gy,
                                          double& Zx, double& Zy, double& W) {
    float lx = -INFINITY, ly = -INFINITY;
    double zx = 0, zy = 0, w = 0;
    bool there = true;
    for (uint32_t c = lane; c < S; c += 64) {
        const uint64_t m = peek(slots + c * kSlotWords + 3), w0 = peek(slots + c * kSlotWords + 0),
                       w1 = peek(slots + c * kSlotWords + 1), w2 = peek(slots + c * kSlotWords + 2);
        there = there && m != kNoPost && w0 != kNoPost && w1 != kNoPost && w2 != kNoPost;
        const double cx = real(w0), cy = real(w1), cw = real(w2);
        const float nx = fmaxf(lx, lo_of(m)), ny = fmaxf(ly, hi_of(m));
        const double ox = merge_factor<EXACT>(lx - nx), oy = merge_factor<EXACT>(ly - ny);  // e^(-inf) = 0 at first
        const double fx = merge_factor<EXACT>(lo_of(m) - nx), fy = merge_factor<EXACT>(hi_of(m) - ny);
        zx = zx * ox + cx * fx;
        w = w * ox + cw * fx;
        zy = zy * oy + cy * fy;
        lx = nx; ly = ny;
    }
    gx = wave_all_max(lx);
    gy = wave_all_max(ly);
    const double fx = merge_factor<EXACT>(lx - gx), fy = merge_factor<EXACT>(ly - gy);  // lanes without a chunk: 0
    Zx = wave_all_sum(zx * fx);
    Zy = wave_all_sum(zy * fy);
    W = wave_all_sum(w * fx);
    return __all(there);
}

template <bool VEC, bool WANT_TV>
__global__ __launch_bounds__(kTvBlock, VEC ? kTvWavesPerSimd : 4) void ldd_tv_kl_kernel(
    const float* __restrict__ X, const float* __restrict__ Y, uint32_t T, uint32_t n, uint64_t ld, uint32_t S,
    uint64_t* slots_all, uint64_t* posts, uint64_t* sums, uint32_t* counters, uint64_t wait_polls) {
    constexpr int PER = VEC ? kPerThreadVec : kPerThreadScalar;
    constexpr uint32_t kChunk = kTvBlock * PER;  // logits of a row per workgroup
    __shared__ TvShared sh;
    // Consecutive workgroup ids go round the XCDs: id % 8 names the XCD, and within an XCD the ids
    // walk through the chunks of one row before they move on to the next.
    const uint32_t xcd = blockIdx.x % kXcds, slot_in_xcd = blockIdx.x / kXcds;
    const uint32_t row = (slot_in_xcd / S) * kXcds + xcd, chunk = slot_in_xcd % S;
    if (row >= T) return;  // the whole workgroup: T need not be a multiple of 8
    const float* x = X + (uint64_t)row * ld;
    const float* y = Y + (uint64_t)row * ld;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint64_t* slots = slots_all + (uint64_t)row * S * kSlotWords;
    auto chunk_len = [&](uint32_t c) { return n - c * kChunk < kChunk ? n - c * kChunk : kChunk; };

    // ---- step 1
    float a[PER], b[PER], mx, my;
    double zx, zy, w;
    load_chunk<VEC>(x, chunk * kChunk, chunk_len(chunk), tid, a);
    load_chunk<VEC>(y, chunk * kChunk, chunk_len(chunk), tid, b);
    chunk_stats<WANT_TV>(a, b, sh, lane, wave, mx, my, zx, zy, w);

    if (!WANT_TV) {  // KL only: the slot is all the finishing kernel needs
        if (tid == 0) put_stats(slots + chunk * kSlotWords, mx, my, zx, zy, w);
        return;
    }

    // ---- steps 2 and 3: count in; the last one merges and posts, the others wait (bounded) for the post
    uint64_t* post = posts + (uint64_t)row * kPostWords;
    float rmx = mx, rmy = my;  // the maxima that a, b refer to
    if (wave == 0) {
        uint32_t before = 0;
        if (lane == 0) {
            put_stats(slots + chunk * kSlotWords, mx, my, zx, zy, w);
            before = count_in(counters + row);
        }
        before = __shfl(before, 0, 64);
        uint64_t p0 = kNoPost, p1 = kNoPost;
        if (before == S - 1) {
            // everybody has counted in; the words of their slots may still be on their way
            float gx, gy;
            double Zx, Zy, W;
            bool there = false;
            for (uint64_t polls = 0; polls <= wait_polls && !there; ++polls)
                there = merge_row<false>(slots, S, lane, gx, gy, Zx, Zy, W);
            if (there) {
                p0 = pair(gx, gy);
                p1 = pair(1.0f / (float)Zx, 1.0f / (float)Zy);
                if (lane == 0) { put(post + 0, p0); put(post + 1, p1); }
            }
        } else if (lane == 0) {
            for (uint64_t polls = 0; polls < wait_polls; ++polls) {
                p0 = peek(post + 0);
                p1 = peek(post + 1);
                if (p0 != kNoPost && p1 != kNoPost) break;
                __builtin_amdgcn_s_sleep(8);
            }
        }
        if (lane == 0) { sh.post[0] = p0; sh.post[1] = p1; }
    }
    __syncthreads();
    if (sh.post[0] == kNoPost || sh.post[1] == kNoPost) {  // the wait ran out: do without the others
        __syncthreads();  // everybody has read sh.post
        for (uint32_t c = 0; c < S; ++c) {
            if (c == chunk) continue;
            load_chunk<VEC>(x, c * kChunk, chunk_len(c), tid, a);
            load_chunk<VEC>(y, c * kChunk, chunk_len(c), tid, b);
            chunk_stats<false>(a, b, sh, lane, wave, mx, my, zx, zy, w);
            if (tid == 0) put_stats(slots + c * kSlotWords, mx, my, zx, zy, w);
        }
        if (wave == 0) {
            if (lane == 0) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_s_waitcnt(0);
            }
            __builtin_amdgcn_wave_barrier();
            float gx, gy;
            double Zx, Zy, W;
            merge_row<false>(slots, S, lane, gx, gy, Zx, Zy, W);
            if (lane == 0) {
                sh.post[0] = pair(gx, gy);
                sh.post[1] = pair(1.0f / (float)Zx, 1.0f / (float)Zy);
                put(post + 0, sh.post[0]);  // the same bits whoever posts
                put(post + 1, sh.post[1]);
            }
        }
        load_chunk<VEC>(x, chunk * kChunk, chunk_len(chunk), tid, a);
        load_chunk<VEC>(y, chunk * kChunk, chunk_len(chunk), tid, b);
        chunk_stats<true>(a, b, sh, lane, wave, rmx, rmy, zx, zy, w);  // its barriers come after the write of sh.post
    }
    const float alpha = exp_nonpos(rmx - lo_of(sh.post[0])) * lo_of(sh.post[1]);
    const float beta = exp_nonpos(rmy - hi_of(sh.post[0])) * hi_of(sh.post[1]);
    double tv = 0;
#pragma unroll
    for (int j = 0; j < PER; j += 4) {
        float st = 0.f;
#pragma unroll
        for (int c = 0; c < 4; ++c) st += prob_gap(a[j + c], alpha, b[j + c], beta);
        tv += st;
    }
    tv = wave_all_sum(tv);
    if (lane == 0) sh.wave_sum[wave][0] = tv;   // everybody is past the reads of wave_sum in chunk_stats
    __syncthreads();
    if (wave == 0) {
        tv = wave_all_sum(lane < kTvWaves ? sh.wave_sum[lane < kTvWaves ? lane : 0][0] : 0.0);
        // The part, at most 1, goes onto the row's sum as a fixed-point number with 62 fraction bits.
        // Nobody here needs the result, so the workgroup does not wait for it.
        if (lane == 0)
            (void)__hip_atomic_fetch_add(sums + row, (uint64_t)__double2ll_rn(tv * kTvFixedOne), __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
    }
}

// The end of a row, one wave per row, after the kernel above has ended: KL from the slots (step 2
// with the fp64 factors), TV from the fixed-point sum, and posts, sums and counters back to the
// state they were found in, for the next call.
__global__ __launch_bounds__(256) void ldd_finish_kernel(uint32_t T, uint32_t S, uint64_t* slots_all, uint64_t* posts,
                                                         uint64_t* sums, uint32_t* counters, double* __restrict__ tv_out,
                                                         double* __restrict__ kl_out) {
    const uint32_t row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= T) return;
    uint64_t* slots = slots_all + (uint64_t)row * S * kSlotWords;
    if (kl_out) {
        float gx, gy;
        double Zx, Zy, W;
        merge_row<true>(slots, S, lane, gx, gy, Zx, Zy, W);
        if (lane == 0) kl_out[row] = W / Zx - ((double)gx + log(Zx)) + ((double)gy + log(Zy));
    }
    for (uint32_t c = lane; c < S; c += 64)  // the lane that read a slot is the one that clears it
        for (int k = 0; k < kSlotWords; ++k) put(slots + c * kSlotWords + k, kNoPost);
    if (tv_out && lane == 0) {
        tv_out[row] = 0.5 * ((double)peek(sums + row) / kTvFixedOne);
        put(sums + row, 0);
        put(posts + (uint64_t)row * kPostWords, kNoPost);
        put(posts + (uint64_t)row * kPostWords + 1, kNoPost);
        __hip_atomic_store(counters + row, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

__global__ void fill_u64_kernel(uint64_t* p, uint64_t count, uint64_t v) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = v;
}

__global__ void fill_u32_kernel(uint32_t* p, uint64_t count, uint32_t v) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = v;
}

// ------------------------------------------------------------------ top-K distance
// With v_1 >= .. >= v_K the K largest logits outside I and w_1 .. w_K the logits of I, the cost of
// a threshold t >= v_K is f(t) = sum_j max(v_j - t, 0) + sum_i max(t - w_i, 0); below v_K the cost
// cannot decrease (at least K non-members lie above t, at most K members below), and f is piecewise
// linear, so the minimum is attained at one of the 2K values.  The K largest non-members are among
// the 2K largest logits of the row.  Those are found without sorting the row: every thread keeps
// the maximum of its own (strided) share while the row streams in from HBM; if tau is the 2K-th
// largest of the 16 r thread maxima that are the r largest of each of the 16 waves (16 r >= 2K), then
// at least 2K logits are >= tau, and only threads whose maximum reaches tau can hold such logits.  A thread
// also keeps its second largest logit and the place of the largest, so that it can tell whether it
// holds one such logit (then it knows which) or more (then its share is read again, which is rare:
// a share is scattered over the row, so reading it again touches a cache line per four logits).
constexpr int kTopkCap = 1024;  // candidate list capacity; beyond it the slow exact path is taken

// A logit and its place as one sortable word: of two keys the larger comes first (the larger logit;
// of equal logits the one with the smaller index; any fixed rule works, values decide the cost).
// The upper half is monotone in v for every v that is not a NaN, and never zero; key 0 is "nothing".
__device__ __forceinline__ uint64_t cand_key(float v, uint32_t idx) {
    const uint32_t u = __float_as_uint(v);
    const uint32_t ord = u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
    return (uint64_t)ord << 32 | (uint32_t)~idx;
}
__device__ __forceinline__ float key_value(uint64_t key) {
    const uint32_t ord = (uint32_t)(key >> 32);
    return __uint_as_float(ord ^ ((ord >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

// the slow path's order: larger value first; equal values: smaller index first
__device__ __forceinline__ bool cand_before(float va, int ia, float vb, int ib) {
    return va > vb || (va == vb && ia < ib);
}

// Workgroup shape of the top-K kernel: one row per workgroup, two workgroups per compute unit (while
// one ranks its candidates the other streams).
constexpr int kTopkBlock = 1024;
constexpr int kTopkWaves = kTopkBlock / 64;
constexpr int kTopkLoads = 8;           // 16-byte loads in flight per thread
constexpr int kTopkWavesPerSimd = 8;    // at most 64 registers

template <bool VEC>
__global__ __launch_bounds__(kTopkBlock, kTopkWavesPerSimd) void topk_distance_kernel(
    const float* __restrict__ X, uint64_t n, uint64_t ld, const int32_t* __restrict__ idx_all, uint32_t K,
    double* __restrict__ out) {
    __shared__ uint64_t tops[2 * IMM_TOPK_MAX + kTopkWaves];  // the r largest thread maxima of every wave, as keys
    __shared__ int member_idx[IMM_TOPK_MAX];
    __shared__ float member_val[IMM_TOPK_MAX];
    __shared__ uint64_t member_key[IMM_TOPK_MAX];  // key of a member on the candidate list, else 0
    __shared__ float top_out[IMM_TOPK_MAX];        // K largest non-members
    __shared__ uint64_t cand[kTopkCap];            // keys of the logits >= tau
    __shared__ unsigned short hot[kTopkBlock];      // threads whose share holds more than one of them
    __shared__ int hot_count;
    __shared__ int cand_count;
    __shared__ int bad_row;
    __shared__ double wave_best[kTopkWaves];
    __shared__ float slow_v[kTopkWaves];
    __shared__ int slow_i[kTopkWaves];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint64_t n4 = VEC ? n >> 2 : 0;
    // a row with fewer than 2K entries has fewer than K non-members: then every entry is accounted for
    const uint32_t Kn = (n - K < K) ? (uint32_t)(n - K) : K;

    const uint64_t row = blockIdx.x;
    const float* x = X + row * ld;
    const int32_t* idx = idx_all + row * K;
    if (tid == 0) { cand_count = 0; hot_count = 0; bad_row = 0; }
    __syncthreads();
    if (tid < K) {
        const int id = idx[tid];
        member_idx[tid] = id;
        if (id < 0 || (uint64_t)id >= n) {
            bad_row = 1;
            member_val[tid] = 0.f;
        } else {
            member_val[tid] = x[id];
        }
    }
    __syncthreads();
    if (tid < K)
        for (uint32_t j = 0; j < tid; ++j)
            if (member_idx[j] == member_idx[tid]) bad_row = 1;

    // pass 1 (HBM): the two largest logits of the thread's share and where the largest one sits,
    // kTopkLoads loads in flight per thread.  A position is a group of four (VEC), one of the up to
    // three logits after the last whole group (VEC, numbered from n4 on), or a single logit.
    float tmax = -INFINITY, second = -INFINITY;
    uint32_t at = 0;
    auto take = [&](float v) { second = __builtin_amdgcn_fmed3f(tmax, second, v); tmax = fmaxf(tmax, v); };
    auto take4 = [&](const v4f& q, uint64_t pos) {
        const float before = tmax;
        take(q.x); take(q.y); take(q.z); take(q.w);
        at = tmax > before ? (uint32_t)pos : at;
    };
    uint64_t g = tid;
    for (; g + (kTopkLoads - 1) * (uint64_t)kTopkBlock < n4; g += kTopkLoads * (uint64_t)kTopkBlock) {
        v4f q[kTopkLoads];
#pragma unroll
        for (int j = 0; j < kTopkLoads; ++j)
            q[j] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(x + 4 * (g + (uint64_t)kTopkBlock * j)));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < kTopkLoads; ++j) take4(q[j], g + (uint64_t)kTopkBlock * j);
    }
    for (; g < n4; g += kTopkBlock) take4(*reinterpret_cast<const v4f*>(x + 4 * g), g);
    for (uint64_t i = 4 * n4 + tid; i < n; i += kTopkBlock) {
        const float before = tmax;
        take(x[i]);
        at = tmax > before ? (uint32_t)(VEC ? n4 + (i - 4 * n4) : i) : at;
    }

    // the r largest thread maxima of this wave (ties between lanes broken by lane number), 16 r >= 2K
    const uint32_t r = (2 * K + kTopkWaves - 1) / kTopkWaves;
    float cur = tmax;     // candidates still in play in this lane
    for (uint32_t it = 0; it < r; ++it) {
        float m = cur;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        if (lane == 0) tops[wave * r + it] = cand_key(m, wave * r + it);
        // retire exactly one lane holding m
        const uint64_t holders = __ballot(cur == m);
        const uint32_t first = (uint32_t)__builtin_ctzll(holders);
        if (lane == first) cur = -INFINITY;
    }
    __syncthreads();
    // tau = the 2K-th largest of these 16 r thread maxima (every wave works it out for itself: a lane
    // counts how many of them come before its own one or two)
    const uint32_t V = kTopkWaves * r;
    const uint64_t mine0 = lane < V ? tops[lane] : 0, mine1 = lane + 64 < V ? tops[lane + 64] : 0;
    uint32_t before0 = 0, before1 = 0;
#pragma unroll 8
    for (uint32_t j = 0; j < V; ++j) {
        const uint64_t other = tops[j];
        before0 += other > mine0 ? 1u : 0u;
        before1 += other > mine1 ? 1u : 0u;
    }
    const uint64_t hit0 = __ballot(lane < V && before0 == 2 * K - 1);
    const uint64_t hit1 = __ballot(lane + 64 < V && before1 == 2 * K - 1);
    const uint64_t tau_key = hit0 ? __shfl(mine0, (int)__builtin_ctzll(hit0), 64)
                                  : __shfl(mine1, (int)__builtin_ctzll(hit1 | (1ull << 63)), 64);
    const float tau = key_value(tau_key);

    // pass 2: only threads whose maximum reaches tau can own a logit >= tau.  Most of them own just
    // that one (their second largest is below tau) and know where it sits, up to its place in a group
    // of four.  The few that own more put their names on a list, and the whole workgroup goes through
    // the shares of the listed threads together, one (owner, position) pair per thread at a time.  All
    // these reads are in flight together: the second look at the row costs one round trip.
    auto push = [&](float v, uint64_t where) {
        const int slot = atomicAdd(&cand_count, 1);
        if (slot < kTopkCap) cand[slot] = cand_key(v, (uint32_t)where);
    };
    const bool reaches = tmax >= tau;
    const bool crowded = reaches && second >= tau;
    if (crowded) hot[atomicAdd(&hot_count, 1)] = (unsigned short)tid;
    // a member is on the candidate list exactly when its logit reaches tau
    if (tid < K) member_key[tid] = member_val[tid] >= tau ? cand_key(member_val[tid], (uint32_t)member_idx[tid]) : 0;
    __syncthreads();
    const bool alone = reaches && !crowded;
    if constexpr (VEC) {
        v4f own = {};
        if (alone && at < n4) own = *reinterpret_cast<const v4f*>(x + 4 * (uint64_t)at);
        const uint64_t tail_i = 4 * n4 + tid;  // the up to three logits after the last whole group
        const float tail_v = tail_i < n && hot_count ? x[tail_i] : -INFINITY;
        const uint64_t per_owner = (n4 + kTopkBlock - 1) / kTopkBlock;
        const uint64_t items = (uint64_t)hot_count * per_owner;
        for (uint64_t w = tid; w < items; w += kTopkBlock) {
            const uint32_t owner = hot[w / per_owner];
            const uint64_t u = owner + (uint64_t)kTopkBlock * (w % per_owner);
            if (u >= n4) continue;
            const v4f q = *reinterpret_cast<const v4f*>(x + 4 * u);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (q[j] >= tau) push(q[j], 4 * u + j);
        }
        // a listed thread's share of the last logits (a thread not listed knows where its only one sits)
        if (tail_v >= tau) {
            bool listed = false;
            for (int h = 0; h < hot_count; ++h) listed |= hot[h] == tid;
            if (listed) push(tail_v, tail_i);
        }
        if (alone) {
            if (at < n4)
                push(tmax, 4 * (uint64_t)at + (own.x == tmax ? 0 : own.y == tmax ? 1 : own.z == tmax ? 2 : 3));
            else
                push(tmax, 4 * n4 + (at - n4));
        }
    } else {
        const uint64_t per_owner = (n + kTopkBlock - 1) / kTopkBlock;
        const uint64_t items = (uint64_t)hot_count * per_owner;
        for (uint64_t w = tid; w < items; w += kTopkBlock) {
            const uint64_t i = hot[w / per_owner] + (uint64_t)kTopkBlock * (w % per_owner);
            if (i >= n) continue;
            const float v = x[i];
            if (v >= tau) push(v, i);
        }
        if (alone) push(tmax, at);
    }
    __syncthreads();
    const int c = cand_count;

    if (c <= kTopkCap) {
        // Rank of every candidate among the candidates that are not members: the number of keys ahead of
        // its own on the list, less the number of members' keys ahead of it; ranks < Kn are the answer.
        // `per` neighbouring lanes share the comparisons of one candidate.
        uint32_t per = 1;
        while (per < 64 && 2 * per * (uint32_t)c <= (uint32_t)kTopkBlock) per *= 2;
        for (uint32_t base = 0; base < (uint32_t)c; base += kTopkBlock / per) {
            const uint32_t i = base + tid / per, sub = tid % per;
            const uint64_t mine = i < (uint32_t)c ? cand[i] : 0;
            uint32_t ahead = 0, members_ahead = 0, is_member = 0;
#pragma unroll 4
            for (uint32_t j = sub; j < (uint32_t)c; j += per) ahead += cand[j] > mine ? 1u : 0u;
#pragma unroll 4
            for (uint32_t j = sub; j < K; j += per) {
                const uint64_t mk = member_key[j];
                members_ahead += mk > mine ? 1u : 0u;
                is_member |= mk == mine ? 1u : 0u;
            }
            for (uint32_t off = per >> 1; off > 0; off >>= 1) {
                ahead += __shfl_xor(ahead, off, 64);
                members_ahead += __shfl_xor(members_ahead, off, 64);
                is_member |= __shfl_xor(is_member, off, 64);
            }
            const uint32_t rank = ahead - members_ahead;
            if (i < (uint32_t)c && sub == 0 && !is_member && rank < Kn) top_out[rank] = key_value(mine);
        }
    } else {
        // More logits tie at (or crowd above) tau than the list holds: exact but slow path, K rounds
        // of "largest non-member after the previous pick", each a scan of the whole row.
        float last_v = INFINITY;
        int last_i = -1;
        for (uint32_t pick = 0; pick < Kn; ++pick) {
            float bv = -INFINITY;
            int bi = 0x7FFFFFFF;
            for (uint64_t i = tid; i < n; i += kTopkBlock) {
                const float v = x[i];
                if (!cand_before(last_v, last_i, v, (int)i)) continue;       // already picked or before it
                bool is_member = false;
                for (uint32_t j = 0; j < K; ++j) is_member |= (member_idx[j] == (int)i);
                if (is_member) continue;
                if (cand_before(v, (int)i, bv, bi)) { bv = v; bi = (int)i; }
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                const float ov = __shfl_xor(bv, off, 64);
                const int oi = __shfl_xor(bi, off, 64);
                if (cand_before(ov, oi, bv, bi)) { bv = ov; bi = oi; }
            }
            __syncthreads();  // the previous pick's scratch has been read by everyone
            if (lane == 0) { slow_v[wave] = bv; slow_i[wave] = bi; }
            __syncthreads();
            bv = slow_v[0]; bi = slow_i[0];
            for (int w = 1; w < kTopkWaves; ++w)
                if (cand_before(slow_v[w], slow_i[w], bv, bi)) { bv = slow_v[w]; bi = slow_i[w]; }
            if (tid == 0) top_out[pick] = bv;
            last_v = bv;
            last_i = bi;
        }
    }
    __syncthreads();

    // Cost of each candidate threshold (with K non-members in hand, thresholds below v_K are never
    // better).  Lane l holds v_l and w_l; the waves share out the 2K thresholds, each a sum over the lanes.
    const bool has_v = lane < Kn, has_w = lane < K;
    const double v_l = has_v ? (double)top_out[lane] : 0.0;
    const double w_l = has_w ? (double)member_val[lane] : 0.0;
    double best = INFINITY;
    for (uint32_t t_ix = wave; t_ix < 2 * K; t_ix += kTopkWaves) {
        if (t_ix < K && t_ix >= Kn) continue;
        const float t = t_ix < K ? top_out[t_ix] : member_val[t_ix - K];
        if (Kn == K && t < top_out[K - 1]) continue;
        const double f = (has_v ? fmax(v_l - (double)t, 0.0) : 0.0) + (has_w ? fmax((double)t - w_l, 0.0) : 0.0);
        best = fmin(best, wave_all_sum(f));
    }
    if (lane == 0) wave_best[wave] = best;
    __syncthreads();
    if (wave == 0) {
        best = lane < kTopkWaves ? wave_best[lane] : INFINITY;
#pragma unroll
        for (int off = kTopkWaves / 2; off > 0; off >>= 1) best = fmin(best, __shfl_xor(best, off, 64));
        if (lane == 0) out[row] = bad_row ? (double)NAN : best;
    }
}

// ------------------------------------------------------------------ tail density
__global__ __launch_bounds__(kLddBlock) void tail_count_kernel(const double* __restrict__ dist, uint64_t T, double t1,
                                                               unsigned long long* __restrict__ count) {
    unsigned long long local = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * kLddBlock + threadIdx.x; i < T; i += (uint64_t)gridDim.x * kLddBlock)
        local += dist[i] > t1 ? 1ull : 0ull;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) local += __shfl_down(local, off, 64);
    if ((threadIdx.x & 63) == 0 && local) atomicAdd(count, local);
}

__global__ void clear_count_kernel(unsigned long long* count) { *count = 0; }

bool vec_ok(const void* p, uint64_t ld) { return reinterpret_cast<uintptr_t>(p) % 16 == 0 && ld % 4 == 0; }

}  // namespace

uint32_t ldd_chunks(uint64_t n, bool vec) {
    const uint64_t chunk = (uint64_t)kTvBlock * (vec ? kPerThreadVec : kPerThreadScalar);
    return (uint32_t)((n + chunk - 1) / chunk);
}
size_t ldd_slot_bytes(uint64_t T, uint64_t n) { return (size_t)T * ldd_chunks(n, false) * kSlotWords * sizeof(uint64_t); }
size_t ldd_post_bytes(uint64_t T) { return (size_t)T * kPostWords * sizeof(uint64_t); }
size_t ldd_sum_bytes(uint64_t T) { return (size_t)T * sizeof(uint64_t); }
size_t ldd_counter_bytes(uint64_t T) { return (size_t)T * sizeof(uint32_t); }

hipError_t ldd_init_sync(hipStream_t stream, uint64_t* slots, size_t slot_bytes, uint64_t* posts, size_t post_bytes,
                         uint64_t* sums, size_t sum_bytes, uint32_t* counters, size_t counter_bytes) {
    const uint64_t nl = slot_bytes / sizeof(uint64_t), np = post_bytes / sizeof(uint64_t),
                   ns = sum_bytes / sizeof(uint64_t), nc = counter_bytes / sizeof(uint32_t);
    hipLaunchKernelGGL(fill_u64_kernel, dim3((unsigned)((nl + 255) / 256)), dim3(256), 0, stream, slots, nl, kNoPost);
    hipLaunchKernelGGL(fill_u64_kernel, dim3((unsigned)((np + 255) / 256)), dim3(256), 0, stream, posts, np, kNoPost);
    hipLaunchKernelGGL(fill_u64_kernel, dim3((unsigned)((ns + 255) / 256)), dim3(256), 0, stream, sums, ns, 0ull);
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((nc + 255) / 256)), dim3(256), 0, stream, counters, nc, 0u);
    return hipGetLastError();
}

hipError_t ldd_tv_kl(hipStream_t stream, const float* X, const float* Y, uint64_t T, uint64_t n, uint64_t ld,
                     uint64_t* slots, uint64_t* posts, uint64_t* sums, uint32_t* counters, uint64_t wait_polls,
                     double* tv_out, double* kl_out) {
    const bool vec = n % 4 == 0 && vec_ok(X, ld) && vec_ok(Y, ld);
    const uint32_t S = ldd_chunks(n, vec);
    const uint64_t blocks = (T + kXcds - 1) / kXcds * kXcds * S;
    if (blocks > 0x7FFFFFFFull || n > (1ull << 30)) return hipErrorInvalidValue;
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kTvBlock), 0, stream, X, Y, (uint32_t)T, (uint32_t)n, ld,
                           S, slots, posts, sums, counters, wait_polls);
    };
    if (vec && tv_out) launch(ldd_tv_kl_kernel<true, true>);
    else if (vec) launch(ldd_tv_kl_kernel<true, false>);
    else if (tv_out) launch(ldd_tv_kl_kernel<false, true>);
    else launch(ldd_tv_kl_kernel<false, false>);
    hipLaunchKernelGGL(ldd_finish_kernel, dim3((unsigned)((T + 3) / 4)), dim3(256), 0, stream, (uint32_t)T, S, slots,
                       posts, sums, counters, tv_out, kl_out);
    return hipGetLastError();
}

hipError_t topk_distance(hipStream_t stream, const float* X, uint64_t T, uint64_t n, uint64_t ld, const int32_t* idx,
                         uint32_t K, double* out) {
    if (T == 0) return hipSuccess;
    if (n >= 4 && vec_ok(X, ld))
        hipLaunchKernelGGL((topk_distance_kernel<true>), dim3((unsigned)T), dim3(kTopkBlock), 0, stream, X, n, ld, idx, K,
                           out);
    else
        hipLaunchKernelGGL((topk_distance_kernel<false>), dim3((unsigned)T), dim3(kTopkBlock), 0, stream, X, n, ld, idx,
                           K, out);
    return hipGetLastError();
}

hipError_t tail_count(hipStream_t stream, const double* dist, uint64_t T, double t1, unsigned long long* count_dev) {
    hipLaunchKernelGGL(clear_count_kernel, dim3(1), dim3(1), 0, stream, count_dev);
    uint64_t blocks = (T + kLddBlock - 1) / kLddBlock;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(tail_count_kernel, dim3((unsigned)blocks), dim3(kLddBlock), 0, stream, dist, T, t1, count_dev);
    return hipGetLastError();
}

}  // namespace k
}  // namespace imm
