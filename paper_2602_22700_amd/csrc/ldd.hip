// gfx950 kernels for the logit-distance step of the audit: total-variation and KL distance of
// two softmax distributions (paper section 4.3), the top-K distance (paper appendix on the
// verification of top-K) and the tail density p(t1) (section 5.3).
//
// One workgroup of 1024 threads owns one decision step (one row of the logits).  A row of a
// 128k vocabulary is 512 KiB per operand, so the kernels are HBM-bound: each row is streamed
// from HBM once; whatever has to be looked at a second time is re-read right away, in reverse
// order, while it is still in the caches.
#include "ldd.h"

#include <math.h>

namespace imm {
namespace k {
namespace {

constexpr int kLddBlock = 1024;
constexpr int kLddWaves = kLddBlock / 64;

typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max_f32(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_down(v, off, 64));
    return v;
}

// Block-wide max / sum, result broadcast to every thread.  `lds` holds kLddWaves entries.
__device__ __forceinline__ float block_max(float v, float* lds) {
    v = wave_max_f32(v);
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = lds[0];
#pragma unroll
    for (int w = 1; w < kLddWaves; ++w) r = fmaxf(r, lds[w]);
    __syncthreads();
    return r;
}
__device__ __forceinline__ double block_sum(double v, double* lds) {
    v = wave_sum_f64(v);
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = lds[0];
#pragma unroll
    for (int w = 1; w < kLddWaves; ++w) r += lds[w];
    __syncthreads();
    return r;
}

// ------------------------------------------------------------------ TV and KL
// Pass 1 (HBM): row maxima.  Pass 2 (cache, reverse order): Z = sum e^(x-mx), Z' = sum e^(y-my)
// and W = sum e^(x-mx) (x - y), which give KL = W/Z - (mx + log Z) + (my + log Z').
// Pass 3 (cache): TV = 1/2 sum |e^(x-mx)/Z - e^(y-my)/Z'|.
//
// Arithmetic: e^d for d = x - mx <= 0 is the hardware base-2 exponential of d * log2(e), all in
// fp32: relative error at most about 2^-24 (2.3 |d| + 4) per term (rounding of d, of the product,
// of the constant, and of the exponential).  Four neighbouring terms are added in fp32, everything
// beyond that is accumulated in fp64, so the error of a sum stays that of its terms.
constexpr float kLog2e = 1.44269504088896340736f;

__device__ __forceinline__ float exp_nonpos(float d) { return __builtin_amdgcn_exp2f(d * kLog2e); }

// |ex/Z - ey/Z'| with both products rounded on their own (no fused multiply-add of one into the
// other), so that identical rows give exactly zero.
__device__ __forceinline__ float prob_gap(float ex, float izx, float ey, float izy) {
#pragma clang fp contract(off)
    const float px = ex * izx, py = ey * izy;
    return fabsf(px - py);
}

template <bool VEC>
__global__ __launch_bounds__(kLddBlock) void ldd_tv_kl_kernel(const float* __restrict__ X, const float* __restrict__ Y,
                                                              uint64_t n, uint64_t ld, double* __restrict__ tv_out,
                                                              double* __restrict__ kl_out) {
    __shared__ float ldsf[kLddWaves];
    __shared__ double ldsd[kLddWaves];
    const float* x = X + (uint64_t)blockIdx.x * ld;
    const float* y = Y + (uint64_t)blockIdx.x * ld;
    const uint32_t tid = threadIdx.x;
    const uint64_t n4 = VEC ? n >> 2 : 0;  // whole float4 groups

    float mx = -INFINITY, my = -INFINITY;
    for (uint64_t g = tid; g < n4; g += kLddBlock) {
        v4f a = *reinterpret_cast<const v4f*>(x + 4 * g), b = *reinterpret_cast<const v4f*>(y + 4 * g);
        mx = fmaxf(mx, fmaxf(fmaxf(a.x, a.y), fmaxf(a.z, a.w)));
        my = fmaxf(my, fmaxf(fmaxf(b.x, b.y), fmaxf(b.z, b.w)));
    }
    for (uint64_t i = 4 * n4 + tid; i < n; i += kLddBlock) {
        mx = fmaxf(mx, x[i]);
        my = fmaxf(my, y[i]);
    }
    mx = block_max(mx, ldsf);
    my = block_max(my, ldsf);

    double zx = 0, zy = 0, w = 0;
    for (uint64_t i = 4 * n4 + tid; i < n; i += kLddBlock) {
        const float ex = exp_nonpos(x[i] - mx), ey = exp_nonpos(y[i] - my);
        zx += ex; zy += ey; w += ex * (x[i] - y[i]);
    }
    for (uint64_t k = tid; k < n4; k += kLddBlock) {
        const uint64_t g = n4 - 1 - k;  // most recently read groups first
        v4f a = *reinterpret_cast<const v4f*>(x + 4 * g), b = *reinterpret_cast<const v4f*>(y + 4 * g);
        float sx = 0.f, sy = 0.f, sw = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float ex = exp_nonpos(a[j] - mx), ey = exp_nonpos(b[j] - my);
            sx += ex; sy += ey; sw += ex * (a[j] - b[j]);
        }
        zx += sx; zy += sy; w += sw;
    }
    zx = block_sum(zx, ldsd);
    zy = block_sum(zy, ldsd);
    w = block_sum(w, ldsd);
    if (tid == 0 && kl_out) kl_out[blockIdx.x] = w / zx - ((double)mx + log(zx)) + ((double)my + log(zy));
    if (!tv_out) return;

    const float izx = (float)(1.0 / zx), izy = (float)(1.0 / zy);
    double tv = 0;
    for (uint64_t g = tid; g < n4; g += kLddBlock) {
        v4f a = *reinterpret_cast<const v4f*>(x + 4 * g), b = *reinterpret_cast<const v4f*>(y + 4 * g);
        float st = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) st += prob_gap(exp_nonpos(a[j] - mx), izx, exp_nonpos(b[j] - my), izy);
        tv += st;
    }
    for (uint64_t i = 4 * n4 + tid; i < n; i += kLddBlock)
        tv += prob_gap(exp_nonpos(x[i] - mx), izx, exp_nonpos(y[i] - my), izy);
    tv = block_sum(tv, ldsd);
    if (tid == 0) tv_out[blockIdx.x] = 0.5 * tv;
}

// ------------------------------------------------------------------ top-K distance
// With v_1 >= .. >= v_K the K largest logits outside I and w_1 .. w_K the logits of I, the cost of
// a threshold t >= v_K is f(t) = sum_j max(v_j - t, 0) + sum_i max(t - w_i, 0); below v_K the cost
// cannot decrease (at least K non-members lie above t, at most K members below), and f is piecewise
// linear, so the minimum is attained at one of the 2K values.  The K largest non-members are among
// the 2K largest logits of the row.  Those are found without sorting the row: every thread keeps
// the maximum of its own (strided) share while the row streams in from HBM; if tau is the smallest,
// over the 16 waves, of the r-th largest thread maximum of the wave (16 r >= 2K), then at least 2K
// logits are >= tau, and only threads whose maximum reaches tau can hold such logits.  Those few
// threads re-read their share (cache-resident) and append what reaches tau to a candidate list.
constexpr int kTopkCap = 1024;  // candidate list capacity; beyond it the slow exact path is taken

struct Cand {
    float v;
    int idx;
};

// larger value first; equal values: smaller index first (any fixed rule works, values decide the cost)
__device__ __forceinline__ bool cand_before(float va, int ia, float vb, int ib) {
    return va > vb || (va == vb && ia < ib);
}

template <bool VEC>
__global__ __launch_bounds__(kLddBlock) void topk_distance_kernel(const float* __restrict__ X, uint64_t n, uint64_t ld,
                                                                  const int32_t* __restrict__ idx_all, uint32_t K,
                                                                  double* __restrict__ out) {
    __shared__ float ldsf[kLddWaves];
    __shared__ int member_idx[IMM_TOPK_MAX];
    __shared__ float member_val[IMM_TOPK_MAX];
    __shared__ float top_out[IMM_TOPK_MAX];  // K largest non-members
    __shared__ Cand cand[kTopkCap];
    __shared__ unsigned char cand_member[kTopkCap];
    __shared__ int cand_count;
    __shared__ int bad_row;
    __shared__ double cost[2 * IMM_TOPK_MAX];
    const float* x = X + (uint64_t)blockIdx.x * ld;
    const int32_t* idx = idx_all + (uint64_t)blockIdx.x * K;
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    const uint64_t n4 = VEC ? n >> 2 : 0;
    // a row with fewer than 2K entries has fewer than K non-members: then every entry is accounted for
    const uint32_t Kn = (n - K < K) ? (uint32_t)(n - K) : K;

    if (tid == 0) { cand_count = 0; bad_row = 0; }
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

    // pass 1 (HBM): maximum of the thread's share
    float tmax = -INFINITY;
    for (uint64_t g = tid; g < n4; g += kLddBlock) {
        v4f a = *reinterpret_cast<const v4f*>(x + 4 * g);
        tmax = fmaxf(tmax, fmaxf(fmaxf(a.x, a.y), fmaxf(a.z, a.w)));
    }
    for (uint64_t i = 4 * n4 + tid; i < n; i += kLddBlock) tmax = fmaxf(tmax, x[i]);

    // r-th largest thread maximum of this wave (ties between lanes broken by lane number)
    const uint32_t r = (2 * K + kLddWaves - 1) / kLddWaves;
    float cur = tmax;     // candidates still in play in this lane
    float rth = -INFINITY;
    for (uint32_t it = 0; it < r; ++it) {
        float m = cur;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        rth = m;
        // retire exactly one lane holding m
        const uint64_t holders = __ballot(cur == m);
        const uint32_t first = (uint32_t)__builtin_ctzll(holders);
        if (lane == first) cur = -INFINITY;
    }
    if (lane == 0) ldsf[tid >> 6] = rth;
    __syncthreads();
    float tau = ldsf[0];
#pragma unroll
    for (int w = 1; w < kLddWaves; ++w) tau = fminf(tau, ldsf[w]);

    // pass 2 (cache): threads that can hold a candidate append every logit >= tau of their share
    if (tmax >= tau) {
        for (uint64_t g = tid; g < n4; g += kLddBlock) {
            v4f a = *reinterpret_cast<const v4f*>(x + 4 * g);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (a[j] >= tau) {
                    const int slot = atomicAdd(&cand_count, 1);
                    if (slot < kTopkCap) { cand[slot].v = a[j]; cand[slot].idx = (int)(4 * g + j); }
                }
        }
        for (uint64_t i = 4 * n4 + tid; i < n; i += kLddBlock)
            if (x[i] >= tau) {
                const int slot = atomicAdd(&cand_count, 1);
                if (slot < kTopkCap) { cand[slot].v = x[i]; cand[slot].idx = (int)i; }
            }
    }
    __syncthreads();
    const int c = cand_count;

    if (c <= kTopkCap) {
        for (int i = tid; i < c; i += kLddBlock) {
            bool is_member = false;
            for (uint32_t j = 0; j < K; ++j) is_member |= (member_idx[j] == cand[i].idx);
            cand_member[i] = is_member ? 1 : 0;
        }
        __syncthreads();
        // rank of every non-member candidate among the non-member candidates; ranks < Kn are the answer
        for (int i = tid; i < c; i += kLddBlock) {
            if (cand_member[i]) continue;
            const float v = cand[i].v;
            const int id = cand[i].idx;
            uint32_t rank = 0;
            for (int j = 0; j < c; ++j)
                rank += (!cand_member[j] && cand_before(cand[j].v, cand[j].idx, v, id)) ? 1u : 0u;
            if (rank < Kn) top_out[rank] = v;
        }
    } else {
        // More logits tie at (or crowd above) tau than the list holds: exact but slow path, K rounds
        // of "largest non-member after the previous pick", each a scan of the whole row.
        float last_v = INFINITY;
        int last_i = -1;
        for (uint32_t pick = 0; pick < Kn; ++pick) {
            float bv = -INFINITY;
            int bi = 0x7FFFFFFF;
            for (uint64_t i = tid; i < n; i += kLddBlock) {
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
            __syncthreads();  // cand[] is free to be reused as per-wave scratch
            if (lane == 0) { cand[tid >> 6].v = bv; cand[tid >> 6].idx = bi; }
            __syncthreads();
            bv = cand[0].v; bi = cand[0].idx;
            for (int w = 1; w < kLddWaves; ++w)
                if (cand_before(cand[w].v, cand[w].idx, bv, bi)) { bv = cand[w].v; bi = cand[w].idx; }
            if (tid == 0) top_out[pick] = bv;
            last_v = bv;
            last_i = bi;
        }
    }
    __syncthreads();

    // cost of each candidate threshold (with K non-members in hand, thresholds below v_K are never better)
    if (tid < 2 * K) {
        const bool usable = tid < K ? tid < Kn : true;
        const float t = tid < K ? (usable ? top_out[tid] : 0.f) : member_val[tid - K];
        double f = INFINITY;
        if (usable && (Kn < K || t >= top_out[K - 1])) {
            f = 0;
            for (uint32_t j = 0; j < Kn; ++j) f += fmax((double)top_out[j] - (double)t, 0.0);
            for (uint32_t j = 0; j < K; ++j) f += fmax((double)t - (double)member_val[j], 0.0);
        }
        cost[tid] = f;
    }
    __syncthreads();
    if (tid == 0) {
        double best = cost[0];
        for (uint32_t j = 1; j < 2 * K; ++j) best = fmin(best, cost[j]);
        out[blockIdx.x] = bad_row ? (double)NAN : best;
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

hipError_t ldd_tv_kl(hipStream_t stream, const float* X, const float* Y, uint64_t T, uint64_t n, uint64_t ld,
                     double* tv_out, double* kl_out) {
    if (vec_ok(X, ld) && vec_ok(Y, ld))
        hipLaunchKernelGGL((ldd_tv_kl_kernel<true>), dim3((unsigned)T), dim3(kLddBlock), 0, stream, X, Y, n, ld, tv_out,
                           kl_out);
    else
        hipLaunchKernelGGL((ldd_tv_kl_kernel<false>), dim3((unsigned)T), dim3(kLddBlock), 0, stream, X, Y, n, ld,
                           tv_out, kl_out);
    return hipGetLastError();
}

hipError_t topk_distance(hipStream_t stream, const float* X, uint64_t T, uint64_t n, uint64_t ld, const int32_t* idx,
                         uint32_t K, double* out) {
    if (vec_ok(X, ld))
        hipLaunchKernelGGL((topk_distance_kernel<true>), dim3((unsigned)T), dim3(kLddBlock), 0, stream, X, n, ld, idx, K,
                           out);
    else
        hipLaunchKernelGGL((topk_distance_kernel<false>), dim3((unsigned)T), dim3(kLddBlock), 0, stream, X, n, ld, idx,
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
