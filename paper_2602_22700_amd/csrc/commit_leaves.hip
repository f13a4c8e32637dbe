// SHA-256 of the 1 MiB leaves of the matrix commitments (paper section 2.1: hash commitments;
// FIPS 180-4 for the hash), one leaf per lane.
//
// A hash chain cannot be split: the 16384 compressions of a leaf follow one another, 1.7 us each
// for a lane whatever the other lanes do, so a launch takes about 28 ms whether it hashes one leaf or
// the 65536 that the chip's lanes hold.  It pays from about five hundred leaves on (all the
// activations and products of a request at once); below that the host, with its SHA instructions,
// is faster.  The part of a compression that does not depend on the state, the message schedule, is
// taken off the chain by a second wave.  A leaf is read 64 bytes at a time, the block after next
// while the next one is prepared; the few hundred GB/s that all lanes together ask for are far
// below what HBM gives.
#include "commit_leaves.h"

#include "sha256_device.h"

namespace imm {
namespace k {
namespace {

typedef uint32_t v4u32 __attribute__((ext_vector_type(4)));

// the 16 message words of the 64-byte block at q, still in memory byte order
template <bool ALIGNED16>
__device__ __forceinline__ void load_block(const uint8_t* q, uint32_t (&raw)[16]) {
    if (ALIGNED16) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const v4u32 v = __builtin_nontemporal_load(reinterpret_cast<const v4u32*>(q) + j);
            raw[4 * j] = v.x; raw[4 * j + 1] = v.y; raw[4 * j + 2] = v.z; raw[4 * j + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) raw[j] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(q) + j);
    }
}

// 64 leaves per workgroup of two waves.  The message schedule of a block does not depend on the hash
// state, so wave 0 prepares it (load, byte order, expansion, round constants) for block t + 1 while
// wave 1 runs the 64 rounds of block t: the chain a leaf has to wait for is the rounds alone.  The
// schedules travel through LDS, two buffers of 64 words per lane; one barrier per block.
typedef uint32_t Schedules[16][64][4];  // [round / 4][lane][round % 4]: 16-byte accesses, lanes side by side

template <bool ALIGNED16>
__global__ __launch_bounds__(128) void commit_leaves_kernel(const LeafDesc* __restrict__ leaves, uint32_t count,
                                                            uint8_t* __restrict__ digests) {
    __shared__ Schedules buf[2];
    const uint32_t lane = threadIdx.x & 63, role = threadIdx.x >> 6;  // role 0 prepares, role 1 hashes
    const uint32_t leaf = blockIdx.x * 64 + lane;
    const bool valid = leaf < count;
    const uint8_t* p = valid ? leaves[leaf].p : nullptr;
    const uint64_t bytes = valid ? leaves[leaf].bytes : 0;
    const uint64_t whole = bytes / 64;
    uint64_t most = whole;  // the longest leaf of the 64 (both waves see the same leaves)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint64_t other = __shfl_xor(most, off, 64);
        most = other > most ? other : most;
    }
    uint32_t h[8], next[16];
    sha::init_h(h);
    auto prepare = [&](Schedules& out) {  // next[] holds the block; leaves the schedule in out
        uint32_t m[16], wk[64];
#pragma unroll
        for (int j = 0; j < 16; ++j) m[j] = sha::bswap(next[j]);
        sha::schedule_plus_k(m, wk);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            v4u32 v;
            v.x = wk[4 * j]; v.y = wk[4 * j + 1]; v.z = wk[4 * j + 2]; v.w = wk[4 * j + 3];
            *reinterpret_cast<v4u32*>(&out[j][lane][0]) = v;
        }
    };
    if (role == 0 && whole) {
        load_block<ALIGNED16>(p, next);
        prepare(buf[0]);
        if (whole > 1) load_block<ALIGNED16>(p + 64, next);
    }
    for (uint64_t t = 0; t < most; ++t) {
        __syncthreads();  // schedule t is complete, and schedule t - 1 has been used up
        if (role == 0) {
            if (t + 1 < whole) {
                prepare(buf[(t + 1) & 1]);
                if (t + 2 < whole) load_block<ALIGNED16>(p + 64 * (t + 2), next);
            }
        } else if (t < whole) {
            uint32_t wk[64];
            const Schedules& in = buf[t & 1];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const v4u32 v = *reinterpret_cast<const v4u32*>(&in[j][lane][0]);
                wk[4 * j] = v.x; wk[4 * j + 1] = v.y; wk[4 * j + 2] = v.z; wk[4 * j + 3] = v.w;
            }
            sha::rounds_on_schedule(h, wk);
        }
    }
    if (role == 0 || !valid) return;
    // padding (FIPS 180-4 section 5.1.1): the left-over bytes, 0x80, zeros, the length in bits as a
    // 64-bit big-endian number at the end of the last block
    uint32_t w[16];
    const uint32_t left = (uint32_t)(bytes % 64);
    const uint8_t* q = p + 64 * whole;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        uint32_t word = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t i = 4 * j + b;
            const uint32_t byte = i < left ? (uint32_t)q[i] : i == left ? 0x80u : 0u;
            word |= byte << (24 - 8 * b);
        }
        w[j] = word;
    }
    if (left >= 56) {  // no room for the length: it goes into a block of its own
        sha::compress(h, w);
#pragma unroll
        for (int j = 0; j < 16; ++j) w[j] = 0;
    }
    w[14] = (uint32_t)((bytes * 8) >> 32);
    w[15] = (uint32_t)(bytes * 8);
    sha::compress(h, w);
    uint32_t* out = reinterpret_cast<uint32_t*>(digests + 32 * (uint64_t)leaf);
#pragma unroll
    for (int j = 0; j < 8; ++j) out[j] = sha::bswap(h[j]);
}

}  // namespace

hipError_t commit_leaves(hipStream_t stream, const LeafDesc* leaves, uint32_t count, bool aligned16, uint8_t* digests) {
    if (count == 0) return hipSuccess;
    const unsigned blocks = (count + 63) / 64;
    if (aligned16)
        hipLaunchKernelGGL(commit_leaves_kernel<true>, dim3(blocks), dim3(128), 0, stream, leaves, count, digests);
    else
        hipLaunchKernelGGL(commit_leaves_kernel<false>, dim3(blocks), dim3(128), 0, stream, leaves, count, digests);
    return hipGetLastError();
}

}  // namespace k
}  // namespace imm
