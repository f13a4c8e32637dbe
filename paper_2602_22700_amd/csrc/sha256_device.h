// SHA-256 compression (FIPS 180-4 section 6.2.2) for one GPU lane, and the few
// fixed-layout transcript messages the round kernel hashes on the device.
//
// The transcript state is kept as the eight 32-bit working words H0..H7; the
// 32-byte state of the host API is their big-endian serialisation, so a state
// that is hashed again enters the next message as W0..W7 without byte swaps.
// Field elements are serialised little-endian, hence the bswap on their halves.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sha {

__device__ __forceinline__ uint32_t rotr(uint32_t x, int s) { return __builtin_amdgcn_alignbit(x, x, s); }
__device__ __forceinline__ uint32_t bswap(uint32_t x) { return __builtin_bswap32(x); }
// three-input xor in one instruction (v_bitop3_b32 with the truth table of a ^ b ^ c)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// cube-root constants of the first 64 primes (FIPS 180-4 section 4.2.2)
__device__ static const uint32_t K[64] = {
    0x428a2f98, 0x71374491, 0xb5c0fbcf, 0xe9b5dba5, 0x3956c25b, 0x59f111f1, 0x923f82a4, 0xab1c5ed5,
    0xd807aa98, 0x12835b01, 0x243185be, 0x550c7dc3, 0x72be5d74, 0x80deb1fe, 0x9bdc06a7, 0xc19bf174,
    0xe49b69c1, 0xefbe4786, 0x0fc19dc6, 0x240ca1cc, 0x2de92c6f, 0x4a7484aa, 0x5cb0a9dc, 0x76f988da,
    0x983e5152, 0xa831c66d, 0xb00327c8, 0xbf597fc7, 0xc6e00bf3, 0xd5a79147, 0x06ca6351, 0x14292967,
    0x27b70a85, 0x2e1b2138, 0x4d2c6dfc, 0x53380d13, 0x650a7354, 0x766a0abb, 0x81c2c92e, 0x92722c85,
    0xa2bfe8a1, 0xa81a664b, 0xc24b8b70, 0xc76c51a3, 0xd192e819, 0xd6990624, 0xf40e3585, 0x106aa070,
    0x19a4c116, 0x1e376c08, 0x2748774c, 0x34b0bcb5, 0x391c0cb3, 0x4ed8aa4a, 0x5b9cca4f, 0x682e6ff3,
    0x748f82ee, 0x78a5636f, 0x84c87814, 0x8cc70208, 0x90befffa, 0xa4506ceb, 0xbef9a3f7, 0xc67178f2};

struct State { uint32_t h[8]; };
struct Block { uint32_t w[16]; };

// One compression; arguments travel by value so that they stay in registers across the call.
// The schedule is kept as a rolling 16-word window.
__device__ __noinline__ State compress_fn(State st, Block bl) {
    uint32_t a = st.h[0], b = st.h[1], c = st.h[2], d = st.h[3], e = st.h[4], f = st.h[5], g = st.h[6], hh = st.h[7];
    uint32_t* w = bl.w;
#pragma unroll
    for (int t = 0; t < 64; ++t) {
        if (t >= 16) {
            uint32_t w15 = w[(t - 15) & 15], w2 = w[(t - 2) & 15];
            uint32_t s0 = xor3(rotr(w15, 7), rotr(w15, 18), w15 >> 3);
            uint32_t s1 = xor3(rotr(w2, 17), rotr(w2, 19), w2 >> 10);
            w[t & 15] = w[t & 15] + s0 + w[(t - 7) & 15] + s1;
        }
        uint32_t S1 = xor3(rotr(e, 6), rotr(e, 11), rotr(e, 25));
        uint32_t ch = __builtin_amdgcn_bitop3_b32(e, f, g, 0xCA);   // e ? f : g
        uint32_t t1 = hh + S1 + ch + K[t] + w[t & 15];
        uint32_t S0 = xor3(rotr(a, 2), rotr(a, 13), rotr(a, 22));
        uint32_t mj = __builtin_amdgcn_bitop3_b32(a, b, c, 0xE8);   // majority
        uint32_t t2 = S0 + mj;
        hh = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + t2;
    }
    st.h[0] += a; st.h[1] += b; st.h[2] += c; st.h[3] += d; st.h[4] += e; st.h[5] += f; st.h[6] += g; st.h[7] += hh;
    return st;
}

__device__ __forceinline__ void compress(uint32_t (&h)[8], uint32_t (&w)[16]) {
    State st;
    Block bl;
#pragma unroll
    for (int i = 0; i < 8; ++i) st.h[i] = h[i];
#pragma unroll
    for (int i = 0; i < 16; ++i) bl.w[i] = w[i];
    st = compress_fn(st, bl);
#pragma unroll
    for (int i = 0; i < 8; ++i) h[i] = st.h[i];
}

// The two halves of a compression for callers that let different waves do them: the message
// schedule with the round constants already added (it does not depend on the hash state), and the
// 64 rounds on such a schedule.
__device__ __forceinline__ void schedule_plus_k(const uint32_t (&m)[16], uint32_t (&wk)[64]) {
    uint32_t w[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) w[t] = m[t];
#pragma unroll
    for (int t = 0; t < 64; ++t) {
        if (t >= 16) {
            uint32_t w15 = w[(t - 15) & 15], w2 = w[(t - 2) & 15];
            uint32_t s0 = xor3(rotr(w15, 7), rotr(w15, 18), w15 >> 3);
            uint32_t s1 = xor3(rotr(w2, 17), rotr(w2, 19), w2 >> 10);
            w[t & 15] = w[t & 15] + s0 + w[(t - 7) & 15] + s1;
        }
        wk[t] = w[t & 15] + K[t];
    }
}
__device__ __forceinline__ void rounds_on_schedule(uint32_t (&h)[8], const uint32_t (&wk)[64]) {
    uint32_t a = h[0], b = h[1], c = h[2], d = h[3], e = h[4], f = h[5], g = h[6], hh = h[7];
#pragma unroll
    for (int t = 0; t < 64; ++t) {
        uint32_t S1 = xor3(rotr(e, 6), rotr(e, 11), rotr(e, 25));
        uint32_t ch = __builtin_amdgcn_bitop3_b32(e, f, g, 0xCA);
        uint32_t t1 = hh + S1 + ch + wk[t];
        uint32_t S0 = xor3(rotr(a, 2), rotr(a, 13), rotr(a, 22));
        uint32_t mj = __builtin_amdgcn_bitop3_b32(a, b, c, 0xE8);
        uint32_t t2 = S0 + mj;
        hh = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + t2;
    }
    h[0] += a; h[1] += b; h[2] += c; h[3] += d; h[4] += e; h[5] += f; h[6] += g; h[7] += hh;
}

__device__ __forceinline__ void init_h(uint32_t (&h)[8]) {
    // square-root constants of the first 8 primes (FIPS 180-4 section 5.3.3)
    h[0] = 0x6a09e667; h[1] = 0xbb67ae85; h[2] = 0x3c6ef372; h[3] = 0xa54ff53a;
    h[4] = 0x510e527f; h[5] = 0x9b05688c; h[6] = 0x1f83d9ab; h[7] = 0x5be0cd19;
}

// s <- SHA256(s || tag || u64le(8*nwords) || words as 8-byte little-endian), nwords in 1..3.
// `tag` is the four tag bytes read as a big-endian word.
__device__ __forceinline__ void absorb_words(uint32_t (&s)[8], uint32_t tag, const uint64_t* words, int nwords) {
    uint32_t w[16], h[8];
    init_h(h);
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = s[i];
    w[8] = tag;
    w[9] = bswap((uint32_t)(8 * nwords));  // low half of the little-endian length
    w[10] = 0;
    // message = 44 header bytes + 8*nwords payload bytes; words 11.. hold the payload
    uint32_t pay[6];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        uint64_t v = i < nwords ? words[i] : 0;
        pay[2 * i] = bswap((uint32_t)v);
        pay[2 * i + 1] = bswap((uint32_t)(v >> 32));
    }
    const uint32_t total_bytes = 44 + 8 * nwords;  // 52, 60 or 68
    if (nwords == 1) {
        w[11] = pay[0]; w[12] = pay[1]; w[13] = 0x80000000u; w[14] = 0; w[15] = total_bytes * 8;
        compress(h, w);
    } else if (nwords == 2) {
        w[11] = pay[0]; w[12] = pay[1]; w[13] = pay[2]; w[14] = pay[3]; w[15] = 0x80000000u;
        compress(h, w);
#pragma unroll
        for (int i = 0; i < 15; ++i) w[i] = 0;
        w[15] = total_bytes * 8;
        compress(h, w);
    } else {
        w[11] = pay[0]; w[12] = pay[1]; w[13] = pay[2]; w[14] = pay[3]; w[15] = pay[4];
        compress(h, w);
        w[0] = pay[5];
        w[1] = 0x80000000u;
#pragma unroll
        for (int i = 2; i < 15; ++i) w[i] = 0;
        w[15] = total_bytes * 8;
        compress(h, w);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) s[i] = h[i];
}

// Squeeze one field element: the first counter whose candidate is below p wins and its
// hash becomes the new state.  The loop ends after one pass except with probability 2^-32.
__device__ __forceinline__ uint64_t challenge(uint32_t (&s)[8]) {
    constexpr uint64_t P = 0xFFFFFFFF00000001ull;
    for (uint32_t ctr = 0;; ++ctr) {
        uint32_t w[16], h[8];
        init_h(h);
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = s[i];
        w[8] = 0x6368616cu;  // "chal"
        w[9] = bswap(ctr);
        w[10] = 0x80000000u;
        w[11] = w[12] = w[13] = w[14] = 0;
        w[15] = 40 * 8;
        compress(h, w);
        uint64_t v = (uint64_t)bswap(h[0]) | ((uint64_t)bswap(h[1]) << 32);
        if (v < P || ctr == 0xFFFFFFFFu) {  // the second test only bounds the loop
#pragma unroll
            for (int i = 0; i < 8; ++i) s[i] = h[i];
            return v < P ? v : v - P;
        }
    }
}

constexpr uint32_t TAG_CLMC = 0x636c6d43u;  // "clmC"
constexpr uint32_t TAG_RND = 0x726e6420u;   // "rnd "
constexpr uint32_t TAG_FIN = 0x66696e20u;   // "fin "

}  // namespace sha
