// SHA-256 written from FIPS 180-4: section 4.1.2 (functions), 4.2.2 (constants),
// 5.1.1 (padding), 5.3.3 (initial hash value), 6.2.2 (hash computation).
#include "sha256.h"

#include <cpuid.h>
#include <immintrin.h>

#include <cstring>

namespace imm {
namespace {

// first 32 bits of the fractional parts of the cube roots of the first 64 primes
const uint32_t K[64] = {
    0x428a2f98, 0x71374491, 0xb5c0fbcf, 0xe9b5dba5, 0x3956c25b, 0x59f111f1, 0x923f82a4, 0xab1c5ed5,
    0xd807aa98, 0x12835b01, 0x243185be, 0x550c7dc3, 0x72be5d74, 0x80deb1fe, 0x9bdc06a7, 0xc19bf174,
    0xe49b69c1, 0xefbe4786, 0x0fc19dc6, 0x240ca1cc, 0x2de92c6f, 0x4a7484aa, 0x5cb0a9dc, 0x76f988da,
    0x983e5152, 0xa831c66d, 0xb00327c8, 0xbf597fc7, 0xc6e00bf3, 0xd5a79147, 0x06ca6351, 0x14292967,
    0x27b70a85, 0x2e1b2138, 0x4d2c6dfc, 0x53380d13, 0x650a7354, 0x766a0abb, 0x81c2c92e, 0x92722c85,
    0xa2bfe8a1, 0xa81a664b, 0xc24b8b70, 0xc76c51a3, 0xd192e819, 0xd6990624, 0xf40e3585, 0x106aa070,
    0x19a4c116, 0x1e376c08, 0x2748774c, 0x34b0bcb5, 0x391c0cb3, 0x4ed8aa4a, 0x5b9cca4f, 0x682e6ff3,
    0x748f82ee, 0x78a5636f, 0x84c87814, 0x8cc70208, 0x90befffa, 0xa4506ceb, 0xbef9a3f7, 0xc67178f2};

inline uint32_t rotr(uint32_t x, int s) { return (x >> s) | (x << (32 - s)); }

void compress_portable(uint32_t h[8], const uint8_t block[64]) {
    uint32_t w[64];
    for (int t = 0; t < 16; ++t)
        w[t] = (uint32_t)block[4 * t] << 24 | (uint32_t)block[4 * t + 1] << 16 | (uint32_t)block[4 * t + 2] << 8 |
               (uint32_t)block[4 * t + 3];
    for (int t = 16; t < 64; ++t) {
        uint32_t s0 = rotr(w[t - 15], 7) ^ rotr(w[t - 15], 18) ^ (w[t - 15] >> 3);
        uint32_t s1 = rotr(w[t - 2], 17) ^ rotr(w[t - 2], 19) ^ (w[t - 2] >> 10);
        w[t] = s1 + w[t - 7] + s0 + w[t - 16];
    }
    uint32_t a = h[0], b = h[1], c = h[2], d = h[3], e = h[4], f = h[5], g = h[6], hh = h[7];
    for (int t = 0; t < 64; ++t) {
        uint32_t S1 = rotr(e, 6) ^ rotr(e, 11) ^ rotr(e, 25);
        uint32_t ch = (e & f) ^ (~e & g);
        uint32_t t1 = hh + S1 + ch + K[t] + w[t];
        uint32_t S0 = rotr(a, 2) ^ rotr(a, 13) ^ rotr(a, 22);
        uint32_t mj = (a & b) ^ (a & c) ^ (b & c);
        uint32_t t2 = S0 + mj;
        hh = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + t2;
    }
    h[0] += a; h[1] += b; h[2] += c; h[3] += d; h[4] += e; h[5] += f; h[6] += g; h[7] += hh;
}

// The same compression with the x86 SHA extensions.  SHA256RNDS2 does two rounds on a state kept as
// the register pair (A,B,E,F) / (C,D,G,H), taking W+K for the two rounds from the low half of its
// third operand and leaving the new (A,B,E,F) in place of (C,D,G,H), whose role the old (A,B,E,F)
// takes over; SHA256MSG1/MSG2 do the sigma0 / sigma1 parts of four message-schedule words.
__attribute__((target("sha,sse4.1,ssse3"))) void compress_shaext(uint32_t h[8], const uint8_t block[64]) {
    const __m128i be = _mm_set_epi64x(0x0c0d0e0f08090a0bll, 0x0405060700010203ll);  // big-endian words
    __m128i abcd = _mm_loadu_si128(reinterpret_cast<const __m128i*>(h));        // dwords A,B,C,D
    __m128i efgh = _mm_loadu_si128(reinterpret_cast<const __m128i*>(h + 4));    // dwords E,F,G,H
    __m128i t = _mm_shuffle_epi32(abcd, 0xB1);                                    // B,A,D,C
    efgh = _mm_shuffle_epi32(efgh, 0x1B);                                         // H,G,F,E
    __m128i abef = _mm_alignr_epi8(t, efgh, 8);                                   // F,E,B,A
    __m128i cdgh = _mm_blend_epi16(efgh, t, 0xF0);                                // H,G,D,C
    const __m128i abef0 = abef, cdgh0 = cdgh;
    __m128i m[4];
    for (int i = 0; i < 4; ++i)
        m[i] = _mm_shuffle_epi8(_mm_loadu_si128(reinterpret_cast<const __m128i*>(block + 16 * i)), be);
    for (int i = 0; i < 16; ++i) {  // four rounds per trip
        __m128i wk = _mm_add_epi32(m[i & 3], _mm_loadu_si128(reinterpret_cast<const __m128i*>(K + 4 * i)));
        cdgh = _mm_sha256rnds2_epu32(cdgh, abef, wk);
        wk = _mm_shuffle_epi32(wk, 0x0E);
        abef = _mm_sha256rnds2_epu32(abef, cdgh, wk);
        if (i < 12) {  // W[t..t+3], t = 4 (i + 4), replace W[t-16..t-13]
            __m128i x = _mm_sha256msg1_epu32(m[i & 3], m[(i + 1) & 3]);                      // + sigma0(W[t-15..t-12])
            x = _mm_add_epi32(x, _mm_alignr_epi8(m[(i + 3) & 3], m[(i + 2) & 3], 4));        // + W[t-7..t-4]
            m[i & 3] = _mm_sha256msg2_epu32(x, m[(i + 3) & 3]);                              // + sigma1(W[t-2..t+1])
        }
    }
    abef = _mm_add_epi32(abef, abef0);
    cdgh = _mm_add_epi32(cdgh, cdgh0);
    t = _mm_shuffle_epi32(abef, 0x1B);                                            // A,B,E,F
    cdgh = _mm_shuffle_epi32(cdgh, 0xB1);                                         // G,H,C,D
    _mm_storeu_si128(reinterpret_cast<__m128i*>(h), _mm_blend_epi16(t, cdgh, 0xF0));      // A,B,C,D
    _mm_storeu_si128(reinterpret_cast<__m128i*>(h + 4), _mm_alignr_epi8(cdgh, t, 8));     // E,F,G,H
}

bool cpu_has_shaext() {
    unsigned a, b, c, d;
    if (!__get_cpuid(1, &a, &b, &c, &d) || !(c & (1u << 9)) || !(c & (1u << 19))) return false;  // SSSE3, SSE4.1
    if (!__get_cpuid_count(7, 0, &a, &b, &c, &d) || !(b & (1u << 29))) return false;             // SHA
    // trust, but verify: one block through both
    uint8_t block[64];
    for (int i = 0; i < 64; ++i) block[i] = (uint8_t)(37 * i + 11);
    uint32_t h1[8], h2[8];
    for (int i = 0; i < 8; ++i) h1[i] = h2[i] = 0x9e3779b9u * (uint32_t)(i + 1);
    compress_portable(h1, block);
    compress_shaext(h2, block);
    return std::memcmp(h1, h2, sizeof(h1)) == 0;
}

using CompressFn = void (*)(uint32_t*, const uint8_t*);
const CompressFn compress = cpu_has_shaext() ? compress_shaext : compress_portable;

}  // namespace

bool sha256_uses_cpu_extensions() { return compress == compress_shaext; }

void Sha256::reset() {
    // first 32 bits of the fractional parts of the square roots of the first 8 primes
    static const uint32_t H0[8] = {0x6a09e667, 0xbb67ae85, 0x3c6ef372, 0xa54ff53a,
                                   0x510e527f, 0x9b05688c, 0x1f83d9ab, 0x5be0cd19};
    std::memcpy(h, H0, sizeof(h));
    total = 0;
    fill = 0;
}

void Sha256::update(const void* data, size_t len) {
    const uint8_t* p = static_cast<const uint8_t*>(data);
    total += len;
    if (fill) {
        size_t take = 64 - fill < len ? 64 - fill : len;
        std::memcpy(buf + fill, p, take);
        fill += (uint32_t)take;
        p += take;
        len -= take;
        if (fill < 64) return;
        compress(h, buf);
        fill = 0;
    }
    while (len >= 64) {
        compress(h, p);
        p += 64;
        len -= 64;
    }
    if (len) {
        std::memcpy(buf, p, len);
        fill = (uint32_t)len;
    }
}

void Sha256::finish(uint8_t out[32]) {
    uint64_t bits = total * 8;
    uint8_t pad[72];
    size_t padlen = (fill < 56) ? 56 - fill : 120 - fill;
    std::memset(pad, 0, sizeof(pad));
    pad[0] = 0x80;
    for (int i = 0; i < 8; ++i) pad[padlen + i] = (uint8_t)(bits >> (56 - 8 * i));
    update(pad, padlen + 8);
    for (int i = 0; i < 8; ++i) {
        out[4 * i] = (uint8_t)(h[i] >> 24);
        out[4 * i + 1] = (uint8_t)(h[i] >> 16);
        out[4 * i + 2] = (uint8_t)(h[i] >> 8);
        out[4 * i + 3] = (uint8_t)h[i];
    }
}

void sha256(const void* data, size_t len, uint8_t out[32]) {
    Sha256 s;
    s.update(data, len);
    s.finish(out);
}

}  // namespace imm
