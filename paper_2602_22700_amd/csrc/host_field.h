// Host-side Goldilocks arithmetic (p = 2^64 - 2^32 + 1) for the verifier, the
// transcript glue and the first claim.  Values are canonical residues in [0, p).
#pragma once
#include <cstdint>

namespace imm {
namespace hf {

constexpr uint64_t P = 0xFFFFFFFF00000001ull;
constexpr uint64_t INV2 = 0x7FFFFFFF80000001ull;  // (p + 1) / 2

inline uint64_t add(uint64_t a, uint64_t b) {
    uint64_t s = a + b;
    return (s < a || s >= P) ? s - P : s;
}
inline uint64_t sub(uint64_t a, uint64_t b) { return a >= b ? a - b : a - b + P; }
inline uint64_t neg(uint64_t a) { return a ? P - a : 0; }

// Reduce a 128-bit value using 2^64 = 2^32 - 1 and 2^96 = -1 (mod p).
inline uint64_t reduce128(unsigned __int128 x) {
    uint64_t lo = (uint64_t)x, hi = (uint64_t)(x >> 64);
    uint64_t hl = hi & 0xFFFFFFFFull, hh = hi >> 32;
    uint64_t t = lo - hh;
    if (lo < hh) t -= 0xFFFFFFFFull;            // borrowed 2^64 = p + (2^32 - 1)
    uint64_t u = (hl << 32) - hl;               // hl * (2^32 - 1)
    uint64_t s = t + u;
    if (s < t) s += 0xFFFFFFFFull;              // carried 2^64 = 2^32 - 1 (mod p); cannot carry again
    return s >= P ? s - P : s;
}
inline uint64_t mul(uint64_t a, uint64_t b) { return reduce128((unsigned __int128)a * b); }

inline uint64_t enc(int64_t x) { return x >= 0 ? (uint64_t)x : P - (uint64_t)(-(x + 1)) - 1; }

// value at r of the quadratic through (0,g0), (1,g1), (2,g2)
inline uint64_t interpolate3(uint64_t g0, uint64_t g1, uint64_t g2, uint64_t r) {
    uint64_t rm1 = sub(r, 1), rm2 = sub(r, 2);
    uint64_t l0 = mul(mul(rm1, rm2), INV2);
    uint64_t l1 = neg(mul(r, rm2));
    uint64_t l2 = mul(mul(r, rm1), INV2);
    return add(add(mul(g0, l0), mul(g1, l1)), mul(g2, l2));
}

// Sum of products of canonical residues, reduced once at the end: 128 bits plus a count of the
// carries out of them, each worth 2^128 = -2^32 (mod p).  Up to 2^32 - 1 products.
struct ProductSum {
    unsigned __int128 s = 0;
    uint64_t carries = 0;
    void add(uint64_t a, uint64_t b) {
        const unsigned __int128 p = (unsigned __int128)a * b;
        s += p;
        carries += s < p;
    }
    uint64_t value() const { return sub(reduce128(s), carries << 32); }
};

// g(0), g(1), g(2) of the round polynomial of two tables of length L >= 2 (leading variable = upper half)
inline void round_evals(const uint64_t* a, const uint64_t* b, uint64_t L, uint64_t g[3]) {
    const uint64_t h = L >> 1;
    ProductSum g0, g1, g2;
    for (uint64_t i = 0; i < h; ++i) {
        const uint64_t a2 = sub(add(a[i + h], a[i + h]), a[i]), b2 = sub(add(b[i + h], b[i + h]), b[i]);
        g0.add(a[i], b[i]);
        g1.add(a[i + h], b[i + h]);
        g2.add(a2, b2);
    }
    g[0] = g0.value();
    g[1] = g1.value();
    g[2] = g2.value();
}
// bind the leading variable of a table of length L to r, in place: x[i] <- x[i] + r (x[i + L/2] - x[i])
inline void fold(uint64_t* x, uint64_t L, uint64_t r) {
    const uint64_t h = L >> 1;
    for (uint64_t i = 0; i < h; ++i) x[i] = add(x[i], mul(r, sub(x[i + h], x[i])));
}

inline int ceil_log2(uint64_t n) {
    int t = 0;
    while (t < 64 && (1ull << t) < n) ++t;
    return t;
}

}  // namespace hf
}  // namespace imm
