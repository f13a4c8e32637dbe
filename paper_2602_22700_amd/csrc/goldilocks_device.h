// Goldilocks field arithmetic for gfx950 device code.  p = 2^64 - 2^32 + 1.
//
// CDNA4 vector ALUs have no 64-bit multiplier: a 64x64 product is four
// 32x32->64 multiply-adds (v_mad_u64_u32).  The streaming reductions therefore
// accumulate raw partial products lazily (struct Acc below) and reduce once per
// lane; everything that leaves a kernel is the canonical residue in [0, p).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gl {

constexpr uint64_t P = 0xFFFFFFFF00000001ull;
constexpr uint64_t EPS = 0xFFFFFFFFull;  // 2^64 mod p

__device__ __forceinline__ uint64_t add(uint64_t a, uint64_t b) {
    uint64_t s = a + b;
    // a, b < p so a + b < 2p: one conditional subtraction.  When the 64-bit add
    // wrapped, s - P (mod 2^64) is still the right residue.
    return (s < a || s >= P) ? s - P : s;
}

__device__ __forceinline__ uint64_t sub(uint64_t a, uint64_t b) {
    uint64_t d = a - b;
    return a < b ? d + P : d;
}

__device__ __forceinline__ uint64_t canon(uint64_t x) { return x >= P ? x - P : x; }

// (hi * 2^64 + lo) mod p, using 2^64 = 2^32 - 1 and 2^96 = -1 (mod p).
__device__ __forceinline__ uint64_t reduce128(uint64_t lo, uint64_t hi) {
    uint64_t hl = hi & EPS, hh = hi >> 32;
    uint64_t t = lo - hh;
    if (lo < hh) t -= EPS;          // the borrowed 2^64 equals p + EPS; t >= 2^64 - EPS here, no underflow
    uint64_t u = (hl << 32) - hl;   // hl * EPS < 2^64
    uint64_t s = t + u;
    if (s < t) s += EPS;            // the carried 2^64 is EPS; s <= 2^64 - 2^33 here, no second carry
    return canon(s);
}

__device__ __forceinline__ uint64_t mul(uint64_t a, uint64_t b) {
    return reduce128(a * b, __umul64hi(a, b));
}

// x mod p for a signed integer held sign-extended in 64 bits.
__device__ __forceinline__ uint64_t enc(int64_t x) {
    // for x < 0 the bit pattern is 2^64 - |x|; adding p - 2^64 = 1 - 2^32 gives p - |x|
    return x < 0 ? (uint64_t)x - EPS : (uint64_t)x;
}

// ---------------------------------------------------------------------------
// Lazy multiply-accumulate.  With x = x1 2^32 + x0 and e = e1 2^32 + e0 the
// product is x0 e0 + (x0 e1 + x1 e0) 2^32 + x1 e1 2^64.  Each of the three
// columns is summed in a 64-bit register whose overflows are counted in a
// 32-bit carry register, so a lane can absorb 2^31 products before a reduction.
// One product costs four v_mad_u64_u32 (the carry-out of the 64-bit add lands in
// an SGPR pair) and four v_addc_co_u32.
struct Acc {
    uint64_t s0, s1, s2;  // column sums modulo 2^64
    uint32_t c0, c1, c2;  // number of times each column wrapped
};

__device__ __forceinline__ void acc_clear(Acc& a) {
    a.s0 = a.s1 = a.s2 = 0;
    a.c0 = a.c1 = a.c2 = 0;
}

// sum += x * e (32 x 32 -> 64, plus 64-bit add); carry += overflow of that add
__device__ __forceinline__ void mad_carry(uint64_t& sum, uint32_t& carry, uint32_t x, uint32_t e) {
    uint64_t co;  // wave-wide carry mask
    asm("v_mad_u64_u32 %0, %1, %3, %4, %0\n\t"
        "v_addc_co_u32 %2, %1, 0, %2, %1"
        : "+v"(sum), "=&s"(co), "+v"(carry)
        : "v"(x), "v"(e));
}

__device__ __forceinline__ void acc_mac(Acc& a, uint64_t x, uint64_t e) {
    uint32_t x0 = (uint32_t)x, x1 = (uint32_t)(x >> 32);
    uint32_t e0 = (uint32_t)e, e1 = (uint32_t)(e >> 32);
    mad_carry(a.s0, a.c0, x0, e0);
    mad_carry(a.s1, a.c1, x0, e1);
    mad_carry(a.s1, a.c1, x1, e0);
    mad_carry(a.s2, a.c2, x1, e1);
}

// Canonical residue of the accumulated sum.
//   value = (s0 + c0 2^64) + (s1 + c1 2^64) 2^32 + (s2 + c2 2^64) 2^64
__device__ __forceinline__ uint64_t acc_reduce(const Acc& a) {
    uint64_t r0 = reduce128(a.s0, a.c0);
    uint64_t r1 = mul(reduce128(a.s1, a.c1), 1ull << 32);
    uint64_t r2 = mul(reduce128(a.s2, a.c2), EPS);
    return add(add(r0, r1), r2);
}

}  // namespace gl
