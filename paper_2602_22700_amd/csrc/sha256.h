// SHA-256 (FIPS 180-4) for host code: transcript and commitments.
#pragma once
#include <cstddef>
#include <cstdint>

namespace imm {

struct Sha256 {
    uint32_t h[8];
    uint8_t buf[64];
    uint64_t total;   // bytes absorbed so far
    uint32_t fill;    // bytes waiting in buf

    Sha256() { reset(); }
    void reset();
    void update(const void* data, size_t len);
    void finish(uint8_t out[32]);
};

void sha256(const void* data, size_t len, uint8_t out[32]);

// Whether the compression function runs on the CPU's SHA extensions (checked against the portable one at start-up).
bool sha256_uses_cpu_extensions();

}  // namespace imm
