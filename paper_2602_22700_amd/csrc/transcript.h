// Fiat-Shamir transcript over SHA-256 (32-byte running state).
#pragma once
#include <cstddef>
#include <cstdint>

namespace imm {

struct Transcript {
    uint8_t s[32];

    explicit Transcript(const uint8_t state[32]);
    static void initial_state(uint8_t out[32]);  // SHA256("IMM-FS-v1")

    // s <- SHA256(s || tag[4] || u64le(len) || data)
    void absorb(const char tag[4], const void* data, size_t len);
    void absorb_words(const char tag[4], const uint64_t* words, size_t count);  // 8-byte LE each

    // first counter whose candidate is canonical; s <- that hash
    uint64_t challenge();

    // the statement header: shapes and the three digests, then mu + nu challenges
    void head(uint64_t m, uint64_t d, uint64_t n, const uint8_t dgA[32], const uint8_t dgB[32],
              const uint8_t dgC[32], int mu, int nu, uint64_t* rx, uint64_t* ry);
};

}  // namespace imm
