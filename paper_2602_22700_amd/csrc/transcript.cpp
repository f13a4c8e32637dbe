#include "transcript.h"

#include <cstring>

#include "host_field.h"
#include "sha256.h"

namespace imm {
namespace {
inline void put_u64le(uint8_t* p, uint64_t v) {
    for (int i = 0; i < 8; ++i) p[i] = (uint8_t)(v >> (8 * i));
}
}  // namespace

Transcript::Transcript(const uint8_t state[32]) { std::memcpy(s, state, 32); }

void Transcript::initial_state(uint8_t out[32]) { sha256("IMM-FS-v1", 9, out); }

void Transcript::absorb(const char tag[4], const void* data, size_t len) {
    Sha256 h;
    uint8_t hdr[44];
    std::memcpy(hdr, s, 32);
    std::memcpy(hdr + 32, tag, 4);
    put_u64le(hdr + 36, (uint64_t)len);
    h.update(hdr, sizeof(hdr));
    h.update(data, len);
    h.finish(s);
}

void Transcript::absorb_words(const char tag[4], const uint64_t* words, size_t count) {
    Sha256 h;
    uint8_t hdr[44];
    std::memcpy(hdr, s, 32);
    std::memcpy(hdr + 32, tag, 4);
    put_u64le(hdr + 36, (uint64_t)(8 * count));
    h.update(hdr, sizeof(hdr));
    for (size_t i = 0; i < count; ++i) {
        uint8_t le[8];
        put_u64le(le, words[i]);
        h.update(le, 8);
    }
    h.finish(s);
}

uint64_t Transcript::challenge() {
    uint8_t msg[40], h[32];
    std::memcpy(msg, s, 32);
    std::memcpy(msg + 32, "chal", 4);
    for (uint32_t ctr = 0;; ++ctr) {
        for (int i = 0; i < 4; ++i) msg[36 + i] = (uint8_t)(ctr >> (8 * i));
        sha256(msg, sizeof(msg), h);
        uint64_t v = 0;
        for (int i = 0; i < 8; ++i) v |= (uint64_t)h[i] << (8 * i);
        if (v < hf::P) {
            std::memcpy(s, h, 32);
            return v;
        }
    }
}

void Transcript::head(uint64_t m, uint64_t d, uint64_t n, const uint8_t dgA[32], const uint8_t dgB[32],
                      const uint8_t dgC[32], int mu, int nu, uint64_t* rx, uint64_t* ry) {
    const uint64_t shape[3] = {m, d, n};
    absorb_words("shap", shape, 3);
    absorb("comA", dgA, 32);
    absorb("comB", dgB, 32);
    absorb("comC", dgC, 32);
    for (int k = 0; k < mu; ++k) rx[k] = challenge();
    for (int k = 0; k < nu; ++k) ry[k] = challenge();
}

}  // namespace imm
