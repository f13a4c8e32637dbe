// Hash commitments of the statement's matrices (host only).
#include <algorithm>
#include <cstring>
#include <new>
#include <thread>
#include <vector>

#include "../../include/imm.h"
#include "sha256.h"
#include "transcript.h"

namespace imm {

constexpr size_t kLeafBytes = size_t(1) << 20;

// Two-level hash: 1 MiB leaves (hashed by a few host threads), then one hash over
// the header and the leaf digests.
void commit_raw(const void* raw, size_t bytes, uint32_t dtype, uint64_t rows, uint64_t cols, uint8_t out[32]) {
    const uint8_t* p = static_cast<const uint8_t*>(raw);
    size_t leaves = (bytes + kLeafBytes - 1) / kLeafBytes;
    std::vector<uint8_t> digests(leaves * 32);
    unsigned hw = std::thread::hardware_concurrency();
    size_t nthreads = std::max<size_t>(1, std::min<size_t>(std::min<size_t>(hw ? hw : 1, 16), leaves / 4));
    auto work = [&](size_t t0) {
        for (size_t t = t0; t < leaves; t += nthreads) {
            size_t off = t * kLeafBytes;
            sha256(p + off, std::min(kLeafBytes, bytes - off), &digests[t * 32]);
        }
    };
    if (nthreads <= 1) {
        work(0);
    } else {
        std::vector<std::thread> pool;
        for (size_t t = 0; t < nthreads; ++t) pool.emplace_back(work, t);
        for (auto& th : pool) th.join();
    }
    Sha256 top;
    uint8_t hdr[13 + 4 + 8 + 8];
    std::memcpy(hdr, "IMM-COMMIT-v1", 13);
    for (int i = 0; i < 4; ++i) hdr[13 + i] = (uint8_t)(dtype >> (8 * i));
    for (int i = 0; i < 8; ++i) hdr[17 + i] = (uint8_t)(rows >> (8 * i));
    for (int i = 0; i < 8; ++i) hdr[25 + i] = (uint8_t)(cols >> (8 * i));
    top.update(hdr, sizeof(hdr));
    top.update(digests.data(), digests.size());
    top.finish(out);
}

static void fill(imm_commit1* c, const void* raw, size_t elem, uint32_t dtype, uint64_t rows, uint64_t cols) {
    commit_raw(raw, size_t(rows) * size_t(cols) * elem, dtype, rows, cols, c->digest);
    c->rows = rows;
    c->cols = cols;
    c->dtype = dtype;
    c->_pad = 0;
}

}  // namespace imm

extern "C" int imm_commit_matmul(const int16_t* A, const int8_t* B, const int64_t* C, uint64_t m, uint64_t d,
                                 uint64_t n, imm_commit* out) {
    if (!out) return IMM_E_NULL;
    const uint64_t lim = 1ull << IMM_MAX_ROUNDS;
    if (m == 0 || d == 0 || n == 0 || m > lim || d > lim || n > lim) return IMM_E_SHAPE;
    try {
        if (A) imm::fill(&out->A, A, 2, IMM_I16, m, d);
        if (B) imm::fill(&out->B, B, 1, IMM_I8, d, n);
        if (C) imm::fill(&out->C, C, 8, IMM_I64, m, n);
    } catch (const std::bad_alloc&) {
        return IMM_E_NOMEM;
    } catch (...) {  // a worker thread could not be started
        return IMM_E_STATE;
    }
    return IMM_OK;
}

extern "C" int imm_transcript_challenge(uint8_t state[32], uint64_t* out) {
    if (!state || !out) return IMM_E_NULL;
    imm::Transcript tr(state);
    *out = tr.challenge();
    std::memcpy(state, tr.s, 32);
    return IMM_OK;
}

extern "C" int imm_fs_init(uint8_t state[32]) {
    if (!state) return IMM_E_NULL;
    imm::Transcript::initial_state(state);
    return IMM_OK;
}
