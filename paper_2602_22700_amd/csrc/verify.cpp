// CPU verifier: replays the transcript, checks every round sum and the final
// product, and (when the matrices are supplied) the digests and the openings.
#include <algorithm>
#include <cstring>
#include <new>
#include <thread>
#include <vector>

#include "../../include/imm.h"
#include "host_field.h"
#include "transcript.h"

namespace imm {

void commit_raw(const void* raw, size_t bytes, uint32_t dtype, uint64_t rows, uint64_t cols, uint8_t out[32]);

namespace {

// eq vector, first point coordinate on the most significant index bit
std::vector<uint64_t> eq_vector(const uint64_t* pt, int t) {
    std::vector<uint64_t> e(size_t(1) << t);
    e[0] = 1;
    size_t len = 1;
    for (int k = 0; k < t; ++k) {
        uint64_t r = pt[k], nr = hf::sub(1, r);
        for (size_t i = len; i-- > 0;) {
            uint64_t v = e[i];
            e[2 * i] = hf::mul(v, nr);
            e[2 * i + 1] = hf::mul(v, r);
        }
        len *= 2;
    }
    return e;
}

// sum_i er[i] * sum_j ec[j] * enc(T[i][j])
template <typename T>
uint64_t open_matrix(const T* M, uint64_t rows, uint64_t cols, const std::vector<uint64_t>& er,
                     const std::vector<uint64_t>& ec) {
    unsigned hw = std::thread::hardware_concurrency();
    size_t nthreads = std::max<size_t>(1, std::min<size_t>(std::min<size_t>(hw ? hw : 1, 16), size_t(rows * cols >> 16)));
    std::vector<uint64_t> part(nthreads, 0);
    auto work = [&](size_t t) {
        uint64_t acc = 0;
        for (uint64_t i = t; i < rows; i += nthreads) {
            const T* row = M + i * cols;
            uint64_t inner = 0;
            for (uint64_t j = 0; j < cols; ++j) inner = hf::add(inner, hf::mul(ec[j], hf::enc((int64_t)row[j])));
            acc = hf::add(acc, hf::mul(er[i], inner));
        }
        part[t] = acc;
    };
    if (nthreads == 1) {
        work(0);
    } else {
        std::vector<std::thread> pool;
        for (size_t t = 0; t < nthreads; ++t) pool.emplace_back(work, t);
        for (auto& th : pool) th.join();
    }
    uint64_t total = 0;
    for (uint64_t v : part) total = hf::add(total, v);
    return total;
}

bool digest_matches(const void* raw, size_t bytes, uint32_t dtype, uint64_t rows, uint64_t cols, const uint8_t want[32]) {
    uint8_t got[32];
    commit_raw(raw, bytes, dtype, rows, cols, got);
    return std::memcmp(got, want, 32) == 0;
}

}  // namespace
}  // namespace imm

namespace imm {
namespace {

int verify_body(const imm_commit* com, const uint8_t transcript_in[32], const imm_proof* proof, const int16_t* A,
                const int8_t* B, const int64_t* C, uint8_t transcript_out[32], int* fail_round) {
    if (fail_round) *fail_round = 0;
    if (!com || !transcript_in || !proof) return IMM_E_NULL;
    const uint64_t m = com->A.rows, d = com->A.cols, n = com->B.cols;
    const uint64_t lim = 1ull << IMM_MAX_ROUNDS;
    if (m == 0 || d == 0 || n == 0 || m > lim || d > lim || n > lim) return IMM_E_SHAPE;
    if (com->B.rows != d || com->C.rows != m || com->C.cols != n) return IMM_E_SHAPE;
    if (com->A.dtype != IMM_I16 || com->B.dtype != IMM_I8 || com->C.dtype != IMM_I64) return IMM_E_DTYPE;
    const int mu = hf::ceil_log2(m), delta = hf::ceil_log2(d), nu = hf::ceil_log2(n);

    if (proof->version != IMM_PROOF_VERSION || (int)proof->mu != mu || (int)proof->delta != delta ||
        (int)proof->nu != nu)
        return IMM_REJ_FORMAT;
    if (proof->c0 >= hf::P || proof->vA >= hf::P || proof->vB >= hf::P) return IMM_REJ_FORMAT;
    for (int k = 0; k < 3 * delta; ++k)
        if (proof->g[k] >= hf::P) return IMM_REJ_FORMAT;
    for (int k = 3 * delta; k < 3 * IMM_MAX_ROUNDS; ++k)
        if (proof->g[k] != 0) return IMM_REJ_FORMAT;

    if (A && !digest_matches(A, size_t(m) * d * 2, IMM_I16, m, d, com->A.digest)) return IMM_REJ_COMMIT;
    if (B && !digest_matches(B, size_t(d) * n, IMM_I8, d, n, com->B.digest)) return IMM_REJ_COMMIT;
    if (C && !digest_matches(C, size_t(m) * n * 8, IMM_I64, m, n, com->C.digest)) return IMM_REJ_COMMIT;

    Transcript tr(transcript_in);
    uint64_t rx[IMM_MAX_ROUNDS], ry[IMM_MAX_ROUNDS], r[IMM_MAX_ROUNDS];
    tr.head(m, d, n, com->A.digest, com->B.digest, com->C.digest, mu, nu, rx, ry);
    tr.absorb_words("clmC", &proof->c0, 1);
    uint64_t claim = proof->c0;
    for (int k = 0; k < delta; ++k) {
        const uint64_t* g = &proof->g[3 * k];
        if (hf::add(g[0], g[1]) != claim) {
            if (fail_round) *fail_round = k + 1;
            return IMM_REJ_ROUND_SUM;
        }
        tr.absorb_words("rnd ", g, 3);
        r[k] = tr.challenge();
        claim = hf::interpolate3(g[0], g[1], g[2], r[k]);
    }
    if (hf::mul(proof->vA, proof->vB) != claim) return IMM_REJ_FINAL;
    const uint64_t fin[2] = {proof->vA, proof->vB};
    tr.absorb_words("fin ", fin, 2);

    if (A || B || C) {
        std::vector<uint64_t> ex = eq_vector(rx, mu), ey = eq_vector(ry, nu), er = eq_vector(r, delta);
        if (A && open_matrix(A, m, d, ex, er) != proof->vA) return IMM_REJ_OPEN_A;
        if (B && open_matrix(B, d, n, er, ey) != proof->vB) return IMM_REJ_OPEN_B;
        if (C && open_matrix(C, m, n, ex, ey) != proof->c0) return IMM_REJ_OPEN_C;
    }
    if (transcript_out) std::memcpy(transcript_out, tr.s, 32);
    // Without all three openings c0, vA and vB are not tied to the commitments: a prover is free to
    // choose c0 and consistent round messages.  That is not an accept.
    return (A && B && C) ? IMM_OK : IMM_REJ_UNOPENED;
}

}  // namespace
}  // namespace imm

extern "C" int imm_verify_points(const imm_commit* com, const uint8_t transcript_in[32], const imm_proof* proof,
                                 uint64_t* rx_out, uint64_t* ry_out, uint64_t* r_out) {
    using namespace imm;
    if (!com || !transcript_in || !proof) return IMM_E_NULL;
    const uint64_t m = com->A.rows, d = com->A.cols, n = com->B.cols;
    const uint64_t lim = 1ull << IMM_MAX_ROUNDS;
    if (m == 0 || d == 0 || n == 0 || m > lim || d > lim || n > lim) return IMM_E_SHAPE;
    if (com->B.rows != d || com->C.rows != m || com->C.cols != n) return IMM_E_SHAPE;
    if (com->A.dtype != IMM_I16 || com->B.dtype != IMM_I8 || com->C.dtype != IMM_I64) return IMM_E_DTYPE;
    const int mu = hf::ceil_log2(m), delta = hf::ceil_log2(d), nu = hf::ceil_log2(n);
    if (proof->version != IMM_PROOF_VERSION || (int)proof->mu != mu || (int)proof->delta != delta ||
        (int)proof->nu != nu || proof->c0 >= hf::P)
        return IMM_REJ_FORMAT;
    for (int k = 0; k < 3 * delta; ++k)
        if (proof->g[k] >= hf::P) return IMM_REJ_FORMAT;
    Transcript tr(transcript_in);
    uint64_t rx[IMM_MAX_ROUNDS] = {}, ry[IMM_MAX_ROUNDS] = {}, r[IMM_MAX_ROUNDS] = {};
    tr.head(m, d, n, com->A.digest, com->B.digest, com->C.digest, mu, nu, rx, ry);
    tr.absorb_words("clmC", &proof->c0, 1);
    for (int k = 0; k < delta; ++k) {
        tr.absorb_words("rnd ", &proof->g[3 * k], 3);
        r[k] = tr.challenge();
    }
    if (rx_out) std::memcpy(rx_out, rx, sizeof(rx));
    if (ry_out) std::memcpy(ry_out, ry, sizeof(ry));
    if (r_out) std::memcpy(r_out, r, sizeof(r));
    return IMM_OK;
}

extern "C" int imm_verify(const imm_commit* com, const uint8_t transcript_in[32], const imm_proof* proof,
                          const int16_t* A, const int8_t* B, const int64_t* C, uint8_t transcript_out[32],
                          int* fail_round) {
    try {
        return imm::verify_body(com, transcript_in, proof, A, B, C, transcript_out, fail_round);
    } catch (const std::bad_alloc&) {
        return IMM_E_NOMEM;  // e.g. the eq vector of a 2^32-row statement
    } catch (...) {
        return IMM_E_STATE;
    }
}
