// Host-only driver for a build of the library's CPU sources (SHA-256, transcript, commitments,
// verifier) with -fsanitize=address,undefined: it runs the calls a verifier makes on inputs read
// from stdin and prints their results, which the test compares with the oracle's.  Input (text):
//   m d n
//   m*d int16 values, d*n int8 values, m*n int64 values
//   transcript state (64 hex digits), proof: mu delta nu c0 vA vB, then 3*delta words
// Output: the three digests, the verifier's code / fail round / state for the full call and for
// the call without matrices, the points, and a challenge squeezed from the given state.
#include <cinttypes>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../include/imm.h"

static void hex(const uint8_t* p, size_t n) {
    for (size_t i = 0; i < n; ++i) std::printf("%02x", p[i]);
    std::printf("\n");
}

int main() {
    unsigned long long m, d, n;
    if (std::scanf("%llu %llu %llu", &m, &d, &n) != 3) return 2;
    std::vector<int16_t> A(m * d);
    std::vector<int8_t> B(d * n);
    std::vector<int64_t> C(m * n);
    for (auto& v : A) { int x; if (std::scanf("%d", &x) != 1) return 2; v = (int16_t)x; }
    for (auto& v : B) { int x; if (std::scanf("%d", &x) != 1) return 2; v = (int8_t)x; }
    for (auto& v : C) { long long x; if (std::scanf("%lld", &x) != 1) return 2; v = x; }
    char hexstate[65];
    if (std::scanf("%64s", hexstate) != 1) return 2;
    uint8_t state[32];
    for (int i = 0; i < 32; ++i) { unsigned b; std::sscanf(hexstate + 2 * i, "%2x", &b); state[i] = (uint8_t)b; }
    imm_proof pr;
    std::memset(&pr, 0, sizeof(pr));
    pr.version = IMM_PROOF_VERSION;
    unsigned long long c0, vA, vB;
    if (std::scanf("%u %u %u %llu %llu %llu", &pr.mu, &pr.delta, &pr.nu, &c0, &vA, &vB) != 6) return 2;
    pr.c0 = c0; pr.vA = vA; pr.vB = vB;
    for (unsigned k = 0; k < 3 * pr.delta; ++k) { unsigned long long g; if (std::scanf("%llu", &g) != 1) return 2; pr.g[k] = g; }

    imm_commit com;
    std::memset(&com, 0, sizeof(com));
    std::printf("commit %d\n", imm_commit_matmul(A.data(), B.data(), C.data(), m, d, n, &com));
    hex(com.A.digest, 32); hex(com.B.digest, 32); hex(com.C.digest, 32);
    uint8_t out[32];
    int fr = -1;
    int rc = imm_verify(&com, state, &pr, A.data(), B.data(), C.data(), out, &fr);
    std::printf("verify_full %d %d\n", rc, fr);
    if (rc == 0) hex(out, 32);
    rc = imm_verify(&com, state, &pr, nullptr, nullptr, nullptr, out, &fr);
    std::printf("verify_transcript %d %d\n", rc, fr);
    if (rc == IMM_REJ_UNOPENED) hex(out, 32);
    uint64_t rx[IMM_MAX_ROUNDS], ry[IMM_MAX_ROUNDS], r[IMM_MAX_ROUNDS];
    rc = imm_verify_points(&com, state, &pr, rx, ry, r);
    std::printf("points %d", rc);
    for (unsigned i = 0; i < pr.mu; ++i) std::printf(" %" PRIu64, rx[i]);
    for (unsigned i = 0; i < pr.nu; ++i) std::printf(" %" PRIu64, ry[i]);
    for (unsigned i = 0; i < pr.delta; ++i) std::printf(" %" PRIu64, r[i]);
    std::printf("\n");
    uint64_t ch = 0;
    uint8_t st2[32];
    std::memcpy(st2, state, 32);
    rc = imm_transcript_challenge(st2, &ch);
    std::printf("challenge %d %" PRIu64 "\n", rc, ch);
    hex(st2, 32);
    // a perturbed product is rejected
    C[0] += 1;
    std::printf("verify_bad_C %d\n", imm_verify(&com, state, &pr, A.data(), B.data(), C.data(), out, &fr));
    return 0;
}
