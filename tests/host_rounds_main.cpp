// Host-only driver for the library's host-side round arithmetic (the rounds of the sumcheck that the
// prover's host thread finishes on short tables).  Input (text): L, then L words of table a, L words
// of table b, then the challenge r.  Output: g(0) g(1) g(2) of the tables as they are, then the two
// tables bound to r (L/2 words each).  The test compares with the oracle's round and fold.
#include <cinttypes>
#include <cstdio>
#include <vector>

#include "../paper_2602_22700_amd/csrc/host_field.h"

int main() {
    unsigned long long L, r;
    if (std::scanf("%llu", &L) != 1 || L < 2) return 2;
    std::vector<uint64_t> a(L), b(L);
    for (auto* t : {&a, &b})
        for (auto& v : *t) { unsigned long long x; if (std::scanf("%llu", &x) != 1) return 2; v = x; }
    if (std::scanf("%llu", &r) != 1) return 2;
    uint64_t g[3];
    imm::hf::round_evals(a.data(), b.data(), L, g);
    std::printf("%" PRIu64 " %" PRIu64 " %" PRIu64 "\n", g[0], g[1], g[2]);
    imm::hf::fold(a.data(), L, r);
    imm::hf::fold(b.data(), L, r);
    for (auto* t : {&a, &b}) {
        for (unsigned long long i = 0; i < L / 2; ++i) std::printf("%" PRIu64 " ", (*t)[i]);
        std::printf("\n");
    }
    return 0;
}
