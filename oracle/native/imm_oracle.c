/* Tier-1 oracle: the same definitions as oracle/reference.py in plain C.
 *
 * TEST INFRASTRUCTURE ONLY.  Every field operation is `unsigned __int128`
 * arithmetic followed by `% P` -- no Goldilocks reduction shortcuts, no lazy
 * accumulation, no blocking.  Loops over independent outputs are spread over
 * host threads with OpenMP; each output is still a plain sequential sum.
 * Hashing stays in Python (hashlib); this file holds only the arithmetic.
 *
 * Conventions (variable order MSB-first, virtual zero padding, x -> x mod p
 * encoding) are those listed at the top of oracle/reference.py, which this
 * file is checked against bit for bit.
 *
 * The statement proven is the matrix product inside the reference model's
 * continuous transformations (paper section 5.2, item 2).
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef unsigned __int128 u128;
static const uint64_t P = 0xFFFFFFFF00000001ULL;

enum { DT_I8 = 1, DT_I16 = 2, DT_I64 = 3, DT_F64P = 4 };

static uint64_t f_add(uint64_t a, uint64_t b) { return (uint64_t)(((u128)a + b) % P); }
static uint64_t f_sub(uint64_t a, uint64_t b) { return (uint64_t)(((u128)a + P - b) % P); }
static uint64_t f_mul(uint64_t a, uint64_t b) { return (uint64_t)(((u128)a * b) % P); }

/* signed integer -> canonical residue */
static uint64_t f_enc(int64_t x) {
    __int128 v = (__int128)x % (__int128)P;
    if (v < 0) v += P;
    return (uint64_t)v;
}

static uint64_t load_enc(const void* T, int dtype, size_t idx) {
    switch (dtype) {
    case DT_I8:  return f_enc(((const int8_t*)T)[idx]);
    case DT_I16: return f_enc(((const int16_t*)T)[idx]);
    case DT_I64: return f_enc(((const int64_t*)T)[idx]);
    default:     return ((const uint64_t*)T)[idx] % P;
    }
}

int orc_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

uint64_t orc_mul(uint64_t a, uint64_t b) { return f_mul(a % P, b % P); }
uint64_t orc_add(uint64_t a, uint64_t b) { return f_add(a % P, b % P); }
uint64_t orc_sub(uint64_t a, uint64_t b) { return f_sub(a % P, b % P); }
uint64_t orc_enc(int64_t x) { return f_enc(x); }

void orc_encode(const void* src, int dtype, size_t count, uint64_t* dst) {
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < count; ++i) dst[i] = load_enc(src, dtype, i);
}

/* eq vector by the doubling recurrence: start from [1]; for k = 1..t every
 * entry e splits into (e*(1-r_k), e*r_k) at indices (2i, 2i+1).  Because r_1 is
 * split first it ends up on the most significant bit. */
void orc_eq_vector(const uint64_t* pt, int t, uint64_t* out) {
    size_t len = 1;
    out[0] = 1;
    for (int k = 0; k < t; ++k) {
        uint64_t r = pt[k], one_minus_r = f_sub(1, r);
        for (size_t i = len; i-- > 0;) {
            uint64_t e = out[i];
            out[2 * i] = f_mul(e, one_minus_r);
            out[2 * i + 1] = f_mul(e, r);
        }
        len *= 2;
    }
}

/* out[j] = sum_{i<rows} eq_rows[i] * T[i][j]   (partial evaluation in the row variables) */
void orc_partial_over_rows(const void* T, int dtype, size_t rows, size_t cols, size_t ld,
                           const uint64_t* eq_rows, uint64_t* out) {
#pragma omp parallel for schedule(static)
    for (size_t j = 0; j < cols; ++j) {
        uint64_t acc = 0;
        for (size_t i = 0; i < rows; ++i) acc = f_add(acc, f_mul(eq_rows[i], load_enc(T, dtype, i * ld + j)));
        out[j] = acc;
    }
}

/* out[i] = sum_{j<cols} eq_cols[j] * T[i][j]   (partial evaluation in the column variables) */
void orc_partial_over_cols(const void* T, int dtype, size_t rows, size_t cols, size_t ld,
                           const uint64_t* eq_cols, uint64_t* out) {
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < rows; ++i) {
        uint64_t acc = 0;
        for (size_t j = 0; j < cols; ++j) acc = f_add(acc, f_mul(eq_cols[j], load_enc(T, dtype, i * ld + j)));
        out[i] = acc;
    }
}

/* T~(prow || pcol) = sum_i sum_j eq_rows[i] * eq_cols[j] * T[i][j] */
uint64_t orc_mle_matrix(const void* T, int dtype, size_t rows, size_t cols, size_t ld,
                        const uint64_t* eq_rows, const uint64_t* eq_cols) {
    uint64_t* per_row = (uint64_t*)malloc(rows * sizeof(uint64_t));
    if (!per_row) return ~0ULL;
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < rows; ++i) {
        uint64_t acc = 0;
        for (size_t j = 0; j < cols; ++j)
            acc = f_add(acc, f_mul(f_mul(eq_rows[i], eq_cols[j]), load_enc(T, dtype, i * ld + j)));
        per_row[i] = acc;
    }
    uint64_t total = 0;
    for (size_t i = 0; i < rows; ++i) total = f_add(total, per_row[i]);
    free(per_row);
    return total;
}

/* Round polynomial of the product of two multilinear tables of length L, with
 * the leading variable free: g(t) = sum_{i<L/2} a_t[i] * b_t[i], where
 * x_t[i] = x[i] + t*(x[i+L/2] - x[i]) is the table with its top variable set to t. */
void orc_round_evals(const uint64_t* a, const uint64_t* b, size_t L, uint64_t g[3]) {
    size_t h = L / 2;
    uint64_t g0 = 0, g1 = 0, g2 = 0;
    for (size_t i = 0; i < h; ++i) {
        uint64_t a0 = a[i], a1 = a[i + h], b0 = b[i], b1 = b[i + h];
        uint64_t a2 = f_add(a0, f_mul(2, f_sub(a1, a0)));
        uint64_t b2 = f_add(b0, f_mul(2, f_sub(b1, b0)));
        g0 = f_add(g0, f_mul(a0, b0));
        g1 = f_add(g1, f_mul(a1, b1));
        g2 = f_add(g2, f_mul(a2, b2));
    }
    g[0] = g0; g[1] = g1; g[2] = g2;
}

/* Bind the leading variable to r: x[i] <- x[i] + r*(x[i+L/2] - x[i]), i < L/2. */
void orc_fold(uint64_t* x, size_t L, uint64_t r) {
    size_t h = L / 2;
    for (size_t i = 0; i < h; ++i) x[i] = f_add(x[i], f_mul(r, f_sub(x[i + h], x[i])));
}

/* C = A.B over the integers, triple loop. */
void orc_matmul_i16_i8(const int16_t* A, const int8_t* B, size_t m, size_t d, size_t n, int64_t* C) {
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < m; ++i) {
        int64_t* crow = C + i * n;
        for (size_t y = 0; y < n; ++y) crow[y] = 0;
        for (size_t j = 0; j < d; ++j) {
            int64_t av = A[i * d + j];
            const int8_t* brow = B + j * n;
            for (size_t y = 0; y < n; ++y) crow[y] += av * (int64_t)brow[y];
        }
    }
}
