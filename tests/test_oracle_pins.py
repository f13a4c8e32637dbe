"""Pins for the CPU oracle: it is checked against things other than itself.

Hand-computed worked examples (tests/golden/worked_examples.txt, re-derived here with
exact rational arithmetic), closed forms of the field, boolean-point and affine
identities of the multilinear extension, the sumcheck invariants, brute force on
4x4x4, and hashlib for the byte layout of the transcript.  CPU only.
"""
import ast
import hashlib
import os
import random
import struct
from fractions import Fraction

import numpy as np
import pytest

from oracle import reference as ref

P = 2**64 - 2**32 + 1
GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_examples.txt")


def load_golden():
    out, cur = {}, None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            cur = line.strip("[]")
            out[cur] = {}
            continue
        k, v = line.split("=", 1)
        out[cur][k.strip()] = ast.literal_eval(v.strip())
    return out


G = load_golden()
F = lambda v: v % P  # noqa: E731


# ------------------------------------------------------------------ golden file is self-consistent over Q
def _frac_eq_weights(point):
    """eq weights over the rationals, MSB-first, written independently of the oracle."""
    w = [Fraction(1)]
    for x in point:
        w = [e * f for e in w for f in (1 - Fraction(x), Fraction(x))]
    return w


@pytest.mark.parametrize("name", ["W1", "W2"])
def test_golden_examples_rederived_over_rationals(name):
    g = G[name]
    A, B, C = g["A"], g["B"], g["C"]
    m, d, n = len(A), len(B), len(B[0])
    assert C == [[sum(A[i][j] * B[j][y] for j in range(d)) for y in range(n)] for i in range(m)]
    ex, ey = _frac_eq_weights(g["rx"]), _frac_eq_weights(g["ry"])
    a = [sum(ex[i] * A[i][j] for i in range(m)) for j in range(d)]
    b = [sum(ey[y] * B[j][y] for y in range(n)) for j in range(d)]
    assert a == g["a"] and b == g["b"]
    assert sum(ex[i] * ey[y] * C[i][y] for i in range(m) for y in range(n)) == g["c0"]
    assert g["c0"] % P == g["c0_hex"]
    claim = Fraction(g["c0"])
    for k, r in enumerate(g["r"]):
        h = len(a) // 2
        at = lambda t: [a[i] + t * (a[i + h] - a[i]) for i in range(h)]  # noqa: E731
        bt = lambda t: [b[i] + t * (b[i + h] - b[i]) for i in range(h)]  # noqa: E731
        gk = [sum(x * y for x, y in zip(at(t), bt(t))) for t in (0, 1, 2)]
        assert gk == g["g"][k]
        assert gk[0] + gk[1] == claim
        a, b = at(r), bt(r)
        claim = sum(x * y for x, y in zip(a, b))
        assert claim == g["claims"][k]
    assert a == [g["vA"]] and b == [g["vB"]] and g["vA"] * g["vB"] == claim


# ------------------------------------------------------------------ field
def test_field_closed_forms(oracle_fast):
    mul = lambda a, b: int(oracle_fast.lib().orc_mul(a, b))  # noqa: E731
    two32 = 1 << 32
    two64 = mul(two32, two32)
    assert two64 == two32 - 1
    two96 = mul(two64, two32)
    assert two96 == P - 1
    two128 = mul(two96, two32)
    assert two128 == P - two32
    two192 = mul(two96, two96)
    assert two192 == 1
    assert mul(P - 1, P - 1) == 1
    assert mul(ref.INV2, 2) == 1 and ref.INV2 == 0x7FFFFFFF80000001
    # non-canonical inputs are reduced first
    assert mul(P, 5) == 0 and mul(2**64 - 1, 1) == two32 - 2
    assert int(oracle_fast.lib().orc_add(P - 1, 1)) == 0
    assert int(oracle_fast.lib().orc_sub(0, 1)) == P - 1


def test_field_random_vs_python_ints(oracle_fast):
    rnd = random.Random(11)
    L = oracle_fast.lib()
    edge = [0, 1, 2, P - 1, P - 2, 2**32, 2**32 - 1, 2**63, P // 2, P // 2 + 1]
    vals = edge + [rnd.randrange(P) for _ in range(500)]
    for a in vals[:40]:
        for b in vals:
            assert int(L.orc_mul(a, b)) == a * b % P
            assert int(L.orc_add(a, b)) == (a + b) % P
            assert int(L.orc_sub(a, b)) == (a - b) % P


# ------------------------------------------------------------------ encoding
def test_encoding_exhaustive_and_golden(oracle_fast):
    e = G["ENC"]
    assert ref.enc(-1) == e["minus1"] and ref.enc(-128) == e["minus128"] and ref.enc(-32768) == e["minus32768"]
    for arr in (np.arange(-128, 128, dtype=np.int8), np.arange(-32768, 32768, dtype=np.int16)):
        enc = oracle_fast.encode(arr)
        assert enc.dtype == np.uint64
        for x, v in zip(arr.tolist(), enc.tolist()):
            assert v == (x if x >= 0 else P + x)
            assert ref.dec(v) == x
    big = np.array([-(2**63), 2**63 - 1, -1, 0, -(2**36)], dtype=np.int64)
    assert oracle_fast.encode(big).tolist() == [int(x) % P for x in big.tolist()]


# ------------------------------------------------------------------ eq vectors
def test_eq_vector_pins(oracle_fast):
    g = G["MLE"]
    assert ref.eq_vector(g["point"]) == [F(v) for v in g["eq"]]
    assert oracle_fast.eq_vector(g["point"]).tolist() == [F(v) for v in g["eq"]]
    rnd = random.Random(5)
    for t in range(0, 8):
        pt = [rnd.randrange(P) for _ in range(t)]
        e0, e1 = ref.eq_vector(pt), oracle_fast.eq_vector(pt).tolist()
        assert e0 == e1 and len(e0) == 1 << t
        assert sum(e0) % P == 1
    # boolean point -> unit vector at the MSB-first index
    for t in range(1, 6):
        for idx in range(1 << t):
            bits = [(idx >> (t - k)) & 1 for k in range(1, t + 1)]
            e = oracle_fast.eq_vector(bits).tolist()
            assert e == [1 if i == idx else 0 for i in range(1 << t)]
    assert oracle_fast.eq_vector([]).tolist() == [1]


# ------------------------------------------------------------------ MLE
def test_mle_golden_and_boolean_points(oracle_fast):
    g = G["MLE"]
    assert ref.mle_table(g["T"], g["point"]) == g["value"]
    rnd = random.Random(6)
    T = [rnd.randrange(-1000, 1000) for _ in range(16)]
    for idx in range(16):
        bits = [(idx >> (4 - k)) & 1 for k in range(1, 5)]
        assert ref.mle_table(T, bits) == F(T[idx])
    # ragged table: virtual zeros
    assert ref.mle_table(T[:11], [1, 1, 0, 0]) == 0 and ref.mle_table(T[:11], [1, 0, 1, 0]) == F(T[10])


def test_mle_is_affine_in_each_variable(oracle_fast):
    rnd = random.Random(7)
    M = np.array([[rnd.randrange(-128, 128) for _ in range(6)] for _ in range(5)], dtype=np.int8)  # ragged 5x6
    pr, pc = [rnd.randrange(P) for _ in range(3)], [rnd.randrange(P) for _ in range(3)]
    for which in range(6):
        vals = []
        for t in (0, 1, 2, 3):
            q = pr + pc
            q[which] = t
            v0 = ref.mle_matrix(M.tolist(), 5, 6, q[:3], q[3:])
            assert oracle_fast.mle_matrix(M, q[:3], q[3:]) == v0
            vals.append(v0)
        assert vals[2] == (2 * vals[1] - vals[0]) % P
        assert vals[3] == (3 * vals[1] - 2 * vals[0]) % P


def test_matrix_mle_at_boolean_points_is_the_entry(oracle_fast):
    rnd = random.Random(8)
    M = np.array([[rnd.randrange(-2**15, 2**15) for _ in range(8)] for _ in range(4)], dtype=np.int16)
    for i in range(4):
        for j in range(8):
            bi = [(i >> 1) & 1, i & 1]
            bj = [(j >> 2) & 1, (j >> 1) & 1, j & 1]
            assert oracle_fast.mle_matrix(M, bi, bj) == F(int(M[i, j]))
            assert ref.mle_matrix(M.tolist(), 4, 8, bi, bj) == F(int(M[i, j]))


def test_partial_evaluations_match_direct_summation(oracle_fast):
    rnd = random.Random(9)
    A = np.array([[rnd.randrange(-2**15, 2**15) for _ in range(7)] for _ in range(5)], dtype=np.int16)
    rx = [rnd.randrange(P) for _ in range(3)]
    cx = [rnd.randrange(P) for _ in range(3)]
    ex, ec = oracle_fast.eq_vector(rx), oracle_fast.eq_vector(cx)
    over_rows = oracle_fast.partial_over_rows(A, ex).tolist()
    over_cols = oracle_fast.partial_over_cols(A, ec).tolist()
    for j in range(7):  # A~(rx, j): column j of A as a table over the row variables
        assert over_rows[j] == ref.mle_table(A[:, j].tolist(), rx)
    for i in range(5):
        assert over_cols[i] == ref.mle_table(A[i, :].tolist(), cx)


# ------------------------------------------------------------------ matmul
def test_matmul_hand_values_and_freivalds(oracle_fast):
    g = G["W2"]
    assert ref.matmul_naive(g["A"], g["B"], 2, 4, 2) == g["C"]
    assert oracle_fast.matmul(np.array(g["A"], dtype=np.int16), np.array(g["B"], dtype=np.int8)).tolist() == g["C"]
    rng = np.random.default_rng(3)
    A = rng.integers(-2**15, 2**15, size=(37, 53), dtype=np.int16)
    B = rng.integers(-128, 128, size=(53, 29), dtype=np.int8)
    C = oracle_fast.matmul(A, B)
    v = [int(x) for x in rng.integers(1, 1000, size=29)]
    Bv = [sum(int(B[j, y]) * v[y] for y in range(29)) for j in range(53)]
    for i in range(37):
        assert sum(int(C[i, y]) * v[y] for y in range(29)) == sum(int(A[i, j]) * Bv[j] for j in range(53))


# ------------------------------------------------------------------ transcript bytes
def test_transcript_byte_layout_against_hashlib():
    init = hashlib.sha256(b"IMM-FS-v1").digest()
    assert ref.FS_INIT == init
    tr = ref.Transcript()
    tr.absorb(b"shap", struct.pack("<QQQ", 2, 4, 2))
    s1 = hashlib.sha256(init + b"shap" + bytes([24, 0, 0, 0, 0, 0, 0, 0])
                        + bytes([2, 0, 0, 0, 0, 0, 0, 0, 4, 0, 0, 0, 0, 0, 0, 0, 2, 0, 0, 0, 0, 0, 0, 0])).digest()
    assert tr.s == s1
    # challenge: first counter whose first 8 bytes (little-endian) fall below p
    ctr = 0
    while True:
        h = hashlib.sha256(s1 + b"chal" + bytes([ctr & 255, ctr >> 8, 0, 0])).digest()
        v = sum(h[i] << (8 * i) for i in range(8))
        if v < P:
            break
        ctr += 1
    assert tr.challenge() == v and tr.s == h
    tr.absorb_field(b"rnd ", [1, P - 1, 2**32])
    data = (bytes([1] + [0] * 7) + bytes([0, 0, 0, 0, 255, 255, 255, 255]) + bytes([0, 0, 0, 0, 1, 0, 0, 0]))
    assert tr.s == hashlib.sha256(h + b"rnd " + bytes([24] + [0] * 7) + data).digest()


def test_challenge_rejection_predicate():
    acc = ref.Transcript.accepts
    assert acc(0) and acc(P - 1) and not acc(P) and not acc(2**64 - 1)


def test_challenge_skips_rejected_candidates(monkeypatch):
    # force the retry branch: reject the first two candidates whatever they are
    tr = ref.Transcript()
    seen = []

    def fake(v):
        seen.append(v)
        return len(seen) > 2

    monkeypatch.setattr(ref.Transcript, "accepts", staticmethod(fake))
    s0 = tr.s
    v = tr.challenge()
    h2 = hashlib.sha256(s0 + b"chal" + struct.pack("<I", 2)).digest()
    assert tr.s == h2 and v == int.from_bytes(h2[:8], "little") and len(seen) == 3


def test_commit_layout_against_hashlib(oracle_fast):
    rng = np.random.default_rng(0)
    B = rng.integers(-128, 128, size=(3, 5), dtype=np.int8)
    raw = bytes((int(x) & 0xFF) for x in B.reshape(-1))
    want = hashlib.sha256(b"IMM-COMMIT-v1" + bytes([1, 0, 0, 0]) + bytes([3] + [0] * 7) + bytes([5] + [0] * 7)
                          + hashlib.sha256(raw).digest()).digest()
    assert oracle_fast.commit_array(B) == want
    assert ref.commit_bytes(raw, ref.DT_I8, 3, 5) == want
    # two leaves: 1 MiB + 1 byte of int8
    big = rng.integers(-128, 128, size=(1, (1 << 20) + 1), dtype=np.int8)
    rawb = big.tobytes()
    want2 = hashlib.sha256(b"IMM-COMMIT-v1" + struct.pack("<IQQ", 1, 1, (1 << 20) + 1)
                           + hashlib.sha256(rawb[:1 << 20]).digest() + hashlib.sha256(rawb[1 << 20:]).digest()).digest()
    assert oracle_fast.commit_array(big) == want2
    A = rng.integers(-2**15, 2**15, size=(2, 2), dtype=np.int16)
    wantA = hashlib.sha256(b"IMM-COMMIT-v1" + struct.pack("<IQQ", 2, 2, 2)
                           + hashlib.sha256(b"".join(struct.pack("<h", int(x)) for x in A.reshape(-1))).digest()).digest()
    assert oracle_fast.commit_array(A) == wantA


# ------------------------------------------------------------------ worked examples through the oracle's own functions
@pytest.mark.parametrize("name", ["W1", "W2"])
def test_worked_examples_tier0_and_tier1(name, oracle_fast):
    g = G[name]
    A, B, C = g["A"], g["B"], g["C"]
    m, d, n = len(A), len(B), len(B[0])
    delta = ref.ceil_log2(d)
    rx, ry = g["rx"], g["ry"]
    # tier 0, by definition
    a0 = [ref.mle_table([A[i][j] for i in range(m)], rx) for j in range(d)]
    b0 = [ref.mle_table(B[j], ry) for j in range(d)]
    assert a0 == [F(v) for v in g["a"]] and b0 == [F(v) for v in g["b"]]
    assert ref.mle_matrix(C, m, n, rx, ry) == F(g["c0"]) == g["c0_hex"]
    prev = []
    for k in range(delta):
        gk = [ref.round_poly_by_definition(a0, b0, delta, prev, t) for t in (0, 1, 2)]
        assert gk == [F(v) for v in g["g"][k]]
        assert ref.interpolate3(*gk, g["r"][k]) == F(g["claims"][k])
        prev.append(g["r"][k])
    assert ref.mle_matrix(A, m, d, rx, prev) == F(g["vA"])
    assert ref.mle_matrix(B, d, n, prev, ry) == F(g["vB"])
    # tier 1, fold recurrence
    An, Bn = np.array(A, dtype=np.int16), np.array(B, dtype=np.int8)
    a1 = oracle_fast.partial_over_rows(An, oracle_fast.eq_vector(rx))
    b1 = oracle_fast.partial_over_cols(Bn, oracle_fast.eq_vector(ry))
    assert a1.tolist() == a0 and b1.tolist() == b0
    L = d
    for k in range(delta):
        assert oracle_fast.round_evals(a1, b1, L) == [F(v) for v in g["g"][k]]
        oracle_fast.fold(a1, L, g["r"][k])
        oracle_fast.fold(b1, L, g["r"][k])
        L //= 2
        if "folded_a" in g:
            assert a1[:L].tolist() == [F(v) for v in g["folded_a"][k]]
            assert b1[:L].tolist() == [F(v) for v in g["folded_b"][k]]
    assert int(a1[0]) == F(g["vA"]) and int(b1[0]) == F(g["vB"])
    assert oracle_fast.mle_matrix(An, rx, g["r"]) == F(g["vA"])
    assert oracle_fast.mle_matrix(Bn, g["r"], ry) == F(g["vB"])


# ------------------------------------------------------------------ round polynomial properties
def test_round_polynomials_degree_and_sum(oracle_fast):
    rnd = random.Random(21)
    delta = 4
    a = [rnd.randrange(P) for _ in range(16)]
    b = [rnd.randrange(P) for _ in range(16)]
    an, bn = np.array(a, dtype=np.uint64), np.array(b, dtype=np.uint64)
    claim = sum(x * y for x, y in zip(a, b)) % P
    prev, L = [], 16
    for k in range(delta):
        g_def = [ref.round_poly_by_definition(a, b, delta, prev, t) for t in (0, 1, 2, 3)]
        assert (g_def[0] + g_def[1]) % P == claim
        assert g_def[3] == (3 * g_def[2] - 3 * g_def[1] + g_def[0]) % P  # degree <= 2
        assert ref.interpolate3(*g_def[:3], 3) == g_def[3]
        assert oracle_fast.round_evals(an, bn, L) == g_def[:3]            # fold-based == definition
        r = rnd.randrange(P)
        claim = ref.interpolate3(*g_def[:3], r)
        assert claim == ref.round_poly_by_definition(a, b, delta, prev, r)
        oracle_fast.fold(an, L, r)
        oracle_fast.fold(bn, L, r)
        L //= 2
        prev.append(r)
    assert claim == ref.mle_table(a, prev) * ref.mle_table(b, prev) % P
    assert int(an[0]) == ref.mle_table(a, prev) and int(bn[0]) == ref.mle_table(b, prev)


def test_interpolation_reproduces_nodes_and_a_known_quadratic():
    q = lambda x: (5 * x * x - 3 * x + 9) % P  # noqa: E731
    for r in (0, 1, 2, 3, 10, P - 1, 2**40 + 17):
        assert ref.interpolate3(q(0), q(1), q(2), r) == q(r)


# ------------------------------------------------------------------ whole protocol on 4x4x4
def _case444(seed):
    rng = np.random.default_rng(seed)
    A = rng.integers(-2**15, 2**15, size=(4, 4), dtype=np.int16)
    B = rng.integers(-128, 128, size=(4, 4), dtype=np.int8)
    return A, B


def test_444_sumcheck_identity_on_all_boolean_points(oracle_fast):
    A, B = _case444(1)
    C = ref.matmul_naive(A.tolist(), B.tolist(), 4, 4, 4)
    bits = lambda v: [(v >> 1) & 1, v & 1]  # noqa: E731
    for x in range(4):
        for y in range(4):
            cxy = ref.mle_matrix(C, 4, 4, bits(x), bits(y))
            assert cxy == F(C[x][y])
            assert cxy == sum(ref.mle_matrix(A.tolist(), 4, 4, bits(x), bits(j))
                              * ref.mle_matrix(B.tolist(), 4, 4, bits(j), bits(y)) for j in range(4)) % P


def test_444_prove_verify_and_every_perturbation_rejected(oracle_fast):
    A, B = _case444(2)
    Al, Bl = A.tolist(), B.tolist()
    C = ref.matmul_naive(Al, Bl, 4, 4, 4)
    com = ref.commit_matmul(Al, Bl, C, 4, 4, 4)
    dg = (com["A"][0], com["B"][0], com["C"][0])
    proof, s_out = ref.prove(Al, Bl, C, 4, 4, 4, dg)
    code, s_v, _ = ref.verify(proof, 4, 4, 4, dg, A=Al, B=Bl, C=C)
    assert code == ref.ACCEPT and s_v == s_out
    assert ref.verify(proof, 4, 4, 4, dg)[0] == ref.ACCEPT
    # tier 1 produces the same bytes
    Cn = np.array(C, dtype=np.int64)
    assert oracle_fast.commit_matmul(A, B, Cn) == dg
    p1, s1 = oracle_fast.prove(A, B, Cn, dg)
    assert ref.proof_words(p1) == ref.proof_words(proof) and s1 == s_out
    assert oracle_fast.verify(p1, 4, 4, 4, dg, A=A, B=B, C=Cn)[0] == ref.ACCEPT
    # a prover that does not hold C derives the same c0
    p2, s2 = oracle_fast.prove(A, B, None, dg)
    assert ref.proof_words(p2) == ref.proof_words(proof) and s2 == s_out

    # every single-entry +-1 perturbation of C is rejected: the honest-statement prover
    # cannot complete, and the honest proof does not verify against the perturbed statement
    for i in range(4):
        for y in range(4):
            for dlt in (1, -1):
                Cb = [row[:] for row in C]
                Cb[i][y] += dlt
                comb = ref.commit_matmul(Al, Bl, Cb, 4, 4, 4)
                dgb = (comb["A"][0], comb["B"][0], comb["C"][0])
                with pytest.raises(AssertionError):
                    ref.prove(Al, Bl, Cb, 4, 4, 4, dgb)
                # a cheating prover that reuses honest round messages under the bad commitment
                codeb = ref.verify(proof, 4, 4, 4, dgb)[0]
                assert codeb != ref.ACCEPT
                # honest-looking proof against honest digests but wrong C matrix supplied for opening
                assert ref.verify(proof, 4, 4, 4, dg, C=Cb)[0] == ref.REJ_COMMIT

    # flipping any proof word is rejected
    words = ["c0", "vA", "vB"]
    for wname in words:
        bad = dict(proof, g=list(proof["g"]))
        bad[wname] = (bad[wname] + 1) % P
        assert ref.verify(bad, 4, 4, 4, dg, A=Al, B=Bl, C=C)[0] != ref.ACCEPT
        assert oracle_fast.verify(bad, 4, 4, 4, dg, A=A, B=B, C=Cn)[0] != ref.ACCEPT
    for k in range(len(proof["g"])):
        bad = dict(proof, g=list(proof["g"]))
        bad["g"][k] = (bad["g"][k] + 1) % P
        assert ref.verify(bad, 4, 4, 4, dg)[0] != ref.ACCEPT
        assert oracle_fast.verify(bad, 4, 4, 4, dg)[0] != ref.ACCEPT
    bad = dict(proof, c0=P)  # non-canonical word
    assert ref.verify(bad, 4, 4, 4, dg)[0] == ref.REJ_FORMAT
    bad = dict(proof, mu=3)
    assert ref.verify(bad, 4, 4, 4, dg)[0] == ref.REJ_FORMAT


def test_wrong_c_with_consistent_sumcheck_fails_the_opening(oracle_fast):
    """A prover may put the true sum_j a[j] b[j] in c0 even though the committed C is wrong:
    then the sumcheck rounds pass and only the opening of C exposes it."""
    A, B = _case444(4)
    C = oracle_fast.matmul(A, B)
    Cb = C.copy()
    Cb[2, 1] += 1
    dgb = oracle_fast.commit_matmul(A, B, Cb)
    proof, _ = oracle_fast.prove(A, B, None, dgb)
    assert oracle_fast.verify(proof, 4, 4, 4, dgb)[0] == ref.ACCEPT            # transcript-only check passes
    assert oracle_fast.verify(proof, 4, 4, 4, dgb, C=Cb)[0] == ref.REJ_OPEN_C  # opening catches it


# ------------------------------------------------------------------ tier 1 == tier 0 on ragged and tiny shapes
@pytest.mark.parametrize("shape", [(1, 1, 1), (1, 5, 3), (3, 1, 2), (5, 6, 7), (8, 16, 4), (2, 9, 1)])
def test_tier1_equals_tier0_on_small_shapes(shape, oracle_fast):
    m, d, n = shape
    rng = np.random.default_rng(100 + m * 31 + d * 7 + n)
    A = rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
    B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
    C = oracle_fast.matmul(A, B)
    assert C.tolist() == ref.matmul_naive(A.tolist(), B.tolist(), m, d, n)
    dg = oracle_fast.commit_matmul(A, B, C)
    com = ref.commit_matmul(A.tolist(), B.tolist(), C.tolist(), m, d, n)
    assert dg == (com["A"][0], com["B"][0], com["C"][0])
    t0, t1 = {}, {}
    p0, s0 = ref.prove(A.tolist(), B.tolist(), C.tolist(), m, d, n, dg, trace=t0)
    p1, s1 = oracle_fast.prove(A, B, C, dg, trace=t1)
    assert ref.proof_words(p0) == ref.proof_words(p1) and s0 == s1
    assert t0["rx"] == t1["rx"] and t0["ry"] == t1["ry"] and t0["r"] == t1["r"]
    assert t0["a"] == t1["a"].tolist() and t0["b"] == t1["b"].tolist()
    assert ref.verify(p1, m, d, n, dg, A=A.tolist(), B=B.tolist(), C=C.tolist()) == (ref.ACCEPT, s0, 0)
    assert oracle_fast.verify(p0, m, d, n, dg, A=A, B=B, C=C) == (ref.ACCEPT, s0, 0)


def test_tiny_config_tier0_equals_tier1(oracle_fast):
    """The 64x64x64 workload: tier 0 (pure Python, by definition) against tier 1."""
    from paper_2602_22700_amd import workloads
    A, B = workloads.tiny()
    C = oracle_fast.matmul(A, B)
    assert np.array_equal(C, workloads.exact_product_int64(A, B))
    dg = oracle_fast.commit_matmul(A, B, C)
    p1, s1 = oracle_fast.prove(A, B, C, dg)
    p0, s0 = ref.prove(A.tolist(), B.tolist(), C.tolist(), 64, 64, 64, dg)
    assert ref.proof_words(p0) == ref.proof_words(p1) and s0 == s1
    assert p1["delta"] == 6 and len(p1["g"]) == 18


def test_chained_state_threads_through(oracle_fast):
    A, B = _case444(9)
    C = oracle_fast.matmul(A, B)
    dg = oracle_fast.commit_matmul(A, B, C)
    items = [(A, B, C, dg)] * 3
    proofs, states = oracle_fast.prove_chain(items, chained=True)
    s = ref.FS_INIT
    for pr, st in zip(proofs, states):
        code, s_next, _ = oracle_fast.verify(pr, 4, 4, 4, dg, state_in=s)
        assert code == ref.ACCEPT and s_next == st
        s = s_next
    assert ref.proof_words(proofs[0]) != ref.proof_words(proofs[1])  # different challenges
    ind, st_ind = oracle_fast.prove_chain(items, chained=False)
    assert all(ref.proof_words(p) == ref.proof_words(ind[0]) for p in ind)
    # resuming a chain in the middle gives the same tail
    tail, st_tail = oracle_fast.prove_chain(items[1:], chained=True, state_in=states[0])
    assert [ref.proof_words(p) for p in tail] == [ref.proof_words(p) for p in proofs[1:]] and st_tail == states[1:]


# ------------------------------------------------------------------ planted mistakes are caught by the pins
def test_planted_lsb_first_order_breaks_the_mle_pin(monkeypatch):
    def eq_weight_lsb(i, point):
        w = 1
        for k, x in enumerate(point):
            w = w * ref.eq1((i >> k) & 1, x) % P
        return w
    monkeypatch.setattr(ref, "eq_weight", eq_weight_lsb)
    g = G["MLE"]
    assert ref.mle_table(g["T"], g["point"]) == 13 != g["value"]


def test_planted_wrong_interpolation_sign_breaks_the_claim_pin(monkeypatch):
    g = G["W1"]
    gk = [F(v) for v in g["g"][0]]

    def bad(g0, g1, g2, r):
        l0 = (r - 1) * (r - 2) % P * ref.INV2 % P
        l1 = (r * (r - 2)) % P  # sign dropped
        l2 = r * (r - 1) % P * ref.INV2 % P
        return (g0 * l0 + g1 * l1 + g2 * l2) % P
    assert bad(*gk, g["r"][0]) != F(g["claims"][0])
    assert ref.interpolate3(*gk, g["r"][0]) == F(g["claims"][0])
