"""Tier-0 oracle: the matmul sumcheck written out with Python integers.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Nothing here is fast and
nothing here is clever: each function is the definition it names.

What is proven (paper section 5.2, item 2 of the VC statement; step
``F_theta*`` of the VC algorithm in the appendix): the matrix products inside
the reference model's continuous transformations were computed from the
committed operands.  Commitments are plain hashes (paper section 2.1).  The
paper leaves the proof system open ("TEEs or zero-knowledge proofs", section
2.2); this oracle fixes the classical interactive sumcheck for
``C = A.B`` made non-interactive with a hash transcript.

Conventions fixed here (the paper is silent on all of them)

* Field: GF(p), p = 2^64 - 2^32 + 1.  Residues are canonical, in [0, p).
* Encoding: a signed integer x becomes x mod p.
* Shapes: A is m x d, B is d x n, C is m x n, all row-major.  mu, delta, nu
  are ceil(log2) of m, d, n.  Dimensions are padded to powers of two with
  zeros; the padding is virtual.  A dimension of 1 has zero variables.
* Variable order is MSB-first: for a table T of length 2^t and a point
  x = (x_1 .. x_t), variable x_1 is tied to the most significant index bit,

      T~(x) = sum_i T[i] * prod_{k=1..t} eq(bit_k(i), x_k),
      bit_k(i) = (i >> (t-k)) & 1,   eq(b, x) = b*x + (1-b)*(1-x).

  For a matrix the point is (row point || column point).
* Transcript: 32-byte state s.  init: s = SHA256("IMM-FS-v1").
  absorb(tag, data): s = SHA256(s || tag || u64le(len(data)) || data) with a
  4-byte ASCII tag.  challenge(): for ctr = 0, 1, ...: h = SHA256(s || "chal"
  || u32le(ctr)); v = first 8 bytes of h as little-endian u64; accept when
  v < p (then s = h).  Field elements are serialised as 8-byte little-endian.
* Commitment of a matrix: SHA256("IMM-COMMIT-v1" || u32le(dtype) ||
  u64le(rows) || u64le(cols) || leaf_0 || leaf_1 ...), leaf_t = SHA256 of the
  t-th 1 MiB slice of the raw row-major little-endian integer bytes.
* Proof schedule: absorb shapes ("shap"), the three digests ("comA", "comB",
  "comC"); squeeze rx (mu values) then ry (nu values); a[j] = A~(rx, j),
  b[j] = B~(j, ry); c0 = C~(rx, ry) is absorbed ("clmC") and becomes the
  first claim; delta rounds over the shared dimension, each sending
  g_k(0), g_k(1), g_k(2) ("rnd ") and receiving r_k; finally vA = A~(rx, r),
  vB = B~(r, ry) ("fin ").
"""
from __future__ import annotations

import hashlib
import struct
from typing import List, Sequence, Tuple

P = 2**64 - 2**32 + 1
INV2 = (P + 1) // 2

DT_I8, DT_I16, DT_I64, DT_F64P = 1, 2, 3, 4
_DT_BYTES = {DT_I8: 1, DT_I16: 2, DT_I64: 8, DT_F64P: 8}

FS_INIT = hashlib.sha256(b"IMM-FS-v1").digest()
LEAF_BYTES = 1 << 20


# --------------------------------------------------------------------------- field
def enc(x: int) -> int:
    """Signed integer -> canonical residue."""
    return x % P


def dec(v: int) -> int:
    """Canonical residue -> the signed integer of smallest magnitude."""
    return v if v <= P // 2 else v - P


def ceil_log2(n: int) -> int:
    if n < 1:
        raise ValueError("dimension must be >= 1")
    return (n - 1).bit_length()


# --------------------------------------------------------------------------- MLE
def eq1(b: int, x: int) -> int:
    """eq(b, x) = b*x + (1-b)*(1-x) for a bit b and a field element x."""
    return (b * x + (1 - b) * (1 - x)) % P


def eq_weight(i: int, point: Sequence[int]) -> int:
    """prod_k eq(bit_k(i), x_k) with x_1 bound to the most significant bit."""
    t = len(point)
    w = 1
    for k in range(1, t + 1):
        w = w * eq1((i >> (t - k)) & 1, point[k - 1]) % P
    return w


def eq_vector(point: Sequence[int]) -> List[int]:
    """All 2^t weights, each by its own product (no doubling recurrence)."""
    return [eq_weight(i, point) for i in range(1 << len(point))]


def mle_table(table: Sequence[int], point: Sequence[int]) -> int:
    """T~(point) by summation.  Entries beyond len(table) are virtual zeros."""
    if len(table) > (1 << len(point)):
        raise ValueError("table longer than 2^t")
    acc = 0
    for i, v in enumerate(table):
        acc = (acc + enc(int(v)) * eq_weight(i, point)) % P
    return acc


def mle_matrix(M, rows: int, cols: int, prow: Sequence[int], pcol: Sequence[int]) -> int:
    """M~(prow || pcol) = sum_{i,j} eq_prow[i] eq_pcol[j] M[i][j], term by term."""
    acc = 0
    for i in range(rows):
        wi = eq_weight(i, prow)
        for j in range(cols):
            acc = (acc + wi * eq_weight(j, pcol) % P * enc(int(M[i][j]))) % P
    return acc


def matmul_naive(A, B, m: int, d: int, n: int) -> List[List[int]]:
    """C[i][y] = sum_j A[i][j] * B[j][y] over the integers."""
    return [[sum(int(A[i][j]) * int(B[j][y]) for j in range(d)) for y in range(n)] for i in range(m)]


# --------------------------------------------------------------------------- transcript
def u64le(v: int) -> bytes:
    return struct.pack("<Q", v)


class Transcript:
    def __init__(self, state: bytes = FS_INIT):
        if len(state) != 32:
            raise ValueError("state must be 32 bytes")
        self.s = bytes(state)

    def absorb(self, tag: bytes, data: bytes) -> None:
        assert len(tag) == 4
        self.s = hashlib.sha256(self.s + tag + u64le(len(data)) + data).digest()

    def absorb_field(self, tag: bytes, vals: Sequence[int]) -> None:
        for v in vals:
            assert 0 <= v < P
        self.absorb(tag, b"".join(u64le(v) for v in vals))

    @staticmethod
    def accepts(v: int) -> bool:
        """Rejection-sampling predicate: a candidate is kept iff it is canonical."""
        return v < P

    def challenge(self) -> int:
        ctr = 0
        while True:
            h = hashlib.sha256(self.s + b"chal" + struct.pack("<I", ctr)).digest()
            v = int.from_bytes(h[:8], "little")
            if self.accepts(v):
                self.s = h
                return v
            ctr += 1


# --------------------------------------------------------------------------- commitments
def commit_bytes(raw: bytes, dtype: int, rows: int, cols: int) -> bytes:
    if len(raw) != rows * cols * _DT_BYTES[dtype]:
        raise ValueError("byte length does not match shape")
    top = hashlib.sha256()
    top.update(b"IMM-COMMIT-v1" + struct.pack("<I", dtype) + u64le(rows) + u64le(cols))
    for off in range(0, len(raw), LEAF_BYTES):
        top.update(hashlib.sha256(raw[off:off + LEAF_BYTES]).digest())
    return top.digest()


def _raw_le(M, rows: int, cols: int, dtype: int) -> bytes:
    fmt = {DT_I8: "b", DT_I16: "h", DT_I64: "q", DT_F64P: "Q"}[dtype]
    flat = [int(M[i][j]) for i in range(rows) for j in range(cols)]
    return struct.pack("<%d%s" % (len(flat), fmt), *flat)


def commit_matmul(A, B, C, m: int, d: int, n: int) -> dict:
    """Digests of A (int16), B (int8), C (int64) with their shapes."""
    return {
        "A": (commit_bytes(_raw_le(A, m, d, DT_I16), DT_I16, m, d), m, d, DT_I16),
        "B": (commit_bytes(_raw_le(B, d, n, DT_I8), DT_I8, d, n), d, n, DT_I8),
        "C": (commit_bytes(_raw_le(C, m, n, DT_I64), DT_I64, m, n), m, n, DT_I64),
    }


# --------------------------------------------------------------------------- sumcheck
def transcript_head(tr: Transcript, m: int, d: int, n: int, digests: Tuple[bytes, bytes, bytes]):
    """Absorb the statement, squeeze the row point rx and the column point ry."""
    tr.absorb(b"shap", u64le(m) + u64le(d) + u64le(n))
    tr.absorb(b"comA", digests[0])
    tr.absorb(b"comB", digests[1])
    tr.absorb(b"comC", digests[2])
    rx = [tr.challenge() for _ in range(ceil_log2(m))]
    ry = [tr.challenge() for _ in range(ceil_log2(n))]
    return rx, ry


def interpolate3(g0: int, g1: int, g2: int, r: int) -> int:
    """Value at r of the degree-<=2 polynomial through (0,g0), (1,g1), (2,g2)."""
    l0 = (r - 1) * (r - 2) % P * INV2 % P
    l1 = (-(r * (r - 2))) % P
    l2 = r * (r - 1) % P * INV2 % P
    return (g0 * l0 + g1 * l1 + g2 * l2) % P


def round_poly_by_definition(a_tab, b_tab, delta: int, prev_r: Sequence[int], t: int) -> int:
    """g_k(t) = sum over b in {0,1}^(delta-k) of a~(r_1..r_{k-1}, t, b) * b~(same point),
    each MLE evaluated by direct summation over the ORIGINAL length-2^delta tables."""
    k = len(prev_r) + 1
    rest = delta - k
    acc = 0
    for tail in range(1 << rest):
        tail_bits = [(tail >> (rest - 1 - u)) & 1 for u in range(rest)]
        pt = list(prev_r) + [t] + tail_bits
        acc = (acc + mle_table(a_tab, pt) * mle_table(b_tab, pt)) % P
    return acc


def prove(A, B, C, m: int, d: int, n: int, digests: Tuple[bytes, bytes, bytes],
          state_in: bytes = FS_INIT, trace: dict | None = None):
    """One matmul proof.  Returns (proof dict, state_out).

    The proof is produced for whatever C is handed in: c0 is C~(rx, ry).  The
    internal assertions hold iff C = A.B (up to the soundness error)."""
    mu, delta, nu = ceil_log2(m), ceil_log2(d), ceil_log2(n)
    D = 1 << delta
    tr = Transcript(state_in)
    rx, ry = transcript_head(tr, m, d, n, digests)

    # a[j] = A~(rx, j) and b[j] = B~(j, ry): partial evaluations by direct summation
    a_tab = [sum(eq_weight(i, rx) * enc(int(A[i][j])) for i in range(m)) % P if j < d else 0
             for j in range(D)]
    b_tab = [sum(eq_weight(y, ry) * enc(int(B[j][y])) for y in range(n)) % P if j < d else 0
             for j in range(D)]
    c0 = mle_matrix(C, m, n, rx, ry)
    tr.absorb_field(b"clmC", [c0])
    claim = c0

    g: List[int] = []
    rs: List[int] = []
    for _k in range(1, delta + 1):
        gk = [round_poly_by_definition(a_tab, b_tab, delta, rs, t) for t in (0, 1, 2)]
        if (gk[0] + gk[1]) % P != claim:
            raise AssertionError("round sum does not match the running claim")
        tr.absorb_field(b"rnd ", gk)
        r = tr.challenge()
        claim = interpolate3(gk[0], gk[1], gk[2], r)
        g.extend(gk)
        rs.append(r)

    vA = mle_matrix(A, m, d, rx, rs)
    vB = mle_matrix(B, d, n, rs, ry)
    if vA * vB % P != claim:
        raise AssertionError("final claim is not A~(rx,r) * B~(r,ry)")
    tr.absorb_field(b"fin ", [vA, vB])
    if trace is not None:
        trace.update(rx=rx, ry=ry, r=rs, a=a_tab, b=b_tab)
    proof = {"mu": mu, "delta": delta, "nu": nu, "c0": c0, "g": g, "vA": vA, "vB": vB}
    return proof, tr.s


# --------------------------------------------------------------------------- verify
ACCEPT = 0
REJ_ROUND_SUM = 1
REJ_FINAL = 2
REJ_OPEN_A = 3
REJ_OPEN_B = 4
REJ_OPEN_C = 5
REJ_COMMIT = 6
REJ_FORMAT = 7


def verify(proof: dict, m: int, d: int, n: int, digests: Tuple[bytes, bytes, bytes],
           state_in: bytes = FS_INIT, A=None, B=None, C=None):
    """Replay the transcript and check the proof.  Returns (code, state_out, fail_round)."""
    mu, delta, nu = ceil_log2(m), ceil_log2(d), ceil_log2(n)
    if (proof["mu"], proof["delta"], proof["nu"]) != (mu, delta, nu) or len(proof["g"]) != 3 * delta:
        return REJ_FORMAT, None, 0
    words = [proof["c0"], proof["vA"], proof["vB"]] + list(proof["g"])
    if any(not (0 <= w < P) for w in words):
        return REJ_FORMAT, None, 0
    if A is not None and commit_bytes(_raw_le(A, m, d, DT_I16), DT_I16, m, d) != digests[0]:
        return REJ_COMMIT, None, 0
    if B is not None and commit_bytes(_raw_le(B, d, n, DT_I8), DT_I8, d, n) != digests[1]:
        return REJ_COMMIT, None, 0
    if C is not None and commit_bytes(_raw_le(C, m, n, DT_I64), DT_I64, m, n) != digests[2]:
        return REJ_COMMIT, None, 0

    tr = Transcript(state_in)
    rx, ry = transcript_head(tr, m, d, n, digests)
    tr.absorb_field(b"clmC", [proof["c0"]])
    claim = proof["c0"]
    rs = []
    for k in range(delta):
        g0, g1, g2 = proof["g"][3 * k:3 * k + 3]
        if (g0 + g1) % P != claim:
            return REJ_ROUND_SUM, None, k + 1
        tr.absorb_field(b"rnd ", [g0, g1, g2])
        r = tr.challenge()
        claim = interpolate3(g0, g1, g2, r)
        rs.append(r)
    if proof["vA"] * proof["vB"] % P != claim:
        return REJ_FINAL, None, 0
    tr.absorb_field(b"fin ", [proof["vA"], proof["vB"]])
    if A is not None and mle_matrix(A, m, d, rx, rs) != proof["vA"]:
        return REJ_OPEN_A, None, 0
    if B is not None and mle_matrix(B, d, n, rs, ry) != proof["vB"]:
        return REJ_OPEN_B, None, 0
    if C is not None and mle_matrix(C, m, n, rx, ry) != proof["c0"]:
        return REJ_OPEN_C, None, 0
    return ACCEPT, tr.s, 0


def proof_words(proof: dict) -> List[int]:
    """Flat canonical word list used when comparing two proofs."""
    return [proof["mu"], proof["delta"], proof["nu"], proof["c0"]] + list(proof["g"]) + [proof["vA"], proof["vB"]]
