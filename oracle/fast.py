"""Tier-1 oracle driver: numpy buffers + the plain-C arithmetic in oracle/native.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  The protocol schedule
below is the one documented at the top of ``oracle/reference.py``; hashing is
``hashlib``; the field sums run in ``imm_oracle.c`` (``unsigned __int128 % p``).
Compared with tier 0 the only differences are that eq vectors are tabulated
first (doubling recurrence) and that the round polynomials use the fold
recurrence a'[i] = a[i] + r (a[i+h] - a[i]); both are checked against the
summation definitions of tier 0 in the test-suite.
"""
from __future__ import annotations

import ctypes
import hashlib
import os
import struct
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

from .reference import (ACCEPT, DT_F64P, DT_I8, DT_I16, DT_I64, FS_INIT, INV2, LEAF_BYTES, P,
                        REJ_COMMIT, REJ_FINAL, REJ_FORMAT, REJ_OPEN_A, REJ_OPEN_B, REJ_OPEN_C,
                        REJ_ROUND_SUM, Transcript, ceil_log2, interpolate3, transcript_head)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "native", "imm_oracle.c")
_LIB = os.path.join(_HERE, "native", "libimm_oracle.so")
_lib = None

_NP_DT = {np.dtype(np.int8): DT_I8, np.dtype(np.int16): DT_I16, np.dtype(np.int64): DT_I64,
          np.dtype(np.uint64): DT_F64P}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP for the row loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u64, sz, vp, i32 = ctypes.c_uint64, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int
        L.orc_threads.restype = i32
        for name in ("orc_mul", "orc_add", "orc_sub"):
            getattr(L, name).restype = u64
            getattr(L, name).argtypes = [u64, u64]
        L.orc_enc.restype = u64
        L.orc_enc.argtypes = [ctypes.c_int64]
        L.orc_encode.argtypes = [vp, i32, sz, vp]
        L.orc_eq_vector.argtypes = [vp, i32, vp]
        L.orc_partial_over_rows.argtypes = [vp, i32, sz, sz, sz, vp, vp]
        L.orc_partial_over_cols.argtypes = [vp, i32, sz, sz, sz, vp, vp]
        L.orc_mle_matrix.restype = u64
        L.orc_mle_matrix.argtypes = [vp, i32, sz, sz, sz, vp, vp]
        L.orc_round_evals.argtypes = [vp, vp, sz, vp]
        L.orc_fold.argtypes = [vp, sz, u64]
        L.orc_matmul_i16_i8.argtypes = [vp, vp, sz, sz, sz, vp]
        _lib = L
    return _lib


def threads() -> int:
    return int(lib().orc_threads())


def _ptr(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _dt(a: np.ndarray) -> int:
    return _NP_DT[a.dtype]


# --------------------------------------------------------------------------- arithmetic
def encode(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x)
    out = np.empty(x.shape, dtype=np.uint64)
    lib().orc_encode(_ptr(x), _dt(x), x.size, _ptr(out))
    return out


def eq_vector(point: Sequence[int]) -> np.ndarray:
    t = len(point)
    pt = np.array([int(v) for v in point], dtype=np.uint64)
    out = np.empty(1 << t, dtype=np.uint64)
    lib().orc_eq_vector(_ptr(pt), t, _ptr(out))
    return out


def partial_over_rows(T: np.ndarray, eq_rows: np.ndarray) -> np.ndarray:
    """out[j] = sum_i eq_rows[i] T[i][j]; eq_rows may be longer than T has rows."""
    T = np.ascontiguousarray(T)
    rows, cols = T.shape
    assert eq_rows.size >= rows
    out = np.empty(cols, dtype=np.uint64)
    lib().orc_partial_over_rows(_ptr(T), _dt(T), rows, cols, cols, _ptr(eq_rows), _ptr(out))
    return out


def partial_over_cols(T: np.ndarray, eq_cols: np.ndarray) -> np.ndarray:
    """out[i] = sum_j eq_cols[j] T[i][j]."""
    T = np.ascontiguousarray(T)
    rows, cols = T.shape
    assert eq_cols.size >= cols
    out = np.empty(rows, dtype=np.uint64)
    lib().orc_partial_over_cols(_ptr(T), _dt(T), rows, cols, cols, _ptr(eq_cols), _ptr(out))
    return out


def mle_matrix(T: np.ndarray, prow: Sequence[int], pcol: Sequence[int]) -> int:
    T = np.ascontiguousarray(T)
    rows, cols = T.shape
    assert len(prow) == ceil_log2(rows) and len(pcol) == ceil_log2(cols)
    er, ec = eq_vector(prow), eq_vector(pcol)
    return int(lib().orc_mle_matrix(_ptr(T), _dt(T), rows, cols, cols, _ptr(er), _ptr(ec)))


def round_evals(a: np.ndarray, b: np.ndarray, L: int):
    g = np.zeros(3, dtype=np.uint64)
    lib().orc_round_evals(_ptr(a), _ptr(b), L, _ptr(g))
    return [int(v) for v in g]


def fold(x: np.ndarray, L: int, r: int) -> None:
    lib().orc_fold(_ptr(x), L, int(r))


def matmul(A: np.ndarray, B: np.ndarray) -> np.ndarray:
    A = np.ascontiguousarray(A, dtype=np.int16)
    B = np.ascontiguousarray(B, dtype=np.int8)
    m, d = A.shape
    d2, n = B.shape
    assert d == d2
    C = np.empty((m, n), dtype=np.int64)
    lib().orc_matmul_i16_i8(_ptr(A), _ptr(B), m, d, n, _ptr(C))
    return C


# --------------------------------------------------------------------------- commitments
def commit_array(M: np.ndarray) -> bytes:
    M = np.ascontiguousarray(M)
    rows, cols = M.shape
    raw = memoryview(M).cast("B")
    top = hashlib.sha256()
    top.update(b"IMM-COMMIT-v1" + struct.pack("<I", _dt(M)) + struct.pack("<Q", rows) + struct.pack("<Q", cols))
    for off in range(0, len(raw), LEAF_BYTES):
        top.update(hashlib.sha256(raw[off:off + LEAF_BYTES]).digest())
    return top.digest()


def commit_matmul(A: np.ndarray, B: np.ndarray, C: np.ndarray) -> Tuple[bytes, bytes, bytes]:
    assert A.dtype == np.int16 and B.dtype == np.int8 and C.dtype == np.int64
    return commit_array(A), commit_array(B), commit_array(C)


# --------------------------------------------------------------------------- prove / verify
def prove(A: np.ndarray, B: np.ndarray, C: Optional[np.ndarray], digests: Tuple[bytes, bytes, bytes],
          state_in: bytes = FS_INIT, trace: Optional[dict] = None, check: bool = True):
    """One matmul proof; same schedule as ``reference.prove``.

    With ``C=None`` the first claim is taken as sum_j a[j] b[j] (which equals
    C~(rx, ry) exactly when C = A.B); this is what a prover that does not hold C
    computes, and is the form timed as the CPU baseline."""
    m, d = A.shape
    d2, n = B.shape
    assert d == d2
    mu, delta, nu = ceil_log2(m), ceil_log2(d), ceil_log2(n)
    D = 1 << delta
    tr = Transcript(state_in)
    rx, ry = transcript_head(tr, m, d, n, digests)
    eqx, eqy = eq_vector(rx), eq_vector(ry)

    a = np.zeros(D, dtype=np.uint64)
    b = np.zeros(D, dtype=np.uint64)
    a[:d] = partial_over_rows(A, eqx)
    b[:d] = partial_over_cols(B, eqy)
    if trace is not None:
        trace.update(rx=rx, ry=ry, eqx=eqx.copy(), eqy=eqy.copy(), a=a.copy(), b=b.copy())

    if C is not None:
        c0 = mle_matrix(C, rx, ry)
    else:
        g_first = round_evals(a, b, D) if delta > 0 else None
        c0 = (g_first[0] + g_first[1]) % P if delta > 0 else int(lib().orc_mul(int(a[0]), int(b[0])))
    tr.absorb_field(b"clmC", [c0])
    claim = c0

    g, rs = [], []
    L = D
    for _k in range(delta):
        gk = round_evals(a, b, L)
        if check and (gk[0] + gk[1]) % P != claim:
            raise AssertionError("round sum does not match the running claim")
        tr.absorb_field(b"rnd ", gk)
        r = tr.challenge()
        claim = interpolate3(gk[0], gk[1], gk[2], r)
        fold(a, L, r)
        fold(b, L, r)
        L //= 2
        g.extend(gk)
        rs.append(r)

    if check:
        # openings from the raw matrices, not from the folded tables
        vA = mle_matrix(A, rx, rs)
        vB = mle_matrix(B, rs, ry)
        if vA != int(a[0]) or vB != int(b[0]):
            raise AssertionError("folded tables disagree with the direct openings")
        if vA * vB % P != claim:
            raise AssertionError("final claim is not A~(rx,r) * B~(r,ry)")
    else:
        vA, vB = int(a[0]), int(b[0])
    tr.absorb_field(b"fin ", [vA, vB])
    if trace is not None:
        trace.update(r=rs)
    proof = {"mu": mu, "delta": delta, "nu": nu, "c0": c0, "g": g, "vA": vA, "vB": vB}
    return proof, tr.s


def verify(proof: dict, m: int, d: int, n: int, digests: Tuple[bytes, bytes, bytes],
           state_in: bytes = FS_INIT, A: Optional[np.ndarray] = None, B: Optional[np.ndarray] = None,
           C: Optional[np.ndarray] = None):
    """Same checks and reject codes as ``reference.verify``; returns (code, state_out, fail_round)."""
    mu, delta, nu = ceil_log2(m), ceil_log2(d), ceil_log2(n)
    if (proof["mu"], proof["delta"], proof["nu"]) != (mu, delta, nu) or len(proof["g"]) != 3 * delta:
        return REJ_FORMAT, None, 0
    words = [proof["c0"], proof["vA"], proof["vB"]] + list(proof["g"])
    if any(not (0 <= w < P) for w in words):
        return REJ_FORMAT, None, 0
    for M, dg in ((A, digests[0]), (B, digests[1]), (C, digests[2])):
        if M is not None and commit_array(M) != dg:
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
    if A is not None and mle_matrix(A, rx, rs) != proof["vA"]:
        return REJ_OPEN_A, None, 0
    if B is not None and mle_matrix(B, rs, ry) != proof["vB"]:
        return REJ_OPEN_B, None, 0
    if C is not None and mle_matrix(C, rx, ry) != proof["c0"]:
        return REJ_OPEN_C, None, 0
    return ACCEPT, tr.s, 0


def prove_chain(items, chained: bool, state_in: bytes = FS_INIT, check: bool = True):
    """Several proofs in order.  chained: the state threads through proof t -> t+1; otherwise
    every proof starts from state_in.  items: iterable of (A, B, C_or_None, digests).
    Returns (proofs, states) with states[t] the transcript state after proof t."""
    proofs, states, s = [], [], state_in
    for (A, B, C, dg) in items:
        pr, s_out = prove(A, B, C, dg, s if chained else state_in, check=check)
        proofs.append(pr)
        states.append(s_out)
        if chained:
            s = s_out
    return proofs, states
