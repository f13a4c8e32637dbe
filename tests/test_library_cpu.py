"""CPU-side checks of libimm.so: it loads, exports what include/imm.h declares, and its
host-only entry points (commit, verify, transcript init) agree with the oracle.
No GPU compute is called here."""
import ctypes
import hashlib
import os
import re

import numpy as np
import pytest

from oracle import reference as ref
from paper_2602_22700_amd import binding as imm
from paper_2602_22700_amd import build as imm_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = ref.P


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(imm.LIB_PATH):
        imm_build.build_library(force=True)
    return imm.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "imm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(imm_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert "imm_commit_matmul" in names and "imm_mle_eval" in names
    assert "imm_sumcheck_matmul_prove" in names and "imm_verify" in names
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(imm.EXPORTS) == names


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(imm.Commit1) == 56 and ctypes.sizeof(imm.Commit) == 168
    assert ctypes.sizeof(imm.Proof) == 16 + 24 + 8 * 3 * imm.IMM_MAX_ROUNDS
    assert imm.Proof.g.offset == 40 and imm.Proof.c0.offset == 16


def test_fs_init_and_sha256_against_hashlib(lib):
    assert imm.imm_fs_init() == hashlib.sha256(b"IMM-FS-v1").digest() == ref.FS_INIT


@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 7), (64, 64, 64), (2, (1 << 20) + 3, 1), (130, 4100, 257)])
def test_commit_matches_oracle(lib, oracle_fast, shape):
    m, d, n = shape
    rng = np.random.default_rng(m * 1000 + n)
    A = rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
    B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
    C = rng.integers(-2**40, 2**40, size=(m, n), dtype=np.int64)
    com = imm.imm_commit_matmul(A, B, C, m, d, n)
    assert com.digests() == oracle_fast.commit_matmul(A, B, C)
    assert (com.A.rows, com.A.cols, com.A.dtype) == (m, d, imm.IMM_I16)
    assert (com.B.rows, com.B.cols, com.B.dtype) == (d, n, imm.IMM_I8)
    assert (com.C.rows, com.C.cols, com.C.dtype) == (m, n, imm.IMM_I64)
    # NULL entries are left untouched
    com2 = imm.imm_commit_matmul(None, B, None, m, d, n)
    assert bytes(com2.B.digest) == bytes(com.B.digest) and bytes(com2.A.digest) == bytes(32)


def test_commit_of_every_small_length_matches_hashlib(lib, oracle_fast):
    """Leaves of 1..200 bytes cross every padding case of SHA-256 (one and two final blocks), whichever
    compression routine the host CPU selects."""
    rng = np.random.default_rng(9)
    for n in range(1, 201):
        B = rng.integers(-128, 128, size=(1, n), dtype=np.int8)
        com = imm.imm_commit_matmul(None, B, None, 1, 1, n)
        assert bytes(com.B.digest) == oracle_fast.commit_array(B), n


def test_commit_rejects_bad_shapes(lib):
    with pytest.raises(imm.ImmError) as e:
        imm.imm_commit_matmul(None, None, None, 0, 1, 1)
    assert e.value.code == -2
    assert lib.imm_commit_matmul(None, None, None, 1, 1, 1, None) == -1


def to_proof(p: dict) -> imm.Proof:
    out = imm.Proof()
    out.version = 1
    out.mu, out.delta, out.nu = p["mu"], p["delta"], p["nu"]
    out.c0, out.vA, out.vB = p["c0"], p["vA"], p["vB"]
    for i, v in enumerate(p["g"]):
        out.g[i] = v
    return out


def make_case(oracle_fast, m, d, n, seed):
    rng = np.random.default_rng(seed)
    A = rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
    B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
    C = oracle_fast.matmul(A, B)
    com = imm.imm_commit_matmul(A, B, C, m, d, n)
    proof, s_out = oracle_fast.prove(A, B, C, com.digests())
    return A, B, C, com, proof, s_out


@pytest.mark.parametrize("shape", [(4, 4, 4), (1, 1, 1), (5, 6, 7), (1, 9, 3), (17, 1, 2), (64, 64, 64)])
def test_verify_accepts_oracle_proofs(lib, oracle_fast, shape):
    m, d, n = shape
    A, B, C, com, proof, s_out = make_case(oracle_fast, m, d, n, 77 + m + d + n)
    # without the matrices nothing ties c0, vA, vB to the commitments: consistent, but not an accept
    code, st, fr = imm.imm_verify(com, ref.FS_INIT, to_proof(proof))
    assert (code, st, fr) == (imm.IMM_REJ_UNOPENED, s_out, 0)
    assert oracle_fast.verify(proof, m, d, n, com.digests())[0] == 0      # the oracle's transcript-only replay
    for part in ((A, None, None), (None, B, None), (None, None, C), (A, B, None), (A, None, C), (None, B, C)):
        assert imm.imm_verify(com, ref.FS_INIT, to_proof(proof), *part)[0] == imm.IMM_REJ_UNOPENED
    code, st, fr = imm.imm_verify(com, ref.FS_INIT, to_proof(proof), A, B, C)
    assert (code, st, fr) == (0, s_out, 0)
    assert oracle_fast.verify(proof, m, d, n, com.digests(), A=A, B=B, C=C)[0] == 0


def test_a_proof_with_a_freely_chosen_claim_is_never_accepted_without_openings(lib, oracle_fast):
    """A prover that picks c0 at will and answers every round consistently passes all transcript checks;
    only the openings catch it.  The verifier must not report ACCEPT for it in any call form."""
    m, d, n = 4, 4, 4
    A, B, C, com, proof, _ = make_case(oracle_fast, m, d, n, 31)
    tr = ref.Transcript(ref.FS_INIT)
    tr.absorb(b"shap", ref.u64le(m) + ref.u64le(d) + ref.u64le(n))
    for tag, dg in zip((b"comA", b"comB", b"comC"), com.digests()):
        tr.absorb(tag, dg)
    for _ in range(2 + 2):
        tr.challenge()
    c0 = 123456789
    forged = dict(proof, c0=c0, g=[])
    tr.absorb_field(b"clmC", [c0])
    claim = c0
    for k in range(2):
        g = [claim, 0, (P - claim) % P]          # g(0) + g(1) = claim; a line through the two points
        forged["g"] += g
        tr.absorb_field(b"rnd ", g)
        r = tr.challenge()
        claim = ref.interpolate3(g[0], g[1], g[2], r)
    forged["vA"], forged["vB"] = claim, 1
    assert imm.imm_verify(com, ref.FS_INIT, to_proof(forged))[0] == imm.IMM_REJ_UNOPENED
    assert imm.imm_verify(com, ref.FS_INIT, to_proof(forged), A, B, C)[0] in (3, 4, 5)
    assert imm.imm_verify(com, ref.FS_INIT, to_proof(forged), None, None, C)[0] == 5


def test_verify_points_match_the_oracle_trace(lib, oracle_fast):
    rng = np.random.default_rng(8)
    A = rng.integers(-2**15, 2**15, size=(5, 9), dtype=np.int16)
    B = rng.integers(-128, 128, size=(9, 3), dtype=np.int8)
    C = oracle_fast.matmul(A, B)
    com = imm.imm_commit_matmul(A, B, C, 5, 9, 3)
    trace = {}
    proof, _ = oracle_fast.prove(A, B, C, com.digests(), trace=trace)
    rx, ry, r = imm.imm_verify_points(com, ref.FS_INIT, to_proof(proof))
    assert (rx, ry, r) == (trace["rx"], trace["ry"], trace["r"])
    # the three proof values are the openings at those points
    assert proof["c0"] == oracle_fast.mle_matrix(C, rx, ry)
    assert proof["vA"] == oracle_fast.mle_matrix(A, rx, r) and proof["vB"] == oracle_fast.mle_matrix(B, r, ry)


def test_verify_reject_codes_match_oracle_on_every_mutation(lib, oracle_fast):
    m, d, n = 4, 8, 4
    A, B, C, com, proof, s_out = make_case(oracle_fast, m, d, n, 5)
    dg = com.digests()
    muts = [("c0", None), ("vA", None), ("vB", None)] + [("g", k) for k in range(3 * proof["delta"])]
    for name, k in muts:
        bad = dict(proof, g=list(proof["g"]))
        if k is None:
            bad[name] = (bad[name] + 1) % P
        else:
            bad["g"][k] = (bad["g"][k] + 1) % P
        want = oracle_fast.verify(bad, m, d, n, dg, A=A, B=B, C=C)
        got = imm.imm_verify(com, ref.FS_INIT, to_proof(bad), A, B, C)
        assert got[0] == want[0] != 0 and got[2] == want[2], (name, k)
        want = oracle_fast.verify(bad, m, d, n, dg)
        got = imm.imm_verify(com, ref.FS_INIT, to_proof(bad))
        assert got[0] == want[0] != 0 and got[2] == want[2], (name, k)


def test_verify_format_commit_and_opening_rejections(lib, oracle_fast):
    m, d, n = 4, 4, 4
    A, B, C, com, proof, s_out = make_case(oracle_fast, m, d, n, 6)
    pr = to_proof(proof)
    bad = pr.copy(); bad.c0 = P
    assert imm.imm_verify(com, ref.FS_INIT, bad)[0] == 7
    bad = pr.copy(); bad.g[0] = 2**64 - 1
    assert imm.imm_verify(com, ref.FS_INIT, bad)[0] == 7
    bad = pr.copy(); bad.mu = 3
    assert imm.imm_verify(com, ref.FS_INIT, bad)[0] == 7
    bad = pr.copy(); bad.version = 2
    assert imm.imm_verify(com, ref.FS_INIT, bad)[0] == 7
    bad = pr.copy(); bad.g[3 * proof["delta"]] = 1   # junk after the last round
    assert imm.imm_verify(com, ref.FS_INIT, bad)[0] == 7
    # wrong starting state: the challenges differ, so a round sum or the final check fails
    assert imm.imm_verify(com, bytes(32), pr)[0] in (1, 2)
    # every single-entry perturbation of C: its digest no longer matches
    for i in range(m):
        for y in range(n):
            Cb = C.copy(); Cb[i, y] += 1
            assert imm.imm_verify(com, ref.FS_INIT, pr, A, B, Cb)[0] == 6
            # committed wrong C, sumcheck of the true product: opening of C fails
            comb = imm.imm_commit_matmul(A, B, Cb, m, d, n)
            pb, _ = oracle_fast.prove(A, B, None, comb.digests())
            assert imm.imm_verify(comb, ref.FS_INIT, to_proof(pb))[0] == imm.IMM_REJ_UNOPENED
            assert imm.imm_verify(comb, ref.FS_INIT, to_proof(pb), None, None, Cb)[0] == 5
    Ab = A.copy(); Ab[0, 0] ^= 1
    assert imm.imm_verify(com, ref.FS_INIT, pr, Ab, None, None)[0] == 6
    # openings of A and B: statement committed to (Ab, B, C) but proof built from A
    comA = imm.imm_commit_matmul(Ab, B, C, m, d, n)
    pA, _ = oracle_fast.prove(A, B, None, comA.digests())
    assert imm.imm_verify(comA, ref.FS_INIT, to_proof(pA), Ab, None, None)[0] == 3
    Bb = B.copy(); Bb[1, 2] ^= 1
    comB = imm.imm_commit_matmul(A, Bb, C, m, d, n)
    pB, _ = oracle_fast.prove(A, B, None, comB.digests())
    assert imm.imm_verify(comB, ref.FS_INIT, to_proof(pB), None, Bb, None)[0] == 4


def test_verify_argument_errors(lib, oracle_fast):
    A, B, C, com, proof, _ = make_case(oracle_fast, 2, 2, 2, 1)
    pr = to_proof(proof)
    st = (ctypes.c_uint8 * 32)()
    assert lib.imm_verify(None, st, ctypes.byref(pr), None, None, None, None, None) == -1
    bad = imm.Commit()
    ctypes.memmove(ctypes.byref(bad), ctypes.byref(com), ctypes.sizeof(com))
    bad.B.rows = 3
    assert lib.imm_verify(ctypes.byref(bad), st, ctypes.byref(pr), None, None, None, None, None) == -2
    bad.B.rows = 2
    bad.C.dtype = imm.IMM_I16
    assert lib.imm_verify(ctypes.byref(bad), st, ctypes.byref(pr), None, None, None, None, None) == -3


def test_verify_chained_states(lib, oracle_fast):
    rng = np.random.default_rng(12)
    items, coms = [], []
    for t in range(3):
        A = rng.integers(-2**15, 2**15, size=(3, 8), dtype=np.int16)
        B = rng.integers(-128, 128, size=(8, 5), dtype=np.int8)
        C = oracle_fast.matmul(A, B)
        com = imm.imm_commit_matmul(A, B, C, 3, 8, 5)
        items.append((A, B, C, com.digests()))
        coms.append(com)
    proofs, states = oracle_fast.prove_chain(items, chained=True)
    s = ref.FS_INIT
    for com, pr, st in zip(coms, proofs, states):
        code, s_next, _ = imm.imm_verify(com, s, to_proof(pr))
        assert code == imm.IMM_REJ_UNOPENED and s_next == st
        A, B, C, _ = items[coms.index(com)]
        assert imm.imm_verify(com, s, to_proof(pr), A, B, C) == (0, st, 0)
        s = s_next


def rejecting_state():
    """tests/golden/rejecting_state.txt: a state whose first challenge candidate is >= p, with the
    oracle's outcome (written by tests/golden/find_rejecting_state.py from oracle/reference.py)."""
    kv = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "rejecting_state.txt")):
        if " = " in line and not line.startswith("#"):
            k, v = line.strip().split(" = ")
            kv[k] = v
    return (bytes.fromhex(kv["state"]), int(kv["first_candidate"], 16), int(kv["challenge"], 16),
            bytes.fromhex(kv["state_after"]))


def test_challenge_takes_the_rejection_branch_like_the_oracle(lib):
    """The library's host transcript on a state whose first candidate is not canonical (probability
    2^-32 per challenge): it must move on to the next counter, not reduce or keep the candidate."""
    state, first, want, after = rejecting_state()
    # the stored values are the oracle's, and the first candidate is indeed rejected
    assert first >= P
    assert int.from_bytes(hashlib.sha256(state + b"chal" + (0).to_bytes(4, "little")).digest()[:8], "little") == first
    tr = ref.Transcript(state)
    assert tr.challenge() == want and tr.s == after and want < P
    assert imm.imm_transcript_challenge(state) == (want, after)
    # ordinary states: the same as the oracle, challenge after challenge
    s_lib, tr = ref.FS_INIT, ref.Transcript(ref.FS_INIT)
    for _ in range(20):
        v, s_lib = imm.imm_transcript_challenge(s_lib)
        assert v == tr.challenge() and s_lib == tr.s


def test_host_sources_under_address_and_undefined_behaviour_sanitizers(oracle_fast, tmp_path):
    """The library's CPU sources (SHA-256 with its instruction-set dispatch, transcript, commitments,
    verifier) compiled with -fsanitize=address,undefined into a small driver; its results on a few
    statements, one of them with a matrix spanning several commitment leaves and a state that takes
    the rejection branch of the challenge derivation, equal the oracle's, and no sanitizer speaks."""
    import shutil
    import subprocess
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host compiler")
    csrc = os.path.join(ROOT, "paper_2602_22700_amd", "csrc")
    exe = str(tmp_path / "host_san")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-o", exe, os.path.join(ROOT, "tests", "host_sanitize_main.cpp")] + \
          [os.path.join(csrc, f) for f in ("sha256.cpp", "transcript.cpp", "commit.cpp", "verify.cpp")] + ["-lpthread"]
    subprocess.check_call(cmd)
    rej_state = rejecting_state()[0]
    for (m, d, n), state in (((4, 4, 4), ref.FS_INIT), ((3, 9, 5), rej_state), ((1, 1, 1), ref.FS_INIT),
                             ((2, (1 << 20) + 5, 3), ref.FS_INIT)):
        rng = np.random.default_rng(m * 100 + n)
        A = rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
        B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
        C = oracle_fast.matmul(A, B)
        dg = oracle_fast.commit_matmul(A, B, C)
        trace = {}
        proof, s_out = oracle_fast.prove(A, B, C, dg, state, trace=trace)
        text = "%d %d %d\n" % (m, d, n) + " ".join(map(str, A.reshape(-1).tolist())) + "\n" + \
            " ".join(map(str, B.reshape(-1).tolist())) + "\n" + " ".join(map(str, C.reshape(-1).tolist())) + "\n" + \
            state.hex() + "\n" + "%d %d %d %d %d %d\n" % (proof["mu"], proof["delta"], proof["nu"], proof["c0"],
                                                           proof["vA"], proof["vB"]) + " ".join(map(str, proof["g"])) + "\n"
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        run = subprocess.run([exe], input=text, capture_output=True, text=True, env=env, timeout=300)
        assert run.returncode == 0 and run.stderr == "", run.stderr[-2000:]
        out = run.stdout.split("\n")
        tr = ref.Transcript(state)
        want_ch = tr.challenge()
        assert out[0] == "commit 0" and out[1:4] == [x.hex() for x in dg]
        assert out[4] == "verify_full 0 0" and out[5] == s_out.hex()
        assert out[6] == "verify_transcript %d 0" % imm.IMM_REJ_UNOPENED and out[7] == s_out.hex()
        assert out[8] == " ".join(["points", "0"] + [str(v) for v in trace["rx"] + trace["ry"] + trace["r"]])
        assert out[9] == "challenge 0 %d" % want_ch and out[10] == tr.s.hex()
        assert out[11] == "verify_bad_C %d" % 6


def test_host_side_rounds_match_the_oracle(oracle_fast, tmp_path):
    """The rounds that the prover's host thread computes on short tables (sums of 128-bit products
    reduced once, fold in place), compiled on their own with the sanitizers: g(0), g(1), g(2) and the
    folded tables equal the oracle's on random tables, on tables of p - 1 throughout (the largest
    products and the most carries) and on the shortest table."""
    import shutil
    import subprocess
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host compiler")
    exe = str(tmp_path / "host_rounds")
    subprocess.check_call([cxx, "-std=c++17", "-O2", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-static-libasan", "-o", exe, os.path.join(ROOT, "tests", "host_rounds_main.cpp")])
    rng = np.random.default_rng(77)
    P = ref.P
    cases = []
    for L in (2, 4, 64, 1024):
        cases.append((rng.integers(0, P, size=L, dtype=np.uint64), rng.integers(0, P, size=L, dtype=np.uint64),
                      int(rng.integers(0, P, dtype=np.uint64))))
    cases.append((np.full(1024, P - 1, dtype=np.uint64), np.full(1024, P - 1, dtype=np.uint64), P - 1))
    cases.append((np.full(8, P - 1, dtype=np.uint64), np.zeros(8, dtype=np.uint64), 0))
    for a, b, r in cases:
        L = len(a)
        text = "%d\n%s\n%s\n%d\n" % (L, " ".join(map(str, a.tolist())), " ".join(map(str, b.tolist())), r)
        run = subprocess.run([exe], input=text, capture_output=True, text=True, timeout=60)
        assert run.returncode == 0 and run.stderr == "", run.stderr[-2000:]
        lines = run.stdout.strip().split("\n")
        h = L // 2
        # the definition, in Python integers
        g0 = sum(int(a[i]) * int(b[i]) for i in range(h)) % P
        g1 = sum(int(a[i + h]) * int(b[i + h]) for i in range(h)) % P
        g2 = sum((2 * int(a[i + h]) - int(a[i])) * (2 * int(b[i + h]) - int(b[i])) for i in range(h)) % P
        assert [int(v) for v in lines[0].split()] == [g0, g1, g2] == oracle_fast.round_evals(a.copy(), b.copy(), L)
        fa, fb = a.copy(), b.copy()
        oracle_fast.fold(fa, L, r)
        oracle_fast.fold(fb, L, r)
        assert [int(v) for v in lines[1].split()] == fa[:h].tolist()
        assert [int(v) for v in lines[2].split()] == fb[:h].tolist()
