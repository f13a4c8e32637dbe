"""GPU parity: every output of the HIP path is compared bit for bit with the CPU oracle
on the same seeded inputs.  All calls go through the C ABI (ctypes binding).  Integer and
field work, so the bar is exact equality everywhere."""
import ctypes
import os
import random

import numpy as np
import pytest

from oracle import reference as ref
from paper_2602_22700_amd import binding as imm
from paper_2602_22700_amd import workloads

pytestmark = pytest.mark.gpu
P = ref.P


@pytest.fixture(scope="module")
def torch():
    import torch as t
    if not t.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    return t


@pytest.fixture(scope="module")
def ctx(torch):
    c = imm.Context(0)
    yield c
    c.close()


def dev(torch, x: np.ndarray):
    x = np.ascontiguousarray(x)
    if x.dtype == np.uint64:  # move the bits as int64, then relabel
        return torch.from_numpy(x.view(np.int64)).cuda().view(torch.uint64)
    return torch.from_numpy(x).cuda()


def host_u64(t) -> np.ndarray:
    return t.contiguous().view(torch_mod().int64).cpu().numpy().view(np.uint64)


def torch_mod():
    import torch as t
    return t


def zeros_u64(torch, n):
    return torch.zeros(n, dtype=torch.int64, device="cuda").view(torch.uint64)


def exact_c(torch, A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """C = A.B as int64 via an exact float64 GEMM on the device (|C| < 2^36)."""
    C = dev(torch, A).double() @ dev(torch, B).double()
    return C.round().to(torch.int64).cpu().numpy()


def freivalds(A, B, C, seed=0):
    rng = np.random.default_rng(seed)
    v = rng.integers(0, 1 << 10, size=B.shape[1]).astype(np.int64)
    assert np.array_equal(C @ v, A.astype(np.int64) @ (B.astype(np.int64) @ v))


# ------------------------------------------------------------------ K1 encode
def test_encode_exhaustive_int8_int16(torch, ctx, oracle_fast):
    for arr in (np.arange(-128, 128, dtype=np.int8), np.arange(-32768, 32768, dtype=np.int16)):
        got = host_u64(ctx.imm_encode(dev(torch, arr)))
        assert np.array_equal(got, oracle_fast.encode(arr))


@pytest.mark.parametrize("count", [0, 1, 2, 3, 255, 256, 257, 1000003])
def test_encode_ragged_counts_and_misaligned_views(torch, ctx, oracle_fast, count):
    rng = np.random.default_rng(count)
    for dt in (np.int8, np.int16, np.int64):
        info = np.iinfo(dt)
        x = rng.integers(info.min, info.max, size=count + 3, dtype=dt, endpoint=True)
        if count >= 2:
            x[3], x[4] = info.min, info.max
        xd = dev(torch, x)
        for off in (0, 1, 3):
            src = xd[off:off + count]
            dst_full = zeros_u64(torch, count + 1)
            for doff in (0, 1):
                dst = dst_full[doff:doff + count]
                ctx.imm_encode(src, dst)
                assert np.array_equal(host_u64(dst), oracle_fast.encode(x[off:off + count]))


# ------------------------------------------------------------------ MLE evaluation (K2 + K3 + dot)
@pytest.mark.parametrize("shape", [(1, 1), (1, 7), (9, 1), (5, 6), (64, 64), (3, 1025), (130, 517), (257, 300),
                                   (1000, 4096), (37, 14336), (9, 8208), (3, 16)])
@pytest.mark.parametrize("dt", [np.int8, np.int16, np.int64, np.uint64])
def test_mle_eval_matches_oracle(torch, ctx, oracle_fast, shape, dt):
    rows, cols = shape
    rnd = random.Random(rows * 7919 + cols)
    rng = np.random.default_rng(rows * 31 + cols)
    if dt == np.uint64:
        T = rng.integers(0, P, size=shape, dtype=np.uint64)
        T.reshape(-1)[0] = P - 1
    else:
        info = np.iinfo(dt)
        T = rng.integers(info.min, info.max, size=shape, dtype=dt, endpoint=True)
    pr = [rnd.randrange(P) for _ in range(ref.ceil_log2(rows))]
    pc = [rnd.randrange(P) for _ in range(ref.ceil_log2(cols))]
    want = oracle_fast.mle_matrix(T, pr, pc)
    assert ctx.imm_mle_eval(dev(torch, T), pr, pc) == want


def test_mle_eval_boolean_point_and_leading_dimension(torch, ctx, oracle_fast):
    rng = np.random.default_rng(4)
    full = rng.integers(-128, 128, size=(40, 700), dtype=np.int8)
    fd = dev(torch, full)
    # a 33 x 515 window with ld = 700, starting at an odd column (exercises the unaligned path)
    for (r0, c0, rows, cols) in [(0, 0, 33, 515), (3, 1, 33, 515), (2, 6, 16, 256)]:
        win = full[r0:r0 + rows, c0:c0 + cols]
        sub = fd[r0:, c0:]
        tr, tc = ref.ceil_log2(rows), ref.ceil_log2(cols)
        i, j = rows - 1, cols - 2
        pr = [(i >> (tr - k)) & 1 for k in range(1, tr + 1)]
        pc = [(j >> (tc - k)) & 1 for k in range(1, tc + 1)]
        got = ctx.imm_mle_eval(sub, pr, pc, rows=rows, cols=cols, ld=700)
        assert got == ref.enc(int(win[i, j]))
        rnd = random.Random(5)
        pr = [rnd.randrange(P) for _ in range(tr)]
        pc = [rnd.randrange(P) for _ in range(tc)]
        assert ctx.imm_mle_eval(sub, pr, pc, rows=rows, cols=cols, ld=700) == \
            oracle_fast.mle_matrix(np.ascontiguousarray(win), pr, pc)


# ------------------------------------------------------------------ K4 round kernel on caller tables
@pytest.mark.parametrize("logL", [1, 2, 3, 8, 12, 14, 15, 16, 17, 20, 22])
def test_round_fold_eval_matches_oracle(torch, ctx, oracle_fast, logL):
    L = 1 << logL
    rng = np.random.default_rng(logL)
    a = rng.integers(0, P, size=L, dtype=np.uint64)
    b = rng.integers(0, P, size=L, dtype=np.uint64)
    a[0], b[0], a[-1] = P - 1, P - 1, P - 1
    ad, bd = dev(torch, a), dev(torch, b)
    rnd = random.Random(logL)
    assert ctx.imm_round_fold_eval(ad, bd, L) == oracle_fast.round_evals(a, b, L)
    assert np.array_equal(host_u64(ad), a) and np.array_equal(host_u64(bd), b)  # evaluation does not write
    cur = L
    for _ in range(min(logL, 4)):
        r = rnd.randrange(P)
        g = ctx.imm_round_fold_eval(ad, bd, cur, fold_r=r)
        oracle_fast.fold(a, cur, r)
        oracle_fast.fold(b, cur, r)
        cur //= 2
        assert np.array_equal(host_u64(ad)[:cur], a[:cur]) and np.array_equal(host_u64(bd)[:cur], b[:cur])
        if cur >= 2:
            assert g == oracle_fast.round_evals(a, b, cur)
        else:
            assert g == [int(a[0]), int(b[0]), 0]


# ------------------------------------------------------------------ whole proofs
def check_proof(torch, ctx, oracle_fast, A, B, C=None, state=ref.FS_INIT, intermediates=True, verify_open=True):
    m, d = A.shape
    n = B.shape[1]
    if C is None:
        C = oracle_fast.matmul(A, B)
    com = imm.imm_commit_matmul(A, B, C, m, d, n)
    assert com.digests() == oracle_fast.commit_matmul(A, B, C)
    trace = {}
    want, s_want = oracle_fast.prove(A, B, C, com.digests(), state, trace=trace)
    ctx.imm_ctx_set_option(imm.IMM_OPT_DEBUG_SNAPSHOTS, 1 if intermediates else 0)
    Ad, Bd = dev(torch, A), dev(torch, B)
    got, s_got = ctx.imm_sumcheck_matmul_prove(Ad, Bd, com, state)
    assert got.words() == ref.proof_words(want)
    assert s_got == s_want
    if intermediates:
        assert ctx.imm_debug_fetch(4).tolist() == trace["rx"] and ctx.imm_debug_fetch(5).tolist() == trace["ry"]
        assert ctx.imm_debug_fetch(6).tolist() == trace["r"]
        assert np.array_equal(ctx.imm_debug_fetch(0), trace["eqx"])
        assert np.array_equal(ctx.imm_debug_fetch(1), trace["eqy"])
        assert np.array_equal(ctx.imm_debug_fetch(2), trace["a"])
        assert np.array_equal(ctx.imm_debug_fetch(3), trace["b"])
    ctx.imm_ctx_set_option(imm.IMM_OPT_DEBUG_SNAPSHOTS, 0)
    # the narrow-read mode and pre-encoded operands give the same bytes
    ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 0)
    got2, s2 = ctx.imm_sumcheck_matmul_prove(Ad, Bd, com, state)
    ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)
    assert got2.words() == got.words() and s2 == s_got
    # the default hashes on the host through the mailbox while the round kernel runs;
    # the same proof with the transcript hashed by the round kernel itself
    ctx.imm_ctx_set_option(imm.IMM_OPT_TRANSCRIPT, imm.IMM_TRANSCRIPT_DEVICE)
    got4, s4 = ctx.imm_sumcheck_matmul_prove(Ad, Bd, com, state)
    ctx.imm_ctx_set_option(imm.IMM_OPT_TRANSCRIPT, imm.IMM_TRANSCRIPT_HOST)
    assert got4.words() == got.words() and s4 == s_got
    Af, Bf = ctx.imm_encode(Ad), ctx.imm_encode(Bd)
    got3, s3 = ctx.imm_sumcheck_matmul_prove(Af, Bf, com, state)
    assert got3.words() == got.words() and s3 == s_got
    # weights widened beforehand, activations read as they are stored
    ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 0)
    got6, s6 = ctx.imm_sumcheck_matmul_prove(Ad, Bf, com, state)
    ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)
    assert got6.words() == got.words() and s6 == s_got
    # wherever the round kernel hands its tables to the host (never, after all but one round, late), the same bytes
    try:
        for t in (0, 1, 3, 6, imm.IMM_HOST_TAIL_MAX):
            ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, t)
            got5, s5 = ctx.imm_sumcheck_matmul_prove(Af, Bf, com, state)
            assert got5.words() == got.words() and s5 == s_got, t
    finally:
        ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, imm.IMM_HOST_TAIL_DEFAULT)
    # the library's own verifier accepts it
    if verify_open:
        assert imm.imm_verify(com, state, got, A, B, C) == (0, s_want, 0)
    else:
        assert imm.imm_verify(com, state, got) == (imm.IMM_REJ_UNOPENED, s_want, 0)
    return got, s_got


@pytest.mark.parametrize("shape", [(1, 1, 1), (1, 5, 3), (3, 1, 2), (2, 2, 2), (4, 4, 4), (5, 6, 7), (2, 9, 1),
                                   (33, 70, 129), (17, 300, 1030), (129, 1025, 515), (7, 2048, 2049),
                                   (2, 32768, 5), (2, 65539, 3), (1, 131072, 2), (5, 67, 8208), (19, 40, 4096), (8, 8, 16),
                                   (2, 200, 3), (3, 1000, 5), (2, 4096, 3), (2, 5000, 2), (3, 16384, 2)])
def test_prove_small_and_ragged_shapes(torch, ctx, oracle_fast, shape):
    m, d, n = shape
    rng = np.random.default_rng(m * 10007 + d * 101 + n)
    A = rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
    B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
    check_proof(torch, ctx, oracle_fast, A, B)


def test_prove_extreme_values(torch, ctx, oracle_fast):
    """All operands at the ends of their ranges: the lazy accumulators see their largest terms."""
    for av, bv in [(-32768, -128), (32767, 127), (-32768, 127), (-1, -1)]:
        A = np.full((64, 1024), av, dtype=np.int16)
        B = np.full((1024, 1536), bv, dtype=np.int8)
        check_proof(torch, ctx, oracle_fast, A, B)


def test_prove_operands_at_odd_addresses(torch, ctx, oracle_fast):
    """Raw operands that start one element into a buffer (2-byte aligned int16, odd-address int8): the
    widening, alone or sharing a launch, and the reductions take their element-wise forms."""
    rng = np.random.default_rng(404)
    for (m, d, n) in ((7, 33, 19), (16, 256, 130), (3, 1000, 257)):
        A = rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
        B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
        C = oracle_fast.matmul(A, B)
        com = imm.imm_commit_matmul(A, B, C, m, d, n)
        want, s_want = oracle_fast.prove(A, B, C, com.digests())
        bufA = torch.zeros(m * d + 8, dtype=torch.int16, device="cuda")
        bufB = torch.zeros(d * n + 8, dtype=torch.int8, device="cuda")
        for offA, offB in ((1, 1), (0, 3), (1, 0)):
            bufA[offA:offA + m * d] = torch.from_numpy(A.reshape(-1)).cuda()
            bufB[offB:offB + d * n] = torch.from_numpy(B.reshape(-1)).cuda()
            Ad, Bd = bufA[offA:offA + m * d].view(m, d), bufB[offB:offB + d * n].view(d, n)
            try:
                for widen, fused in ((1, 1), (1, 0), (0, 1)):
                    ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, widen)
                    ctx.imm_ctx_set_option(imm.IMM_OPT_FUSE_REDUCTIONS, fused)
                    got, s_got = ctx.imm_sumcheck_matmul_prove(Ad, Bd, com, imm.imm_fs_init())
                    assert got.words() == ref.proof_words(want) and s_got == s_want, (m, d, n, offA, offB, widen, fused)
            finally:
                ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)
                ctx.imm_ctx_set_option(imm.IMM_OPT_FUSE_REDUCTIONS, 1)


def test_config1_tiny(torch, ctx, oracle_fast):
    A, B = workloads.tiny()
    got, _ = check_proof(torch, ctx, oracle_fast, A, B)
    assert (got.mu, got.delta, got.nu) == (6, 6, 6)
    # tier 0 (pure Python, by definition) agrees as well
    C = oracle_fast.matmul(A, B)
    p0, _ = ref.prove(A.tolist(), B.tolist(), C.tolist(), 64, 64, 64, oracle_fast.commit_matmul(A, B, C))
    assert got.words() == ref.proof_words(p0)


def test_config2_attention_projection(torch, ctx, oracle_fast):
    A, B = workloads.attn_proj()
    C = exact_c(torch, A, B)
    assert np.array_equal(C, oracle_fast.matmul(A, B))
    got, _ = check_proof(torch, ctx, oracle_fast, A, B, C)
    assert (got.mu, got.delta, got.nu) == (9, 12, 12)


@pytest.mark.timeout(600)
def test_config3_ffn_up_projection(torch, ctx, oracle_fast):
    A, B = workloads.ffn_up()
    C = exact_c(torch, A, B)
    freivalds(A, B, C)
    got, _ = check_proof(torch, ctx, oracle_fast, A, B, C)
    assert (got.mu, got.delta, got.nu) == (11, 12, 14)
    # a one-entry perturbation of C is rejected by the verifier (digest, and opening if re-committed)
    Cb = C.copy()
    Cb[1234, 5678] += 1
    com = imm.imm_commit_matmul(A, B, C, 2048, 4096, 14336)
    assert imm.imm_verify(com, ref.FS_INIT, got, None, None, Cb)[0] == 6
    comb = imm.imm_commit_matmul(None, None, Cb, 2048, 4096, 14336, out=com)
    bad, _ = ctx.imm_sumcheck_matmul_prove(dev(torch, A), dev(torch, B), comb, ref.FS_INIT)
    assert imm.imm_verify(comb, ref.FS_INIT, bad)[0] == imm.IMM_REJ_UNOPENED
    assert imm.imm_verify(comb, ref.FS_INIT, bad, None, None, Cb)[0] == 5


@pytest.mark.timeout(900)
def test_config4_moe_expert_batch(torch, ctx, oracle_fast):
    X, routes = workloads.moe_activations()
    assert sum(len(r) for r in routes) == 2 * 4096
    items, oracle_items, keep = [], [], []
    for e in range(8):
        A = np.ascontiguousarray(X[routes[e]])
        B = workloads.moe_expert_weight(e)
        C = exact_c(torch, A, B)
        com = imm.imm_commit_matmul(A, B, C, A.shape[0], 4096, 14336)
        oracle_items.append((A, B, C, com.digests()))
        items.append((dev(torch, A), dev(torch, B), com))
    want, want_states = oracle_fast.prove_chain(oracle_items, chained=False)
    got, states, final = ctx.imm_sumcheck_matmul_prove_batch(items, False, ref.FS_INIT)
    for e in range(8):
        assert got[e].words() == ref.proof_words(want[e]) and states[e] == want_states[e]
        assert got[e].mu == ref.ceil_log2(len(routes[e]))
    assert final == want_states[-1]
    assert {int(p.mu) for p in got} <= {10, 11}
    # the same eight proofs in the other execution modes: narrow-read reductions, the transcript hashed
    # by the round kernel, weights widened beforehand
    for mode, got_m, states_m, final_m in other_modes(ctx, items, False, ref.FS_INIT):
        assert [p.words() for p in got_m] == [ref.proof_words(p) for p in want], mode
        assert states_m == want_states and final_m == want_states[-1], mode


def other_modes(ctx, items, chained, state):
    """Runs a batch in the execution modes beside the default one (widened tables, host transcript);
    yields (mode, proofs, states, final state) for each."""
    try:
        ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 0)
        yield ("narrow-read",) + tuple(ctx.imm_sumcheck_matmul_prove_batch(items, chained, state))
        ctx.imm_ctx_set_option(imm.IMM_OPT_TRANSCRIPT, imm.IMM_TRANSCRIPT_DEVICE)
        yield ("narrow-read, device transcript",) + tuple(ctx.imm_sumcheck_matmul_prove_batch(items, chained, state))
        ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)
        yield ("widened, device transcript",) + tuple(ctx.imm_sumcheck_matmul_prove_batch(items, chained, state))
        ctx.imm_ctx_set_option(imm.IMM_OPT_TRANSCRIPT, imm.IMM_TRANSCRIPT_HOST)
        pre = [(A, ctx.imm_encode(B), com) for (A, B, com) in items]
        yield ("weights pre-encoded",) + tuple(ctx.imm_sumcheck_matmul_prove_batch(pre, chained, state))
        ctx.imm_ctx_set_option(imm.IMM_OPT_TRANSCRIPT, imm.IMM_TRANSCRIPT_DEVICE)
        yield ("weights pre-encoded, device transcript",) + tuple(ctx.imm_sumcheck_matmul_prove_batch(pre, chained, state))
        ctx.imm_ctx_set_option(imm.IMM_OPT_TRANSCRIPT, imm.IMM_TRANSCRIPT_HOST)
        ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, 0)
        yield ("weights pre-encoded, every round on the device",) + tuple(ctx.imm_sumcheck_matmul_prove_batch(pre, chained, state))
        del pre
    finally:
        ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)
        ctx.imm_ctx_set_option(imm.IMM_OPT_TRANSCRIPT, imm.IMM_TRANSCRIPT_HOST)
        ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, imm.IMM_HOST_TAIL_DEFAULT)


@pytest.mark.timeout(1200)
def test_config5_dense_layers_chained(torch, ctx, oracle_fast):
    """Chained transcript over the 7 statements of each decoder layer.  IMM_TEST_LAYERS picks how many
    of the 32 layers run (default: all 32, 224 proofs); the chain is proven layer by layer, resuming from the stored
    state, which is also the checkpoint/resume property of the transcript."""
    layers = int(os.environ.get("IMM_TEST_LAYERS", "32"))
    s_gpu = s_cpu = ref.FS_INIT
    total = 0
    for layer in range(layers):
        items, oracle_items = [], []
        for name, A, B in workloads.dense_layer(layer):
            C = exact_c(torch, A, B)
            com = imm.imm_commit_matmul(A, B, C, A.shape[0], A.shape[1], B.shape[1])
            oracle_items.append((A, B, C, com.digests()))
            items.append((dev(torch, A), dev(torch, B), com))
        want, want_states = oracle_fast.prove_chain(oracle_items, chained=True, state_in=s_cpu)
        if layer in (0, layers - 1):
            # first and last layer also in the other execution modes (W_down has d = 14336: its tables
            # of 2^14 entries enter the round loop through the hand-over from global memory to LDS)
            for mode, got_m, states_m, final_m in other_modes(ctx, items, True, s_gpu):
                assert [p.words() for p in got_m] == [ref.proof_words(p) for p in want], (layer, mode)
                assert states_m == want_states and final_m == want_states[-1], (layer, mode)
        got, states, s_gpu = ctx.imm_sumcheck_matmul_prove_batch(items, True, s_gpu)
        s_cpu = want_states[-1]
        for t in range(7):
            assert got[t].words() == ref.proof_words(want[t]), (layer, t)
            assert states[t] == want_states[t]
        assert s_gpu == s_cpu
        total += 7
        print("layer", layer, "ok", flush=True)
    assert total == 7 * layers


def test_batch_chained_and_independent_small(torch, ctx, oracle_fast):
    rng = np.random.default_rng(99)
    shapes = [(5, 33, 12), (1, 64, 300), (9, 7, 2), (16, 128, 64), (3, 1, 4), (2, 2, 2)]
    items, oracle_items = [], []
    for (m, d, n) in shapes:
        A = rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
        B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
        C = oracle_fast.matmul(A, B)
        com = imm.imm_commit_matmul(A, B, C, m, d, n)
        oracle_items.append((A, B, C, com.digests()))
        items.append((dev(torch, A), dev(torch, B), com))
    for chained in (True, False):
        want, want_states = oracle_fast.prove_chain(oracle_items, chained=chained)
        got, states, final = ctx.imm_sumcheck_matmul_prove_batch(items, chained, ref.FS_INIT)
        assert [p.words() for p in got] == [ref.proof_words(p) for p in want]
        assert states == want_states and final == want_states[-1]
    # split chain == unsplit chain
    want, want_states = oracle_fast.prove_chain(oracle_items, chained=True)
    g1, st1, f1 = ctx.imm_sumcheck_matmul_prove_batch(items[:2], True, ref.FS_INIT)
    g2, st2, f2 = ctx.imm_sumcheck_matmul_prove_batch(items[2:], True, f1)
    assert [p.words() for p in g1 + g2] == [ref.proof_words(p) for p in want] and f2 == want_states[-1]
    # empty batch leaves the state alone
    g0, st0, f0 = ctx.imm_sumcheck_matmul_prove_batch([], True, ref.FS_INIT)
    assert g0 == [] and f0 == ref.FS_INIT


def test_independent_batch_larger_than_one_group(torch, ctx, oracle_fast):
    """More independent proofs than one launch of the round kernel takes, with mixed round counts."""
    rng = np.random.default_rng(123)
    items, oracle_items = [], []
    for t in range(19):
        m, d, n = 1 + t % 5, [16, 3, 64, 1, 200][t % 5], 16 * (1 + t % 3)
        A = rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
        B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
        C = oracle_fast.matmul(A, B)
        com = imm.imm_commit_matmul(A, B, C, m, d, n)
        oracle_items.append((A, B, C, com.digests()))
        items.append((dev(torch, A), dev(torch, B), com))
    want, want_states = oracle_fast.prove_chain(oracle_items, chained=False)
    for widen in (1, 0):
        ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, widen)
        got, states, final = ctx.imm_sumcheck_matmul_prove_batch(items, False, ref.FS_INIT)
        assert [p.words() for p in got] == [ref.proof_words(p) for p in want]
        assert states == want_states and final == want_states[-1]
    ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)


def test_batches_where_the_host_finishes_some_round_loops_and_not_others(torch, ctx, oracle_fast):
    """Independent and chained proofs with 12, 10, 5 and 0 rounds in one batch: for each setting of the
    table length from which the host finishes the rounds, some proofs are split and some are not (the
    length is lowered for proofs that share a launch, and a proof needs two rounds beyond it)."""
    rng = np.random.default_rng(321)
    items, oracle_items = [], []
    for (m, d, n) in ((3, 4096, 5), (2, 600, 9), (4, 20, 3), (2, 1, 2), (5, 2048, 4)):
        A = rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
        B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
        C = oracle_fast.matmul(A, B)
        com = imm.imm_commit_matmul(A, B, C, m, d, n)
        oracle_items.append((A, B, C, com.digests()))
        items.append((dev(torch, A), dev(torch, B), com))
    try:
        for chained in (False, True):
            want, want_states = oracle_fast.prove_chain(oracle_items, chained=chained)
            for t in (0, 2, 5, imm.IMM_HOST_TAIL_DEFAULT, imm.IMM_HOST_TAIL_MAX):
                ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, t)
                got, states, final = ctx.imm_sumcheck_matmul_prove_batch(items, chained, ref.FS_INIT)
                assert [p.words() for p in got] == [ref.proof_words(p) for p in want], (chained, t)
                assert states == want_states and final == want_states[-1], (chained, t)
    finally:
        ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, imm.IMM_HOST_TAIL_DEFAULT)


def test_proofs_are_deterministic_and_survive_other_streams(torch, ctx, oracle_fast):
    A, B = workloads.tiny()
    C = oracle_fast.matmul(A, B)
    com = imm.imm_commit_matmul(A, B, C, 64, 64, 64)
    Ad, Bd = dev(torch, A), dev(torch, B)
    first, s_first = ctx.imm_sumcheck_matmul_prove(Ad, Bd, com, ref.FS_INIT)
    side = torch.cuda.Stream()
    for _ in range(100):
        p, s = ctx.imm_sumcheck_matmul_prove(Ad, Bd, com, ref.FS_INIT)
        assert p.words() == first.words() and s == s_first
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        p, s = ctx.imm_sumcheck_matmul_prove(Ad, Bd, com, ref.FS_INIT, stream=side)
    side.synchronize()
    assert p.words() == first.words() and s == s_first
    # the same bytes from every launch geometry: the grids and the way partial results are summed
    # change with the execution mode (one launch or several, partial vectors summed by a launch of
    # their own, in another kernel's launch, or by the last workgroup), the arithmetic must not
    rng = np.random.default_rng(31)
    A2 = rng.integers(-2**15, 2**15, size=(300, 2048), dtype=np.int16)
    B2 = rng.integers(-128, 128, size=(2048, 1040), dtype=np.int8)
    com2 = imm.imm_commit_matmul(A2, B2, oracle_fast.matmul(A2, B2), 300, 2048, 1040)
    A2d, B2d = dev(torch, A2), dev(torch, B2)
    base, s_base = ctx.imm_sumcheck_matmul_prove(A2d, B2d, com2, ref.FS_INIT)
    try:
        for widen in (1, 0):
            for fused in (1, 0):
                ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, widen)
                ctx.imm_ctx_set_option(imm.IMM_OPT_FUSE_REDUCTIONS, fused)
                for _ in range(25):
                    p, s = ctx.imm_sumcheck_matmul_prove(A2d, B2d, com2, ref.FS_INIT)
                    assert p.words() == base.words() and s == s_base, (widen, fused)
    finally:
        ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)
        ctx.imm_ctx_set_option(imm.IMM_OPT_FUSE_REDUCTIONS, 1)


def test_host_transcript_bounded_waits(torch, oracle_fast):
    """The round kernel's wait for a challenge is bounded.  With a spin limit of zero it gives up at
    once, every wave leaves the kernel, the call reports an error after the host's own (shortened)
    patience, and the context keeps working afterwards."""
    A, B = workloads.tiny()
    C = oracle_fast.matmul(A, B)
    com = imm.imm_commit_matmul(A, B, C, 64, 64, 64)
    Ad, Bd = dev(torch, A), dev(torch, B)
    c = imm.Context(0)
    want, s_want = c.imm_sumcheck_matmul_prove(Ad, Bd, com, ref.FS_INIT)
    c.imm_ctx_set_option(imm.IMM_OPT_TRANSCRIPT, imm.IMM_TRANSCRIPT_HOST)
    c.imm_ctx_set_option(imm.IMM_OPT_SPIN_LIMIT, 0)
    c.imm_ctx_set_option(imm.IMM_OPT_HOST_WAIT_MS, 50)
    with pytest.raises(imm.ImmError) as e:
        c.imm_sumcheck_matmul_prove(Ad, Bd, com, ref.FS_INIT)
    assert e.value.code == -5 and "mailbox" in str(e.value)
    torch.cuda.synchronize()
    c.imm_ctx_set_option(imm.IMM_OPT_SPIN_LIMIT, 1 << 21)
    c.imm_ctx_set_option(imm.IMM_OPT_HOST_WAIT_MS, 30000)
    got, s_got = c.imm_sumcheck_matmul_prove(Ad, Bd, com, ref.FS_INIT)
    assert got.words() == want.words() and s_got == s_want
    c.close()


def test_chain_with_the_next_proof_queued_ahead_or_not(torch, oracle_fast):
    """In a chained batch the kernels of proof p + 1 are queued while the host still serves proof p's
    round loop, its eq kernel waiting on the device for the points.  Same proofs and states with that
    switched off, in every execution mode, for a chain that mixes statements the round kernel takes
    with ones it does not (a single shared index; tables longer than one workgroup's limit), buffers
    that have to grow while kernels are queued, and after a failure with kernels queued behind it."""
    rng = np.random.default_rng(515)
    shapes = [(4, 64, 8), (3, 700, 5), (2, 1, 3), (5, 4096, 16), (2, 65539, 3), (6, 33, 40), (3, 2048, 64), (4, 8, 4)]
    items, oracle_items = [], []
    for (m, d, n) in shapes:
        A = rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
        B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
        C = oracle_fast.matmul(A, B)
        com = imm.imm_commit_matmul(A, B, C, m, d, n)
        oracle_items.append((A, B, C, com.digests()))
        items.append((dev(torch, A), dev(torch, B), com))
    want, want_states = oracle_fast.prove_chain(oracle_items, chained=True)
    want_words = [ref.proof_words(p) for p in want]
    c = imm.Context(0)   # a fresh context: its buffers grow as the chain goes
    for ahead in (1, 0):
        c.imm_ctx_set_option(imm.IMM_OPT_QUEUE_AHEAD, ahead)
        for widen in (1, 0):
            c.imm_ctx_set_option(imm.IMM_OPT_WIDEN, widen)
            for tail in (imm.IMM_HOST_TAIL_DEFAULT, 0):
                c.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, tail)
                for _ in range(2):
                    got, states, final = c.imm_sumcheck_matmul_prove_batch(items, True, ref.FS_INIT)
                    assert [p.words() for p in got] == want_words, (ahead, widen, tail)
                    assert states == want_states and final == want_states[-1], (ahead, widen, tail)
    c.imm_ctx_set_option(imm.IMM_OPT_QUEUE_AHEAD, 1)
    c.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)
    c.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, imm.IMM_HOST_TAIL_DEFAULT)
    pre = [(A, c.imm_encode(B), com) for (A, B, com) in items]
    got, states, final = c.imm_sumcheck_matmul_prove_batch(pre, True, ref.FS_INIT)
    assert [p.words() for p in got] == want_words and final == want_states[-1]
    # challenges and points through pinned host memory instead of host-written device memory
    c.imm_ctx_set_option(imm.IMM_OPT_REPLY_IN_DEVICE_MEMORY, 0)
    for widen in (1, 0):
        c.imm_ctx_set_option(imm.IMM_OPT_WIDEN, widen)
        got, states, final = c.imm_sumcheck_matmul_prove_batch(items, True, ref.FS_INIT)
        assert [p.words() for p in got] == want_words and states == want_states, widen
    c.imm_ctx_set_option(imm.IMM_OPT_REPLY_IN_DEVICE_MEMORY, 1)
    c.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)
    # a wait that runs out with the next proof's kernels queued: error, everything drains, and the context works on
    c.imm_ctx_set_option(imm.IMM_OPT_SPIN_LIMIT, 0)
    c.imm_ctx_set_option(imm.IMM_OPT_HOST_WAIT_MS, 50)
    with pytest.raises(imm.ImmError) as e:
        c.imm_sumcheck_matmul_prove_batch(items, True, ref.FS_INIT)
    assert e.value.code == -5
    torch.cuda.synchronize()
    c.imm_ctx_set_option(imm.IMM_OPT_SPIN_LIMIT, 1 << 21)
    c.imm_ctx_set_option(imm.IMM_OPT_HOST_WAIT_MS, 30000)
    got, states, final = c.imm_sumcheck_matmul_prove_batch(items, True, ref.FS_INIT)
    assert [p.words() for p in got] == want_words and states == want_states
    c.close()


def test_operands_of_the_next_proof_widened_ahead_or_not(torch, oracle_fast):
    """In a sequence of proofs the next proof's raw operands are widened on a second stream while the
    current proof's rounds run.  Same proofs and states with that switched off; with operands that
    repeat (the activations shared by consecutive statements), that are pre-encoded, or that change
    size from one proof to the next; and after a call that failed with tables queued that nobody takes."""
    rng = np.random.default_rng(2024)
    c = imm.Context(0)
    shapes = [(40, 300, 64), (40, 300, 17), (40, 300, 64), (3, 5000, 129), (64, 64, 2048), (1, 2, 3), (9, 1, 4)]
    A_shared = rng.integers(-2**15, 2**15, size=(40, 300), dtype=np.int16)
    items, oracle_items = [], []
    for t, (m, d, n) in enumerate(shapes):
        A = A_shared if (m, d) == (40, 300) else rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
        B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
        C = oracle_fast.matmul(A, B)
        com = imm.imm_commit_matmul(A, B, C, m, d, n)
        oracle_items.append((A, B, C, com.digests()))
        items.append([dev(torch, A), dev(torch, B), com])
    shared = items[0][0]
    for it in items[1:3]:
        it[0] = shared                                   # the same device buffer, not a copy
    items[4][1] = c.imm_encode(items[4][1])              # one weight table comes pre-encoded
    items = [tuple(it) for it in items]
    want, want_states = oracle_fast.prove_chain(oracle_items, chained=True)
    try:
        for ahead in (1, 0, 1):
            c.imm_ctx_set_option(imm.IMM_OPT_ENCODE_AHEAD, ahead)
            got, states, final = c.imm_sumcheck_matmul_prove_batch(items, True, ref.FS_INIT)
            assert [p.words() for p in got] == [ref.proof_words(p) for p in want], ahead
            assert states == want_states and final == want_states[-1]
        # profiling sees the encode launches wherever they ran: 6 of A and 5 of B ahead of time, and the
        # first proof's own, which shares a launch booked under B
        c.imm_ctx_reset_profiling()
        c.imm_ctx_set_profiling((1 << imm.IMM_K_COUNT) - 1)
        c.imm_sumcheck_matmul_prove_batch(items, True, ref.FS_INIT)
        c.imm_ctx_set_profiling(0)
        assert c.imm_ctx_kernel_time(imm.IMM_K_ENCODE_A)[0] == 6 and c.imm_ctx_kernel_time(imm.IMM_K_ENCODE_B)[0] == 6
        # a sequence that stops at its first proof (the round kernel gives up at once) leaves the second
        # proof's tables queued; the next calls, for those operands or for others, are not disturbed
        c.imm_ctx_set_option(imm.IMM_OPT_SPIN_LIMIT, 0)
        c.imm_ctx_set_option(imm.IMM_OPT_HOST_WAIT_MS, 50)
        with pytest.raises(imm.ImmError):
            c.imm_sumcheck_matmul_prove_batch(items[3:5], True, ref.FS_INIT)
        torch.cuda.synchronize()
        c.imm_ctx_set_option(imm.IMM_OPT_SPIN_LIMIT, 1 << 21)
        c.imm_ctx_set_option(imm.IMM_OPT_HOST_WAIT_MS, 30000)
        got, s_got = c.imm_sumcheck_matmul_prove(items[0][0], items[0][1], items[0][2], ref.FS_INIT)
        assert got.words() == ref.proof_words(want[0]) and s_got == want_states[0]
        c.imm_ctx_set_option(imm.IMM_OPT_SPIN_LIMIT, 0)
        c.imm_ctx_set_option(imm.IMM_OPT_HOST_WAIT_MS, 50)
        with pytest.raises(imm.ImmError):
            c.imm_sumcheck_matmul_prove_batch(items[0:2], True, ref.FS_INIT)
        torch.cuda.synchronize()
        c.imm_ctx_set_option(imm.IMM_OPT_SPIN_LIMIT, 1 << 21)
        c.imm_ctx_set_option(imm.IMM_OPT_HOST_WAIT_MS, 30000)
        got, states, final = c.imm_sumcheck_matmul_prove_batch(items[1:], True, want_states[0])
        assert [p.words() for p in got] == [ref.proof_words(p) for p in want[1:]] and final == want_states[-1]
    finally:
        c.close()


def test_argument_errors(torch, ctx):
    L = imm.load()
    A = torch.zeros((2, 2), dtype=torch.int16, device="cuda")
    B = torch.zeros((2, 2), dtype=torch.int8, device="cuda")
    com = imm.Commit()
    st = (ctypes.c_uint8 * 32)()
    pr = imm.Proof()
    h = ctx._h
    f = L.imm_sumcheck_matmul_prove
    assert f(None, None, A.data_ptr(), 2, B.data_ptr(), 1, 2, 2, 2, ctypes.byref(com), st, ctypes.byref(pr)) == -1
    assert f(h, None, None, 2, B.data_ptr(), 1, 2, 2, 2, ctypes.byref(com), st, ctypes.byref(pr)) == -1
    assert f(h, None, A.data_ptr(), 2, B.data_ptr(), 1, 0, 2, 2, ctypes.byref(com), st, ctypes.byref(pr)) == -2
    assert f(h, None, A.data_ptr(), 2, B.data_ptr(), 1, 2, 2, (1 << 32) + 1, ctypes.byref(com), st,
             ctypes.byref(pr)) == -2
    assert f(h, None, A.data_ptr(), 1, B.data_ptr(), 1, 2, 2, 2, ctypes.byref(com), st, ctypes.byref(pr)) == -3
    assert f(h, None, A.data_ptr(), 2, B.data_ptr(), 2, 2, 2, 2, ctypes.byref(com), st, ctypes.byref(pr)) == -3
    # commitments that are not those of the statement: other shapes, or not int16 x int8 -> int64
    zero = np.zeros((2, 2))
    good = imm.imm_commit_matmul(zero.astype(np.int16), zero.astype(np.int8), zero.astype(np.int64), 2, 2, 2)
    assert f(h, None, A.data_ptr(), 2, B.data_ptr(), 1, 2, 2, 2, ctypes.byref(com), st, ctypes.byref(pr)) == -2
    assert f(h, None, A.data_ptr(), 2, B.data_ptr(), 1, 2, 2, 1, ctypes.byref(good), st, ctypes.byref(pr)) == -2
    good.C.dtype = imm.IMM_I16
    assert f(h, None, A.data_ptr(), 2, B.data_ptr(), 1, 2, 2, 2, ctypes.byref(good), st, ctypes.byref(pr)) == -3
    good.C.dtype = imm.IMM_I64
    assert f(h, None, A.data_ptr(), 2, B.data_ptr(), 1, 2, 2, 2, ctypes.byref(good), st, ctypes.byref(pr)) == 0
    out = ctypes.c_uint64(0)
    assert L.imm_mle_eval(h, None, A.data_ptr(), 2, 2, 2, 1, None, None, ctypes.byref(out)) == -2   # ld < cols
    assert L.imm_mle_eval(h, None, A.data_ptr(), 9, 2, 2, 2, None, None, ctypes.byref(out)) == -3
    assert L.imm_mle_eval(h, None, A.data_ptr(), 2, 2, 2, 2, None, None, ctypes.byref(out)) == -1   # points missing
    bad_pt = (ctypes.c_uint64 * 1)(P)
    assert L.imm_mle_eval(h, None, A.data_ptr(), 2, 2, 2, 2, bad_pt, bad_pt, ctypes.byref(out)) == -2
    g = (ctypes.c_uint64 * 3)()
    assert L.imm_round_fold_eval(h, None, A.data_ptr(), B.data_ptr(), 3, None, g) == -2
    assert L.imm_encode(h, None, A.data_ptr(), 4, 4, A.data_ptr()) == -3
    assert L.imm_ctx_set_option(h, imm.IMM_OPT_HOST_TAIL, imm.IMM_HOST_TAIL_MAX + 1) == -2
    assert L.imm_ctx_set_option(h, imm.IMM_OPT_HOST_TAIL, -1) == -2
    assert L.imm_ctx_set_option(h, imm.IMM_OPT_HOST_TAIL, imm.IMM_HOST_TAIL_DEFAULT) == 0
    bad = ctypes.c_void_p()
    assert L.imm_ctx_create(ctypes.byref(bad), 99, 0) == -5
    assert b"device" in L.imm_last_error()
    cnt = ctypes.c_uint64(0)
    fresh = imm.Context(0)
    assert L.imm_debug_fetch(fresh._h, 0, None, 0, ctypes.byref(cnt)) == -6
    fresh.close()


def test_profiling_counts_launches(torch, ctx, oracle_fast):
    A, B = workloads.tiny()
    com = imm.imm_commit_matmul(A, B, oracle_fast.matmul(A, B), 64, 64, 64)
    Ad, Bd = dev(torch, A), dev(torch, B)
    try:
        for widen, fused in ((1, 1), (1, 0), (0, 1), (0, 0)):
            ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, widen)
            ctx.imm_ctx_set_option(imm.IMM_OPT_FUSE_REDUCTIONS, fused)
            ctx.imm_ctx_reset_profiling()
            ctx.imm_ctx_set_profiling((1 << imm.IMM_K_COUNT) - 1)
            for _ in range(3):
                ctx.imm_sumcheck_matmul_prove(Ad, Bd, com, ref.FS_INIT)
            ctx.imm_ctx_set_profiling(0)
            counts = {imm.KERNEL_NAMES[k]: ctx.imm_ctx_kernel_time(k) for k in range(imm.IMM_K_COUNT)}
            # widened with shared launches: the widening of both operands and the eq vectors are one launch,
            # booked under encode_B
            assert counts["encode_A"][0] == (3 if widen and not fused else 0)
            assert counts["encode_B"][0] == (3 if widen else 0)
            assert counts["eq_build"][0] == (0 if widen and fused else 3)
            # in narrow-read mode one launch covers both reductions and the sum of A's partial vectors,
            # unless that is switched off
            assert counts["reduce_A"][0] == (0 if (fused and not widen) else 3) and counts["reduce_B"][0] == 3
            assert counts["combine"][0] == (0 if fused else counts["combine"][0]) and counts["combine"][0] <= 6
            assert counts["round"][0] == 3       # all rounds of a proof run in one launch
            assert all(ms > 0 for (n, ms) in counts.values() if n)
    finally:
        ctx.imm_ctx_set_option(imm.IMM_OPT_FUSE_REDUCTIONS, 1)
        ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)
    ctx.imm_ctx_reset_profiling()
    assert ctx.imm_ctx_kernel_time(imm.IMM_K_ROUND) == (0, 0.0)


def test_reductions_in_one_launch_or_two(torch, ctx, oracle_fast):
    """Same proofs whether the partial evaluations of A and B share a launch or not, in the three
    operand forms the shared launch covers and in one it does not (odd row length)."""
    rng = np.random.default_rng(123)
    for (m, d, n) in ((70, 300, 96), (33, 128, 4096), (5, 67, 31)):
        A = rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
        B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
        C = oracle_fast.matmul(A, B)
        com = imm.imm_commit_matmul(A, B, C, m, d, n)
        want, s_want = oracle_fast.prove(A, B, C, com.digests())
        Ad, Bd = dev(torch, A), dev(torch, B)
        Be = ctx.imm_encode(Bd)
        try:
            for fused in (1, 0):
                ctx.imm_ctx_set_option(imm.IMM_OPT_FUSE_REDUCTIONS, fused)
                for widen, Bx in ((1, Bd), (0, Bd), (1, Be)):
                    ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, widen)
                    got, s_got = ctx.imm_sumcheck_matmul_prove(Ad, Bx, com, imm.imm_fs_init())
                    assert got.words() == ref.proof_words(want) and s_got == s_want, (m, d, n, fused, widen)
        finally:
            ctx.imm_ctx_set_option(imm.IMM_OPT_FUSE_REDUCTIONS, 1)
            ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)


def test_challenges_through_the_mailbox_or_through_device_memory(torch, ctx, oracle_fast):
    """The host hands r_k to the round kernel either in device memory (default where the device memory
    is mapped into the host's address space) or in the pinned mailbox; the proofs are the same."""
    rng = np.random.default_rng(77)
    A = rng.integers(-2**15, 2**15, size=(37, 300), dtype=np.int16)
    B = rng.integers(-128, 128, size=(300, 41), dtype=np.int8)
    C = oracle_fast.matmul(A, B)
    com = imm.imm_commit_matmul(A, B, C, 37, 300, 41)
    want, s_want = oracle_fast.prove(A, B, C, com.digests())
    Ad, Bd = dev(torch, A), dev(torch, B)
    try:
        for mode in (0, 1, 0, 1):
            ctx.imm_ctx_set_option(imm.IMM_OPT_REPLY_IN_DEVICE_MEMORY, mode)
            got, s_got = ctx.imm_sumcheck_matmul_prove(Ad, Bd, com, imm.imm_fs_init())
            assert got.words() == ref.proof_words(want) and s_got == s_want
    finally:
        ctx.imm_ctx_set_option(imm.IMM_OPT_REPLY_IN_DEVICE_MEMORY, 1)


def test_device_challenge_takes_the_rejection_branch_like_the_oracle(torch, ctx):
    """The challenge derivation that lane 0 of the round kernel runs when the device hashes the
    transcript, on the stored state whose first candidate is not canonical, and on ordinary states."""
    from tests.test_library_cpu import rejecting_state
    state, first, want, after = rejecting_state()
    assert first >= P
    assert ctx.imm_debug_device_challenge(state) == (want, after)
    s_dev, tr = ref.FS_INIT, ref.Transcript(ref.FS_INIT)
    for _ in range(5):
        v, s_dev = ctx.imm_debug_device_challenge(s_dev)
        assert v == tr.challenge() and s_dev == tr.s
