"""imm_mle_eval_static, the entry point that allocates nothing, against imm_mle_eval (and the oracle)
through the C ABI: calls in a row on the same device share one static array, a larger table first,
smaller ones after it, so that anything a call wrongly took over from the one before would show."""
import ctypes
import random

import numpy as np
import pytest

from oracle import reference as ref
from paper_2602_22700_amd import binding as imm

pytestmark = pytest.mark.gpu
P = ref.P


@pytest.fixture(scope="module")
def torch():
    import torch as t
    if not t.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    return t


def table_and_points(shape, dt, seed):
    rows, cols = shape
    rng = np.random.default_rng(seed)
    rnd = random.Random(seed)
    if dt == np.uint64:
        T = rng.integers(0, P, size=shape, dtype=np.uint64)
        T.reshape(-1)[0] = P - 1
    else:
        info = np.iinfo(dt)
        T = rng.integers(info.min, info.max, size=shape, dtype=dt, endpoint=True)
    pr = [rnd.randrange(P) for _ in range(ref.ceil_log2(rows))]
    pc = [rnd.randrange(P) for _ in range(ref.ceil_log2(cols))]
    return T, pr, pc


def to_dev(torch, T):
    if T.dtype == np.uint64:
        return torch.from_numpy(T.view(np.int64)).cuda().view(torch.uint64)
    return torch.from_numpy(T).cuda()


def test_static_entry_point_matches_the_allocating_one(torch, oracle_fast):
    """Two calls in a row, the second on a smaller table, then more shapes that take the other
    reduction order and several column splits; every value against imm_mle_eval and the oracle."""
    out = torch.full((4,), 0x5555, dtype=torch.int64, device="cuda").view(torch.uint64)
    # in a fresh process this first call finds the static array's address itself; after other tests a
    # context has already looked it up
    T, pr, pc = table_and_points((9, 300), np.int16, 1000)
    imm.imm_mle_eval_static(to_dev(torch, T), pr, pc, out)
    torch.cuda.synchronize()
    assert int(out.view(torch.int64)[0].item()) & (2**64 - 1) == oracle_fast.mle_matrix(T, pr, pc)
    ctx = imm.Context(0)
    try:
        cases = [((700, 9000), np.int64), ((37, 515), np.int64),            # larger, then smaller
                 ((2048, 14336), np.int64),                                  # the product matrix of the FFN shape
                 ((300, 130), np.int16), ((5, 6), np.int8), ((1, 1), np.int64),
                 ((64, 20000), np.int8), ((4100, 64), np.uint64), ((3, 1025), np.uint64), ((1, 7), np.int16)]
        for seed, (shape, dt) in enumerate(cases):
            T, pr, pc = table_and_points(shape, dt, seed)
            Td = to_dev(torch, T)
            imm.imm_mle_eval_static(Td, pr, pc, out)
            torch.cuda.synchronize()
            got = int(out.view(torch.int64)[0].item()) & (2**64 - 1)
            assert got == ctx.imm_mle_eval(Td, pr, pc), (shape, dt)
            assert got == oracle_fast.mle_matrix(T, pr, pc), (shape, dt)
            assert int(out.view(torch.int64)[1].item()) == 0x5555      # one word is written, no more
        # a window of a larger table: leading dimension beyond the column count, odd start
        full, _, _ = table_and_points((40, 700), np.int8, 77)
        fd = to_dev(torch, full)
        T = np.ascontiguousarray(full[3:36, 1:516])
        _, pr, pc = table_and_points(T.shape, np.int8, 78)
        imm.imm_mle_eval_static(fd[3:, 1:], pr, pc, out, rows=33, cols=515, ld=700)
        torch.cuda.synchronize()
        assert int(out.view(torch.int64)[0].item()) & (2**64 - 1) == oracle_fast.mle_matrix(T, pr, pc)
    finally:
        ctx.close()


def test_static_entry_point_refuses_what_does_not_fit(torch):
    L = imm.load()
    t = torch.zeros(16, dtype=torch.int8, device="cuda")
    out = torch.zeros(1, dtype=torch.int64, device="cuda")
    pts = (ctypes.c_uint64 * 32)(*([3] * 32))
    f = L.imm_mle_eval_static
    # eq vector of 2^21 entries alone is 16 MiB: beyond the static array, refused before any launch
    assert f(None, t.data_ptr(), imm.IMM_I8, 1, 1 << 21, 1 << 21, None, pts, out.data_ptr()) == imm.IMM_E_SHAPE
    assert b"static" in L.imm_last_error()
    assert f(None, None, imm.IMM_I8, 4, 4, 4, pts, pts, out.data_ptr()) == imm.IMM_E_NULL
    assert f(None, t.data_ptr(), imm.IMM_I8, 4, 4, 4, pts, pts, None) == imm.IMM_E_NULL
    assert f(None, t.data_ptr(), imm.IMM_I8, 4, 4, 3, pts, pts, out.data_ptr()) == imm.IMM_E_SHAPE
    assert f(None, t.data_ptr(), 9, 4, 4, 4, pts, pts, out.data_ptr()) == imm.IMM_E_DTYPE
    assert f(None, t.data_ptr(), imm.IMM_I8, 4, 4, 4, None, pts, out.data_ptr()) == imm.IMM_E_NULL
    bad = (ctypes.c_uint64 * 2)(P, 0)
    assert f(None, t.data_ptr(), imm.IMM_I8, 4, 4, 4, bad, pts, out.data_ptr()) == imm.IMM_E_SHAPE
