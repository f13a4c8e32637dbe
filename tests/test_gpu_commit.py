"""GPU parity of the commitments hashed on the device: the digests must be the bytes the CPU oracle
computes for the same matrices (a hash: exact equality), whatever the number of leaves and the length
of the last one.  All calls go through the C ABI (ctypes binding)."""
import numpy as np
import pytest

from paper_2602_22700_amd import binding as imm

pytestmark = pytest.mark.gpu
MIB = 1 << 20


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


def statement(rng, m, d, n):
    A = rng.integers(-2**15, 2**15, size=(m, d), dtype=np.int16)
    B = rng.integers(-128, 128, size=(d, n), dtype=np.int8)
    C = rng.integers(-2**40, 2**40, size=(m, n), dtype=np.int64)   # any bytes: only hashed here
    return A, B, C


# byte lengths: 1 and 2 bytes, around one block (55, 56, 63, 64, 65 bytes), exactly one leaf, one byte
# more, several leaves with a ragged end
SHAPES = [(1, 1, 1), (1, 55, 1), (1, 28, 2), (1, 63, 1), (1, 32, 2), (5, 13, 1), (1, 64, 119), (8, 8, 8),
          (512, 1024, 1024), (512, 1024, 1025), (1, MIB + 1, 1), (700, 3000, 77), (33, 70000, 9)]


def test_device_commitments_match_the_oracle(torch, ctx, oracle_fast):
    rng = np.random.default_rng(2026)
    tables, want = [], []
    for (m, d, n) in SHAPES:
        A, B, C = statement(rng, m, d, n)
        want += list(oracle_fast.commit_matmul(A, B, C))
        tables += [torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), torch.from_numpy(C).cuda()]
    got = ctx.imm_commit_tables_device(tables)
    assert [bytes(c.digest) for c in got] == want
    for c, t in zip(got, tables):
        assert (c.rows, c.cols) == tuple(t.shape) and c.dtype == imm._tensor_dtype(t)
    # one table at a time, and the library's own host commitment
    for k in (0, 5, 26, 38):
        assert bytes(ctx.imm_commit_tables_device([tables[k]])[0].digest) == want[k]
    A, B, C = (t.cpu().numpy() for t in tables[27:30])
    assert imm.imm_commit_matmul(A, B, C, *A.shape, B.shape[1]).digests() == tuple(want[27:30])
    assert ctx.imm_commit_tables_device([]) == []


def test_device_commitments_over_many_workgroups(torch, ctx, oracle_fast):
    """More leaves than one workgroup hashes (64), of different lengths side by side in a wave."""
    rng = np.random.default_rng(11)
    arrays = [rng.integers(-2**62, 2**62, size=(2048, 6400), dtype=np.int64),      # 100 leaves
              rng.integers(-128, 128, size=(3, 5), dtype=np.int8),
              rng.integers(-2**15, 2**15, size=(1500, 1400), dtype=np.int16),       # 5 leaves, the last one short
              rng.integers(-128, 128, size=(40, MIB), dtype=np.int8),               # 40 whole leaves
              rng.integers(-2**62, 2**62, size=(9, 1), dtype=np.int64)]
    got = ctx.imm_commit_tables_device([torch.from_numpy(a).cuda() for a in arrays])
    assert [bytes(c.digest) for c in got] == [oracle_fast.commit_array(a) for a in arrays]


def test_device_commitments_of_tables_that_are_only_4_byte_aligned(torch, ctx, oracle_fast):
    rng = np.random.default_rng(7)
    A, B, C = statement(rng, 3, 700001, 2)
    flat = torch.zeros(B.size + 64, dtype=torch.int8, device="cuda")
    for off in (4, 8, 12, 16):
        flat[off:off + B.size] = torch.from_numpy(B.reshape(-1)).cuda()
        view = flat[off:off + B.size].view(B.shape)
        assert view.data_ptr() % 16 == off % 16
        got = ctx.imm_commit_tables_device([view])
        assert bytes(got[0].digest) == oracle_fast.commit_array(B)


def test_device_commitment_argument_errors(torch, ctx):
    t8 = torch.zeros((4, 64), dtype=torch.int8, device="cuda")
    with pytest.raises(imm.ImmError) as e:
        ctx.imm_commit_tables_device([t8.view(-1)[1:129].view(2, 64)])      # address not a multiple of 4
    assert e.value.code == imm.IMM_E_SHAPE
    with pytest.raises(imm.ImmError) as e:
        ctx.imm_commit_tables_device([torch.zeros((2, 2), dtype=torch.int64, device="cuda").view(torch.uint64)])
    assert e.value.code == imm.IMM_E_DTYPE
    lib = imm.load()
    out = (imm.Commit1 * 1)()
    assert lib.imm_commit_tables_device(ctx._h, None, 1, None, out) == imm.IMM_E_NULL
    assert lib.imm_commit_tables_device(ctx._h, None, -1, None, out) == imm.IMM_E_SHAPE
    d = (imm.TableDesc * 1)()
    d[0].table_dev, d[0].dtype, d[0].rows, d[0].cols = t8.data_ptr(), imm.IMM_I8, 0, 64
    assert lib.imm_commit_tables_device(ctx._h, None, 1, d, out) == imm.IMM_E_SHAPE


def test_device_commitment_is_profiled(torch, ctx):
    t = torch.zeros((3, MIB), dtype=torch.int8, device="cuda")
    ctx.imm_ctx_reset_profiling()
    ctx.imm_ctx_set_profiling(1 << imm.IMM_K_COMMIT)
    ctx.imm_commit_tables_device([t, t])
    ctx.imm_ctx_set_profiling(0)
    n, ms = ctx.imm_ctx_kernel_time(imm.IMM_K_COMMIT)
    assert n == 1 and ms > 0
    ctx.imm_ctx_reset_profiling()
