"""ctypes binding of libimm.so -- argument marshalling only.

Every function here has the name of the C entry point it forwards to
(include/imm.h).  Device buffers are torch tensors on the GPU (torch is used
for device memory and streams only); host buffers are numpy arrays or bytes.
There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libimm.so")

IMM_MAX_ROUNDS = 32
IMM_I8, IMM_I16, IMM_I64, IMM_F64P = 1, 2, 3, 4
IMM_OPT_DEBUG_SNAPSHOTS, IMM_OPT_WIDEN, IMM_OPT_TRANSCRIPT, IMM_OPT_SPIN_LIMIT, IMM_OPT_HOST_WAIT_MS = 1, 2, 3, 4, 5
IMM_OPT_REPLY_IN_DEVICE_MEMORY = 6
IMM_OPT_FUSE_REDUCTIONS = 7
IMM_OPT_ENCODE_AHEAD = 8
IMM_OPT_TIMELINE = 9
IMM_OPT_HOST_TAIL = 10
IMM_OPT_QUEUE_AHEAD = 11
IMM_HOST_TAIL_DEFAULT = 9
IMM_HOST_TAIL_MAX = 10
TIMELINE_NAMES = ["entry", "head_hashed", "front_launched", "reductions_launched", "rounds_launched", "first_message",
                  "first_challenge", "last_challenge", "final_values", "exit"]
IMM_TRANSCRIPT_DEVICE, IMM_TRANSCRIPT_HOST = 0, 1
(IMM_K_ENCODE_A, IMM_K_ENCODE_B, IMM_K_EQ, IMM_K_REDUCE_A, IMM_K_REDUCE_B, IMM_K_ROUND,
 IMM_K_COMBINE, IMM_K_LDD, IMM_K_TOPK, IMM_K_COMMIT, IMM_K_COUNT) = range(11)
IMM_TOPK_MAX = 64
IMM_OK, IMM_E_NULL, IMM_E_SHAPE, IMM_E_DTYPE, IMM_E_NOMEM, IMM_E_HIP, IMM_E_STATE = 0, -1, -2, -3, -4, -5, -6
IMM_REJ_UNOPENED = 8
KERNEL_NAMES = ["encode_A", "encode_B", "eq_build", "reduce_A", "reduce_B", "round", "combine", "ldd_tv_kl",
                "topk_distance", "commit_leaves"]

EXPORTS = [
    "imm_ctx_create", "imm_ctx_destroy", "imm_last_error", "imm_fs_init", "imm_commit_matmul", "imm_encode",
    "imm_mle_eval", "imm_sumcheck_matmul_prove", "imm_sumcheck_matmul_prove_batch", "imm_round_fold_eval",
    "imm_verify", "imm_debug_fetch", "imm_ctx_set_option", "imm_ctx_set_profiling", "imm_ctx_kernel_time",
    "imm_ctx_reset_profiling", "imm_ldd_tv_kl", "imm_topk_distance", "imm_tail_density",
    "imm_commit_tables_device", "imm_mle_eval_static", "imm_verify_points", "imm_transcript_challenge",
    "imm_debug_device_challenge", "imm_debug_timeline",
]


class ImmError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        super().__init__("%s failed with code %d%s" % (where, code, (": " + detail) if detail else ""))
        self.code = code


class Commit1(ctypes.Structure):
    _fields_ = [("digest", ctypes.c_uint8 * 32), ("rows", ctypes.c_uint64), ("cols", ctypes.c_uint64),
                ("dtype", ctypes.c_uint32), ("_pad", ctypes.c_uint32)]


class TableDesc(ctypes.Structure):
    _fields_ = [("table_dev", ctypes.c_void_p), ("dtype", ctypes.c_uint32), ("_pad", ctypes.c_uint32),
                ("rows", ctypes.c_uint64), ("cols", ctypes.c_uint64)]


class Commit(ctypes.Structure):
    _fields_ = [("A", Commit1), ("B", Commit1), ("C", Commit1)]

    def digests(self) -> Tuple[bytes, bytes, bytes]:
        return bytes(self.A.digest), bytes(self.B.digest), bytes(self.C.digest)


class Proof(ctypes.Structure):
    _fields_ = [("version", ctypes.c_uint32), ("mu", ctypes.c_uint32), ("delta", ctypes.c_uint32),
                ("nu", ctypes.c_uint32), ("c0", ctypes.c_uint64), ("vA", ctypes.c_uint64), ("vB", ctypes.c_uint64),
                ("g", ctypes.c_uint64 * (3 * IMM_MAX_ROUNDS))]

    def words(self) -> List[int]:
        """Flat word list: mu, delta, nu, c0, g_1(0..2) .. g_delta(0..2), vA, vB."""
        return ([int(self.mu), int(self.delta), int(self.nu), int(self.c0)]
                + [int(v) for v in self.g[:3 * self.delta]] + [int(self.vA), int(self.vB)])

    def copy(self) -> "Proof":
        out = Proof()
        ctypes.memmove(ctypes.byref(out), ctypes.byref(self), ctypes.sizeof(Proof))
        return out


class MatmulDesc(ctypes.Structure):
    _fields_ = [("A_dev", ctypes.c_void_p), ("B_dev", ctypes.c_void_p), ("dtA", ctypes.c_uint32),
                ("dtB", ctypes.c_uint32), ("m", ctypes.c_uint64), ("d", ctypes.c_uint64), ("n", ctypes.c_uint64),
                ("com", ctypes.POINTER(Commit))]


_lib = None


def load() -> ctypes.CDLL:
    """Load libimm.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libimm.so is not built: run `python -m paper_2602_22700_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    vp, u64, i32, u32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int, ctypes.c_uint32
    L.imm_ctx_create.argtypes = [ctypes.POINTER(vp), i32, ctypes.c_size_t]
    L.imm_ctx_destroy.argtypes = [vp]
    L.imm_last_error.restype = ctypes.c_char_p
    L.imm_fs_init.argtypes = [vp]
    L.imm_commit_matmul.argtypes = [vp, vp, vp, u64, u64, u64, ctypes.POINTER(Commit)]
    L.imm_encode.argtypes = [vp, vp, vp, i32, u64, vp]
    L.imm_mle_eval.argtypes = [vp, vp, vp, i32, u64, u64, u64, vp, vp, ctypes.POINTER(u64)]
    L.imm_sumcheck_matmul_prove.argtypes = [vp, vp, vp, i32, vp, i32, u64, u64, u64, ctypes.POINTER(Commit), vp,
                                            ctypes.POINTER(Proof)]
    L.imm_sumcheck_matmul_prove_batch.argtypes = [vp, vp, i32, ctypes.POINTER(MatmulDesc), i32, vp,
                                                  ctypes.POINTER(Proof), vp]
    L.imm_round_fold_eval.argtypes = [vp, vp, vp, vp, u64, ctypes.POINTER(u64), ctypes.POINTER(u64)]
    L.imm_verify.argtypes = [ctypes.POINTER(Commit), vp, ctypes.POINTER(Proof), vp, vp, vp, vp,
                             ctypes.POINTER(i32)]
    L.imm_debug_fetch.argtypes = [vp, i32, vp, u64, ctypes.POINTER(u64)]
    L.imm_ctx_set_option.argtypes = [vp, i32, ctypes.c_int64]
    L.imm_ctx_set_profiling.argtypes = [vp, u32]
    L.imm_ctx_kernel_time.argtypes = [vp, i32, ctypes.POINTER(u64), ctypes.POINTER(ctypes.c_double)]
    L.imm_ctx_reset_profiling.argtypes = [vp]
    L.imm_ldd_tv_kl.argtypes = [vp, vp, vp, vp, u64, u64, u64, vp, vp]
    L.imm_topk_distance.argtypes = [vp, vp, vp, u64, u64, u64, vp, u32, vp]
    L.imm_tail_density.argtypes = [vp, vp, vp, u64, ctypes.c_double, ctypes.POINTER(ctypes.c_double)]
    L.imm_commit_tables_device.argtypes = [vp, vp, i32, ctypes.POINTER(TableDesc), ctypes.POINTER(Commit1)]
    L.imm_mle_eval_static.argtypes = [vp, vp, i32, u64, u64, u64, vp, vp, vp]
    L.imm_verify_points.argtypes = [ctypes.POINTER(Commit), vp, ctypes.POINTER(Proof), vp, vp, vp]
    L.imm_transcript_challenge.argtypes = [vp, ctypes.POINTER(u64)]
    L.imm_debug_device_challenge.argtypes = [vp, vp, vp, ctypes.POINTER(u64)]
    L.imm_debug_timeline.argtypes = [vp, vp, vp, u32, ctypes.POINTER(u32)]
    for name in EXPORTS:
        if name != "imm_last_error":
            getattr(L, name).restype = i32
    _lib = L
    return L


def _check(rc: int, where: str) -> None:
    if rc < 0:
        raise ImmError(rc, where, load().imm_last_error().decode(errors="replace"))


def _host_ptr(a: Optional[np.ndarray], dtype) -> Optional[int]:
    if a is None:
        return None
    assert a.dtype == dtype and a.flags["C_CONTIGUOUS"], "host array must be C-contiguous %s" % dtype
    return a.ctypes.data


_TORCH_DT = None


def _tensor_dtype(t) -> int:
    global _TORCH_DT
    import torch
    if _TORCH_DT is None:
        _TORCH_DT = {torch.int8: IMM_I8, torch.int16: IMM_I16, torch.int64: IMM_I64, torch.uint64: IMM_F64P}
    return _TORCH_DT[t.dtype]


def _stream_handle(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


# ----------------------------------------------------------------------------- host-only calls
def imm_fs_init() -> bytes:
    buf = (ctypes.c_uint8 * 32)()
    _check(load().imm_fs_init(buf), "imm_fs_init")
    return bytes(buf)


def imm_commit_matmul(A: Optional[np.ndarray], B: Optional[np.ndarray], C: Optional[np.ndarray],
                      m: int, d: int, n: int, out: Optional[Commit] = None) -> Commit:
    com = out if out is not None else Commit()
    rc = load().imm_commit_matmul(_host_ptr(A, np.int16), _host_ptr(B, np.int8), _host_ptr(C, np.int64), m, d, n,
                                  ctypes.byref(com))
    _check(rc, "imm_commit_matmul")
    return com


def imm_verify(com: Commit, transcript_in: bytes, proof: Proof, A: Optional[np.ndarray] = None,
               B: Optional[np.ndarray] = None, C: Optional[np.ndarray] = None) -> Tuple[int, Optional[bytes], int]:
    """Returns (code, state_out or None, fail_round); code 0 = ACCEPT (all three openings checked),
    > 0 = reject reason; IMM_REJ_UNOPENED: nothing failed but a matrix was not supplied."""
    assert len(transcript_in) == 32
    sin = (ctypes.c_uint8 * 32).from_buffer_copy(transcript_in)
    sout = (ctypes.c_uint8 * 32)()
    fr = ctypes.c_int(0)
    rc = load().imm_verify(ctypes.byref(com), sin, ctypes.byref(proof), _host_ptr(A, np.int16),
                           _host_ptr(B, np.int8), _host_ptr(C, np.int64), sout, ctypes.byref(fr))
    _check(rc, "imm_verify")
    return rc, (bytes(sout) if rc in (0, IMM_REJ_UNOPENED) else None), fr.value


def imm_verify_points(com: Commit, transcript_in: bytes, proof: Proof) -> Tuple[List[int], List[int], List[int]]:
    """(rx, ry, r): the points at which c0, vA, vB of the proof are openings of C, A, B."""
    sin = (ctypes.c_uint8 * 32).from_buffer_copy(transcript_in)
    bufs = [(ctypes.c_uint64 * IMM_MAX_ROUNDS)() for _ in range(3)]
    rc = load().imm_verify_points(ctypes.byref(com), sin, ctypes.byref(proof), *bufs)
    if rc:
        raise ImmError(rc, "imm_verify_points", load().imm_last_error().decode(errors="replace") if rc < 0 else "")
    return ([int(v) for v in bufs[0][:proof.mu]], [int(v) for v in bufs[1][:proof.nu]],
            [int(v) for v in bufs[2][:proof.delta]])


def imm_transcript_challenge(state: bytes) -> Tuple[int, bytes]:
    """(challenge, next state) squeezed from a 32-byte transcript state on the host."""
    st = (ctypes.c_uint8 * 32).from_buffer_copy(state)
    out = ctypes.c_uint64(0)
    _check(load().imm_transcript_challenge(st, ctypes.byref(out)), "imm_transcript_challenge")
    return out.value, bytes(st)


# ----------------------------------------------------------------------------- device calls
IMM_STATIC_SCRATCH_BYTES = 8 << 20


def imm_mle_eval_static(table, pt_rows: Sequence[int], pt_cols: Sequence[int], out, stream=None,
                        rows: Optional[int] = None, cols: Optional[int] = None, ld: Optional[int] = None) -> None:
    """The allocation-free form of imm_mle_eval: no context; the value lands in out[0] (a device uint64
    tensor the caller owns) in stream order.  Nothing is synchronised."""
    import torch
    assert table.is_cuda and out.is_cuda and out.dtype == torch.uint64 and out.numel() >= 1
    if rows is None:
        assert table.dim() == 2 and table.is_contiguous()
        rows, cols = table.shape
        ld = cols
    pr = np.array([int(v) for v in pt_rows], dtype=np.uint64)
    pc = np.array([int(v) for v in pt_cols], dtype=np.uint64)
    rc = load().imm_mle_eval_static(_stream_handle(stream), table.data_ptr(), _tensor_dtype(table), rows, cols, ld,
                                    pr.ctypes.data if pr.size else None, pc.ctypes.data if pc.size else None,
                                    out.data_ptr())
    _check(rc, "imm_mle_eval_static")


class Context:
    """Owns an imm_ctx.  Methods carry the names of the C entry points."""

    def __init__(self, device: int = 0, scratch_bytes: int = 0):
        self._h = ctypes.c_void_p()
        _check(load().imm_ctx_create(ctypes.byref(self._h), device, scratch_bytes), "imm_ctx_create")

    def close(self) -> None:
        if self._h:
            load().imm_ctx_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def imm_ctx_set_option(self, option: int, value: int) -> None:
        _check(load().imm_ctx_set_option(self._h, option, value), "imm_ctx_set_option")

    def imm_ctx_set_profiling(self, mask: int) -> None:
        _check(load().imm_ctx_set_profiling(self._h, mask), "imm_ctx_set_profiling")

    def imm_ctx_reset_profiling(self) -> None:
        _check(load().imm_ctx_reset_profiling(self._h), "imm_ctx_reset_profiling")

    def imm_ctx_kernel_time(self, kernel_id: int) -> Tuple[int, float]:
        n, ms = ctypes.c_uint64(0), ctypes.c_double(0.0)
        _check(load().imm_ctx_kernel_time(self._h, kernel_id, ctypes.byref(n), ctypes.byref(ms)),
               "imm_ctx_kernel_time")
        return n.value, ms.value

    def imm_encode(self, src, dst=None, stream=None):
        import torch
        assert src.is_cuda and src.is_contiguous()
        if dst is None:
            dst = torch.empty(src.shape, dtype=torch.int64, device=src.device).view(torch.uint64)
        assert dst.is_cuda and dst.is_contiguous() and dst.dtype == torch.uint64 and dst.numel() == src.numel()
        _check(load().imm_encode(self._h, _stream_handle(stream), src.data_ptr(), _tensor_dtype(src), src.numel(),
                                 dst.data_ptr()), "imm_encode")
        return dst

    def imm_mle_eval(self, table, pt_rows: Sequence[int], pt_cols: Sequence[int], stream=None,
                     rows: Optional[int] = None, cols: Optional[int] = None, ld: Optional[int] = None) -> int:
        assert table.is_cuda
        if rows is None:
            assert table.dim() == 2 and table.is_contiguous()
            rows, cols = table.shape
            ld = cols
        pr = np.array([int(v) for v in pt_rows], dtype=np.uint64)
        pc = np.array([int(v) for v in pt_cols], dtype=np.uint64)
        out = ctypes.c_uint64(0)
        rc = load().imm_mle_eval(self._h, _stream_handle(stream), table.data_ptr(), _tensor_dtype(table), rows, cols,
                                 ld, pr.ctypes.data if pr.size else None, pc.ctypes.data if pc.size else None,
                                 ctypes.byref(out))
        _check(rc, "imm_mle_eval")
        return out.value

    def imm_sumcheck_matmul_prove(self, A, B, com: Commit, state: bytes, stream=None,
                                  shape: Optional[Tuple[int, int, int]] = None) -> Tuple[Proof, bytes]:
        """A, B: device tensors (int16 / int8 raw, or uint64 pre-encoded).  Returns (proof, state_out)."""
        assert A.is_cuda and B.is_cuda and A.is_contiguous() and B.is_contiguous()
        if shape is None:
            m, d = A.shape
            d2, n = B.shape
            assert d == d2
        else:
            m, d, n = shape
        st = (ctypes.c_uint8 * 32).from_buffer_copy(state)
        proof = Proof()
        rc = load().imm_sumcheck_matmul_prove(self._h, _stream_handle(stream), A.data_ptr(), _tensor_dtype(A),
                                              B.data_ptr(), _tensor_dtype(B), m, d, n, ctypes.byref(com), st,
                                              ctypes.byref(proof))
        _check(rc, "imm_sumcheck_matmul_prove")
        return proof, bytes(st)

    def imm_sumcheck_matmul_prove_batch(self, items, chained: bool, state: bytes, stream=None):
        """items: list of (A_dev, B_dev, Commit).  Returns (proofs, states, final_state)."""
        count = len(items)
        descs = (MatmulDesc * max(count, 1))()
        keep = []
        for t, (A, B, com) in enumerate(items):
            assert A.is_cuda and B.is_cuda and A.is_contiguous() and B.is_contiguous()
            m, d = A.shape
            d2, n = B.shape
            assert d == d2
            descs[t].A_dev, descs[t].B_dev = A.data_ptr(), B.data_ptr()
            descs[t].dtA, descs[t].dtB = _tensor_dtype(A), _tensor_dtype(B)
            descs[t].m, descs[t].d, descs[t].n = m, d, n
            descs[t].com = ctypes.pointer(com)
            keep.append(com)
        proofs = (Proof * max(count, 1))()
        states = (ctypes.c_uint8 * (32 * max(count, 1)))()
        st = (ctypes.c_uint8 * 32).from_buffer_copy(state)
        rc = load().imm_sumcheck_matmul_prove_batch(self._h, _stream_handle(stream), count, descs, 1 if chained else 0,
                                                    st, proofs, states)
        _check(rc, "imm_sumcheck_matmul_prove_batch")
        sb = bytes(states)
        return ([proofs[t].copy() for t in range(count)], [sb[32 * t:32 * t + 32] for t in range(count)], bytes(st))

    def imm_ldd_tv_kl(self, logits, ref, want_tv: bool = True, want_kl: bool = True, stream=None):
        """logits, ref: device float32 T x n.  Returns (tv, kl) device float64[T] tensors (None if not wanted)."""
        import torch
        assert logits.is_cuda and ref.is_cuda and logits.dtype == torch.float32 and ref.dtype == torch.float32
        assert logits.dim() == 2 and logits.shape == ref.shape and logits.stride(1) == 1 and ref.stride(1) == 1
        assert logits.stride(0) == ref.stride(0)
        T, n = logits.shape
        tv = torch.empty(T, dtype=torch.float64, device=logits.device) if want_tv else None
        kl = torch.empty(T, dtype=torch.float64, device=logits.device) if want_kl else None
        rc = load().imm_ldd_tv_kl(self._h, _stream_handle(stream), logits.data_ptr(), ref.data_ptr(), T, n,
                                  logits.stride(0), tv.data_ptr() if want_tv else None,
                                  kl.data_ptr() if want_kl else None)
        _check(rc, "imm_ldd_tv_kl")
        return tv, kl

    def imm_topk_distance(self, logits, idx, stream=None):
        """logits: device float32 T x n; idx: device int32 T x K.  Returns device float64[T]."""
        import torch
        assert logits.is_cuda and idx.is_cuda and logits.dtype == torch.float32 and idx.dtype == torch.int32
        assert logits.dim() == 2 and idx.dim() == 2 and logits.stride(1) == 1 and idx.is_contiguous()
        T, n = logits.shape
        assert idx.shape[0] == T
        out = torch.empty(T, dtype=torch.float64, device=logits.device)
        rc = load().imm_topk_distance(self._h, _stream_handle(stream), logits.data_ptr(), T, n, logits.stride(0),
                                      idx.data_ptr(), idx.shape[1], out.data_ptr())
        _check(rc, "imm_topk_distance")
        return out

    def imm_tail_density(self, dist, t1: float, stream=None) -> float:
        import torch
        assert dist.is_cuda and dist.dtype == torch.float64 and dist.is_contiguous()
        out = ctypes.c_double(0.0)
        rc = load().imm_tail_density(self._h, _stream_handle(stream), dist.data_ptr(), dist.numel(), float(t1),
                                     ctypes.byref(out))
        _check(rc, "imm_tail_density")
        return out.value

    def imm_commit_tables_device(self, tables, stream=None) -> List[Commit1]:
        """tables: contiguous 2-D device tensors of int8 / int16 / int64.  Returns one Commit1 per table."""
        count = len(tables)
        descs = (TableDesc * max(count, 1))()
        for t, tab in enumerate(tables):
            assert tab.is_cuda and tab.dim() == 2 and tab.is_contiguous()
            descs[t].table_dev, descs[t].dtype = tab.data_ptr(), _tensor_dtype(tab)
            descs[t].rows, descs[t].cols = tab.shape
        out = (Commit1 * max(count, 1))()
        rc = load().imm_commit_tables_device(self._h, _stream_handle(stream), count, descs, out)
        _check(rc, "imm_commit_tables_device")
        res = []
        for t in range(count):
            c = Commit1()
            ctypes.memmove(ctypes.byref(c), ctypes.byref(out[t]), ctypes.sizeof(Commit1))
            res.append(c)
        return res

    def prepare_batch(self, items, chained: bool, state: bytes, stream=None) -> "PreparedBatch":
        """Marshal a batch once; PreparedBatch.run() then only performs the C call."""
        return PreparedBatch(self, items, chained, state, stream)

    def imm_round_fold_eval(self, a, b, L: int, fold_r: Optional[int] = None, stream=None) -> List[int]:
        import torch
        assert a.is_cuda and b.is_cuda and a.dtype == torch.uint64 and b.dtype == torch.uint64
        assert a.numel() >= L and b.numel() >= L and a.is_contiguous() and b.is_contiguous()
        g = (ctypes.c_uint64 * 3)()
        r = ctypes.c_uint64(fold_r) if fold_r is not None else None
        rc = load().imm_round_fold_eval(self._h, _stream_handle(stream), a.data_ptr(), b.data_ptr(), L,
                                        ctypes.byref(r) if r is not None else None, g)
        _check(rc, "imm_round_fold_eval")
        return [int(v) for v in g]

    def imm_debug_timeline(self) -> List[Tuple[str, int]]:
        """[(point name, CLOCK_MONOTONIC ns)] of the most recent proof (needs IMM_OPT_TIMELINE)."""
        ids, ns, cnt = (ctypes.c_uint32 * 32)(), (ctypes.c_uint64 * 32)(), ctypes.c_uint32(0)
        _check(load().imm_debug_timeline(self._h, ids, ns, 32, ctypes.byref(cnt)), "imm_debug_timeline")
        return [(TIMELINE_NAMES[ids[i]], int(ns[i])) for i in range(min(cnt.value, 32))]

    def imm_debug_device_challenge(self, state: bytes, stream=None) -> Tuple[int, bytes]:
        st = (ctypes.c_uint8 * 32).from_buffer_copy(state)
        out = ctypes.c_uint64(0)
        _check(load().imm_debug_device_challenge(self._h, _stream_handle(stream), st, ctypes.byref(out)),
               "imm_debug_device_challenge")
        return out.value, bytes(st)

    def imm_debug_fetch(self, which: int) -> np.ndarray:
        cnt = ctypes.c_uint64(0)
        _check(load().imm_debug_fetch(self._h, which, None, 0, ctypes.byref(cnt)), "imm_debug_fetch")
        out = np.zeros(cnt.value, dtype=np.uint64)
        if cnt.value:
            _check(load().imm_debug_fetch(self._h, which, out.ctypes.data, cnt.value, ctypes.byref(cnt)),
                   "imm_debug_fetch")
        return out


class PreparedBatch:
    """Pre-marshalled arguments of imm_sumcheck_matmul_prove_batch for repeated calls on the same
    device buffers (what a serving loop or a benchmark does).  run() resets the starting state and
    forwards to the C entry point; the results are read from .proofs / .states / .final_state."""

    def __init__(self, ctx: Context, items, chained: bool, state: bytes, stream=None):
        self._ctx = ctx
        self._count = len(items)
        n = max(self._count, 1)
        self._descs = (MatmulDesc * n)()
        self._keep = []
        for t, (A, B, com) in enumerate(items):
            assert A.is_cuda and B.is_cuda and A.is_contiguous() and B.is_contiguous()
            m, d = A.shape
            d2, nn = B.shape
            assert d == d2
            self._descs[t].A_dev, self._descs[t].B_dev = A.data_ptr(), B.data_ptr()
            self._descs[t].dtA, self._descs[t].dtB = _tensor_dtype(A), _tensor_dtype(B)
            self._descs[t].m, self._descs[t].d, self._descs[t].n = m, d, nn
            self._descs[t].com = ctypes.pointer(com)
            self._keep.append((A, B, com))
        self._proofs = (Proof * n)()
        self._states = (ctypes.c_uint8 * (32 * n))()
        self._state0 = bytes(state)
        self._st = (ctypes.c_uint8 * 32)()
        self._chained = 1 if chained else 0
        self._stream = _stream_handle(stream)
        self._fn = load().imm_sumcheck_matmul_prove_batch

    def run(self) -> None:
        ctypes.memmove(self._st, self._state0, 32)
        rc = self._fn(self._ctx._h, self._stream, self._count, self._descs, self._chained, self._st, self._proofs,
                      self._states)
        if rc:
            _check(rc, "imm_sumcheck_matmul_prove_batch")

    @property
    def proofs(self) -> List[Proof]:
        return [self._proofs[t].copy() for t in range(self._count)]

    @property
    def states(self) -> List[bytes]:
        sb = bytes(self._states)
        return [sb[32 * t:32 * t + 32] for t in range(self._count)]

    @property
    def final_state(self) -> bytes:
        return bytes(self._st)
