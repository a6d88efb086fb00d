"""ctypes binding of libquoka's C ABI (see include/quoka.h).

Argument marshalling only: every function takes torch tensors that already live on the GPU, passes
their device pointers and the current HIP stream to the C entry point of the same name, and raises
QuokaError on a non-zero status.  No arithmetic of the method happens in Python, and there is no
fallback: if the shared library has not been built the import of a symbol fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

QUOKA_F32 = 0
QUOKA_BF16 = 1

_LIB_NAME = "libquoka.so"
_lib: Optional[ctypes.CDLL] = None

EXPORTS = (
    "quoka_workspace_bytes", "quoka_select_queries", "quoka_score_keys", "quoka_topk_keys", "quoka_select_keys",
    "quoka_sparse_attn", "quoka_dense_attn", "quoka_chunk_attn", "quoka_prefill_attn", "quoka_topk_keys_noalloc",
    "quoka_probe_mfma", "quoka_probe_read", "quoka_probe_attn_mix", "quoka_status_string", "quoka_version",
)
_STATUS_EXPORTS = EXPORTS[:-2]   # everything that returns a quoka_status


class QuokaError(RuntimeError):
    def __init__(self, fn: str, status: int, msg: str):
        super().__init__(f"{fn} failed: status {status} ({msg})")
        self.status = status


class QuokaShape(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("chunk_len", ctypes.c_int32), ("max_kv_len", ctypes.c_int32),
        ("n_retain", ctypes.c_int32), ("max_budget", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("score_flags", ctypes.c_int32),
        ("q_stride", ctypes.c_int64 * 3), ("kv_stride", ctypes.c_int64 * 3),
        ("ck_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3),
    ]

    @property
    def n_keep(self) -> int:
        return min(self.n_retain, self.chunk_len)


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), _LIB_NAME)


def load_library() -> ctypes.CDLL:
    """Load the in-tree libquoka.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: build it with `python -m paper_2602_08722_amd.build`")
    lib = ctypes.CDLL(path)
    P, I32P, F32P, SZ = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t
    SH = ctypes.POINTER(QuokaShape)
    lib.quoka_workspace_bytes.argtypes = [SH, ctypes.POINTER(ctypes.c_size_t)]
    lib.quoka_select_queries.argtypes = [SH, P, I32P, F32P, P, SZ, P]
    lib.quoka_score_keys.argtypes = [SH, F32P, P, I32P, F32P, P, SZ, P]
    lib.quoka_topk_keys.argtypes = [SH, F32P, I32P, I32P, I32P, I32P, P, SZ, P]
    lib.quoka_select_keys.argtypes = [SH, F32P, P, I32P, I32P, F32P, I32P, I32P, P, SZ, P]
    lib.quoka_sparse_attn.argtypes = [SH, P, P, P, I32P, I32P, P, P, P, F32P, P, SZ, P]
    lib.quoka_dense_attn.argtypes = [SH, P, P, P, I32P, P, P, P, F32P, P, SZ, P]
    lib.quoka_chunk_attn.argtypes = [SH, P, P, P, I32P, I32P, P, P, I32P, F32P, F32P, I32P, I32P, P, F32P, P, SZ, P]
    lib.quoka_prefill_attn.argtypes = [SH, ctypes.c_int, P, P, P, I32P, I32P, I32P, F32P, F32P, I32P, I32P, P, P, SZ, P]
    lib.quoka_topk_keys_noalloc.argtypes = [SH, F32P, I32P, I32P, I32P, I32P, P]
    lib.quoka_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, F32P, P]
    lib.quoka_probe_read.argtypes = [P, SZ, F32P, P]
    lib.quoka_probe_attn_mix.argtypes = [ctypes.c_int, ctypes.c_int, F32P, P]
    for name in _STATUS_EXPORTS:
        getattr(lib, name).restype = ctypes.c_int
    lib.quoka_status_string.argtypes = [ctypes.c_int]
    lib.quoka_status_string.restype = ctypes.c_char_p
    lib.quoka_version.argtypes = []
    lib.quoka_version.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(fn: str, status: int) -> None:
    if status != 0:
        raise QuokaError(fn, status, load_library().quoka_status_string(status).decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _strides3(t: torch.Tensor):
    assert t.dim() == 4 and t.stride(3) == 1, "expected [batch, heads, tokens, head_dim] with head_dim contiguous"
    return (ctypes.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2))


QUOKA_SCORE_DOT, QUOKA_SCORE_MEAN, QUOKA_SELECT_UNIFORM, QUOKA_SCORE_QBAR_BF16, QUOKA_ATTN_SCALE_F32 = 1, 2, 4, 8, 16   # quoka.h


def make_shape(q: torch.Tensor, k_cache: torch.Tensor, k_chunk: torch.Tensor, out: torch.Tensor,
               n_retain: int, max_budget: int, score_flags: int = 0) -> QuokaShape:
    """Describe the problem from the tensors' own shapes and strides (no copies)."""
    b, n_q, C, d = q.shape
    n_kv, t_max = k_cache.shape[1], k_cache.shape[2]
    if q.dtype == torch.bfloat16:
        dt = QUOKA_BF16
    elif q.dtype == torch.float32:
        dt = QUOKA_F32
    else:
        raise TypeError(f"unsupported dtype {q.dtype}")
    s = QuokaShape()
    s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim = b, n_q, n_kv, d
    s.chunk_len, s.max_kv_len, s.n_retain, s.max_budget = C, t_max, n_retain, max_budget
    s.dtype, s.score_flags = dt, int(score_flags)
    s.q_stride = _strides3(q)
    if t_max > 0:
        s.kv_stride = _strides3(k_cache)
    else:
        s.kv_stride = (ctypes.c_int64 * 3)(0, 0, d)
    s.ck_stride = _strides3(k_chunk)
    s.o_stride = _strides3(out)
    return s


def quoka_version() -> int:
    return load_library().quoka_version()


def quoka_workspace_bytes(shape: QuokaShape) -> int:
    n = ctypes.c_size_t(0)
    _check("quoka_workspace_bytes", load_library().quoka_workspace_bytes(ctypes.byref(shape), ctypes.byref(n)))
    return int(n.value)


def quoka_select_queries(shape, q, q_idx, qbar, workspace, stream=None) -> None:
    _check("quoka_select_queries", load_library().quoka_select_queries(
        ctypes.byref(shape), _ptr(q), _ptr(q_idx), _ptr(qbar), _ptr(workspace), workspace.numel(), _stream(stream)))


def quoka_score_keys(shape, qbar, k_cache, kv_lens, scores, workspace, stream=None) -> None:
    _check("quoka_score_keys", load_library().quoka_score_keys(
        ctypes.byref(shape), _ptr(qbar), _ptr(k_cache), _ptr(kv_lens), _ptr(scores), _ptr(workspace),
        workspace.numel(), _stream(stream)))


def quoka_topk_keys(shape, scores, kv_lens, budgets, k_idx, k_cnt, workspace, stream=None) -> None:
    _check("quoka_topk_keys", load_library().quoka_topk_keys(
        ctypes.byref(shape), _ptr(scores), _ptr(kv_lens), _ptr(budgets), _ptr(k_idx), _ptr(k_cnt), _ptr(workspace),
        workspace.numel(), _stream(stream)))


def quoka_select_keys(shape, qbar, k_cache, kv_lens, budgets, scores, k_idx, k_cnt, workspace, stream=None) -> None:
    _check("quoka_select_keys", load_library().quoka_select_keys(
        ctypes.byref(shape), _ptr(qbar), _ptr(k_cache), _ptr(kv_lens), _ptr(budgets), _ptr(scores), _ptr(k_idx),
        _ptr(k_cnt), _ptr(workspace), workspace.numel(), _stream(stream)))


def quoka_topk_keys_noalloc(shape, scores, kv_lens, budgets, k_idx, k_cnt, stream=None) -> None:
    _check("quoka_topk_keys_noalloc", load_library().quoka_topk_keys_noalloc(
        ctypes.byref(shape), _ptr(scores), _ptr(kv_lens), _ptr(budgets), _ptr(k_idx), _ptr(k_cnt), _stream(stream)))


def quoka_probe_mfma(blocks: int, iters: int, sink, stream=None) -> None:
    _check("quoka_probe_mfma", load_library().quoka_probe_mfma(int(blocks), int(iters), _ptr(sink), _stream(stream)))


def quoka_probe_attn_mix(blocks: int, steps: int, sink, stream=None) -> None:
    _check("quoka_probe_attn_mix", load_library().quoka_probe_attn_mix(int(blocks), int(steps), _ptr(sink),
                                                                       _stream(stream)))


def quoka_probe_read(src, nbytes: int, sink, stream=None) -> None:
    _check("quoka_probe_read", load_library().quoka_probe_read(_ptr(src), int(nbytes), _ptr(sink), _stream(stream)))


def quoka_sparse_attn(shape, q, k_cache, v_cache, k_idx, k_cnt, k_chunk, v_chunk, out, lse, workspace,
                      stream=None) -> None:
    _check("quoka_sparse_attn", load_library().quoka_sparse_attn(
        ctypes.byref(shape), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_idx), _ptr(k_cnt), _ptr(k_chunk),
        _ptr(v_chunk), _ptr(out), _ptr(lse), _ptr(workspace), workspace.numel(), _stream(stream)))


def quoka_dense_attn(shape, q, k_cache, v_cache, kv_lens, k_chunk, v_chunk, out, lse, workspace, stream=None) -> None:
    _check("quoka_dense_attn", load_library().quoka_dense_attn(
        ctypes.byref(shape), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(kv_lens), _ptr(k_chunk), _ptr(v_chunk),
        _ptr(out), _ptr(lse), _ptr(workspace), workspace.numel(), _stream(stream)))


def quoka_chunk_attn(shape, q, k_cache, v_cache, kv_lens, budgets, k_chunk, v_chunk, q_idx, qbar, scores, k_idx,
                     k_cnt, out, lse, workspace, stream=None) -> None:
    _check("quoka_chunk_attn", load_library().quoka_chunk_attn(
        ctypes.byref(shape), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(kv_lens), _ptr(budgets), _ptr(k_chunk),
        _ptr(v_chunk), _ptr(q_idx), _ptr(qbar), _ptr(scores), _ptr(k_idx), _ptr(k_cnt), _ptr(out), _ptr(lse),
        _ptr(workspace), workspace.numel(), _stream(stream)))


def quoka_prefill_attn(shape, sparse, q, k, v, kv_lens_all, budgets_all, q_idx, qbar, scores, k_idx, k_cnt, out,
                       workspace, stream=None) -> None:
    _check("quoka_prefill_attn", load_library().quoka_prefill_attn(
        ctypes.byref(shape), int(bool(sparse)), _ptr(q), _ptr(k), _ptr(v), _ptr(kv_lens_all), _ptr(budgets_all),
        _ptr(q_idx), _ptr(qbar), _ptr(scores), _ptr(k_idx), _ptr(k_cnt), _ptr(out), _ptr(workspace),
        workspace.numel(), _stream(stream)))


class PrefillBuffers:
    """Device buffers for chunked prefill of a whole prompt (allocation only; torch owns the memory).

    q [b, n_Q, L, d], k / v [b, n_KV, L, d]; `budget` is B_SA per chunk: an int, or a callable of the cache length.
    """

    def __init__(self, q, k, v, chunk, n_retain, budget, score_flags=0):
        dev = q.device
        b, n_q, L, d = q.shape
        n_kv = k.shape[1]
        self.q, self.k, self.v = q, k, v
        n_chunks = -(-L // chunk)
        lens = [[i * chunk] * b for i in range(n_chunks)]
        bud = [[int(budget(i * chunk)) if callable(budget) else int(budget)] * b for i in range(n_chunks)]
        max_budget = max(0, min(max(x[0] for x in bud), L))
        self.kv_lens_all = torch.tensor(lens, dtype=torch.int32, device=dev)
        self.budgets_all = torch.tensor(bud, dtype=torch.int32, device=dev)
        self.out = torch.empty_like(q)
        # the shape describes one chunk of `chunk` rows taken from the prompt tensors (their strides, no copies)
        self.shape = make_shape(q[:, :, :chunk], k, k[:, :, :chunk], self.out[:, :, :chunk], n_retain, max_budget,
                                score_flags)
        n_keep = self.shape.n_keep
        self.q_idx = torch.empty((b, n_q, n_keep), dtype=torch.int32, device=dev)
        self.qbar = torch.empty((b, n_kv, n_keep, d), dtype=torch.float32, device=dev)
        self.scores = torch.empty((b, n_kv, L), dtype=torch.float32, device=dev)
        self.k_idx = torch.empty((b, n_kv, max(max_budget, 1)), dtype=torch.int32, device=dev)
        self.k_cnt = torch.empty((b, n_kv), dtype=torch.int32, device=dev)
        self.workspace = torch.empty(quoka_workspace_bytes(self.shape), dtype=torch.uint8, device=dev)

    def run(self, sparse=True):
        quoka_prefill_attn(self.shape, sparse, self.q, self.k, self.v, self.kv_lens_all, self.budgets_all, self.q_idx,
                           self.qbar, self.scores, self.k_idx, self.k_cnt, self.out, self.workspace)
        return self.out


class ChunkBuffers:
    """Device buffers for one chunk-attention problem (allocation only; torch owns the memory)."""

    def __init__(self, q, k_cache, v_cache, k_chunk, v_chunk, kv_lens, budgets, n_retain, max_budget=None,
                 score_flags=0):
        dev = q.device
        b, n_q, C, d = q.shape
        n_kv, t_max = k_cache.shape[1], k_cache.shape[2]
        self.q, self.k_cache, self.v_cache, self.k_chunk, self.v_chunk = q, k_cache, v_cache, k_chunk, v_chunk
        self.kv_lens = torch.as_tensor(kv_lens, dtype=torch.int32).to(dev)
        self.budgets = torch.as_tensor(budgets, dtype=torch.int32).to(dev)
        if max_budget is None:
            max_budget = min(int(max(budgets)), t_max) if len(budgets) else 0
        self.out = torch.empty_like(q)
        self.shape = make_shape(q, k_cache, k_chunk, self.out, n_retain, max_budget, score_flags)
        n_keep = self.shape.n_keep
        self.q_idx = torch.empty((b, n_q, n_keep), dtype=torch.int32, device=dev)
        self.qbar = torch.empty((b, n_kv, n_keep, d), dtype=torch.float32, device=dev)
        self.scores = torch.empty((b, n_kv, max(t_max, 1)), dtype=torch.float32, device=dev)
        self.k_idx = torch.empty((b, n_kv, max(max_budget, 1)), dtype=torch.int32, device=dev)
        self.k_cnt = torch.empty((b, n_kv), dtype=torch.int32, device=dev)
        self.lse = torch.empty((b, n_q, C), dtype=torch.float32, device=dev)
        self.workspace = torch.empty(quoka_workspace_bytes(self.shape), dtype=torch.uint8, device=dev)

    # the five stage calls and the fused convenience call, on the current stream
    def select_queries(self):
        quoka_select_queries(self.shape, self.q, self.q_idx, self.qbar, self.workspace)

    def score_keys(self):
        quoka_score_keys(self.shape, self.qbar, self.k_cache, self.kv_lens, self.scores, self.workspace)

    def topk_keys(self):
        quoka_topk_keys(self.shape, self.scores, self.kv_lens, self.budgets, self.k_idx, self.k_cnt, self.workspace)

    def select_keys(self):
        quoka_select_keys(self.shape, self.qbar, self.k_cache, self.kv_lens, self.budgets, self.scores, self.k_idx,
                          self.k_cnt, self.workspace)

    def sparse_attn(self, out=None, lse=None):
        quoka_sparse_attn(self.shape, self.q, self.k_cache, self.v_cache, self.k_idx, self.k_cnt, self.k_chunk,
                          self.v_chunk, self.out if out is None else out, self.lse if lse is None else lse,
                          self.workspace)
        return self.out if out is None else out

    def dense_attn(self, out=None, lse=None):
        quoka_dense_attn(self.shape, self.q, self.k_cache, self.v_cache, self.kv_lens, self.k_chunk, self.v_chunk,
                         self.out if out is None else out, self.lse if lse is None else lse, self.workspace)
        return self.out if out is None else out

    def chunk_attn(self):
        quoka_chunk_attn(self.shape, self.q, self.k_cache, self.v_cache, self.kv_lens, self.budgets, self.k_chunk,
                         self.v_chunk, self.q_idx, self.qbar, self.scores, self.k_idx, self.k_cnt, self.out, self.lse,
                         self.workspace)
        return self.out
