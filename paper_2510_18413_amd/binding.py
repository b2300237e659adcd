"""ctypes binding of libadamas.so: argument marshalling only.

Every function mirrors the C entry point of the same name in include/adamas.h, takes torch
tensors that already live on the GPU, checks dtype / device / contiguity, and passes raw
device pointers plus the current HIP stream.  All arithmetic happens in the HIP kernels; there
is no CPU or PyTorch fallback: if the shared library is missing and cannot be built, loading
raises.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

from . import build as _build

EXPORTED_SYMBOLS = (
    "adamas_status_string",
    "adamas_build_id",
    "adamas_last_hip_error",
    "adamas_workspace_bytes",
    "adamas_encode_keys",
    "adamas_encode_query",
    "adamas_manhattan_distance",
    "adamas_select_topk",
    "adamas_sparse_attn",
    "adamas_decode_step",
    "adamas_decode_step_stages",
    "adamas_decode_step_static",
    "adamas_phase_trace",
    "adamas_stream_read",
    "adamas_decode_step_paged",
    "adamas_full_attn_workspace_bytes",
    "adamas_full_attn",
)

HEAD_DIM = 128
CODE_ROW_BYTES = 32
VARIANT_NO_HADAMARD = 1
VARIANT_L2 = 2
STAGE_SCAN, STAGE_SELECT_ATTN, STAGE_ALL = 1, 2, 3
STATIC_SCRATCH_BYTES = 16 << 20


class AdamasError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        hip = library().adamas_last_hip_error() if status == -4 else 0
        super().__init__("%s: %s (%d)%s" % (where, adamas_status_string(status), status,
                                            " hipError %d" % hip if hip else ""))


class Config(ctypes.Structure):
    """Mirror of struct adamas_config."""
    _fields_ = [
        ("head_dim", ctypes.c_int32),
        ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("variant", ctypes.c_uint32),
        ("pool_tokens", ctypes.c_int64),
        ("thr_k", ctypes.c_float * 7),
        ("thr_q", ctypes.c_float * 7),
        ("sm_scale", ctypes.c_float),
        ("code_bits", ctypes.c_int32),
    ]

    @property
    def code_row_bytes(self) -> int:
        return self.head_dim // 8 * (self.code_bits or 2)

    @classmethod
    def make(cls, num_q_heads: int, num_kv_heads: int, pool_tokens: int,
             thr_k: Sequence[float] = (-1.0, 0.0, 1.0), thr_q: Optional[Sequence[float]] = None,
             sm_scale: float = 0.0, head_dim: int = HEAD_DIM, variant: int = 0,
             code_bits: int = 0) -> "Config":
        """thr_k / thr_q hold 2^code_bits - 1 thresholds (three for the default 2-bit codes)."""
        thr_q = thr_k if thr_q is None else thr_q
        n_thr = (1 << (code_bits or 2)) - 1
        if len(thr_k) != n_thr or len(thr_q) != n_thr:
            raise ValueError("%d thresholds needed for %d-bit codes" % (n_thr, code_bits or 2))
        pad = lambda t: (ctypes.c_float * 7)(*(list(t) + [0.0] * (7 - len(t))))
        return cls(head_dim, num_q_heads, num_kv_heads, variant, pool_tokens, pad(thr_k), pad(thr_q),
                   sm_scale, code_bits)


_lib = None


def library_path():
    return _build.LIB


def library() -> ctypes.CDLL:
    """Loads libadamas.so, building it first (in a child process, before anything here touches
    the GPU library) when it is missing or was built from sources other than the tree's.  The
    environment variable ADAMAS_LIBRARY names another built library to load instead."""
    global _lib
    if _lib is None:
        # torch first: the process then has one HIP runtime (the one torch ships), and this
        # library, which only needs the public HIP launch API, binds to it.
        import torch  # noqa: F401
        path = os.environ.get("ADAMAS_LIBRARY")     # a library built elsewhere: loaded as it is
        if not path:
            if _build.is_stale():
                _build.build()
            path = str(_build.LIB)
        lib = ctypes.CDLL(path)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        cfgp = ctypes.POINTER(Config)
        lib.adamas_status_string.restype = ctypes.c_char_p
        lib.adamas_status_string.argtypes = [ctypes.c_int]
        lib.adamas_build_id.restype = ctypes.c_char_p
        lib.adamas_build_id.argtypes = []
        lib.adamas_last_hip_error.restype = ctypes.c_int
        lib.adamas_last_hip_error.argtypes = []
        lib.adamas_workspace_bytes.restype = sz
        lib.adamas_workspace_bytes.argtypes = [cfgp, i32, i64, i32]
        lib.adamas_encode_keys.restype = ctypes.c_int
        lib.adamas_encode_keys.argtypes = [cfgp, vp, vp, i64, i64, vp]
        lib.adamas_encode_query.restype = ctypes.c_int
        lib.adamas_encode_query.argtypes = [cfgp, vp, vp, i32, vp]
        lib.adamas_manhattan_distance.restype = ctypes.c_int
        lib.adamas_manhattan_distance.argtypes = [cfgp, vp, vp, vp, vp, i32, vp, i64, vp]
        lib.adamas_select_topk.restype = ctypes.c_int
        lib.adamas_select_topk.argtypes = [cfgp, vp, vp, vp, vp, i32, i32, vp, vp, i64, vp, sz, vp]
        lib.adamas_sparse_attn.restype = ctypes.c_int
        lib.adamas_sparse_attn.argtypes = [cfgp, vp, vp, vp, vp, vp, i32, i32, vp, i64, vp, sz, vp]
        lib.adamas_decode_step.restype = ctypes.c_int
        lib.adamas_decode_step.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp,
                                           i64, vp, sz, vp]
        lib.adamas_decode_step_static.restype = ctypes.c_int
        lib.adamas_decode_step_static.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp,
                                                  vp, i64, vp]
        lib.adamas_phase_trace.restype = ctypes.c_int
        lib.adamas_phase_trace.argtypes = [vp, vp, i64]
        lib.adamas_decode_step_paged.restype = ctypes.c_int
        lib.adamas_decode_step_paged.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp,
                                                 i32, i32, vp, vp, i64, vp, sz, vp,
                                                 ctypes.c_uint32]
        lib.adamas_full_attn_workspace_bytes.restype = sz
        lib.adamas_full_attn_workspace_bytes.argtypes = [cfgp, i32, i64]
        lib.adamas_full_attn.restype = ctypes.c_int
        lib.adamas_full_attn.argtypes = [cfgp, vp, vp, vp, vp, vp, i32, vp, i64, vp, sz, vp]
        lib.adamas_stream_read.restype = ctypes.c_int
        lib.adamas_stream_read.argtypes = [vp, sz, vp, vp]
        lib.adamas_decode_step_stages.restype = ctypes.c_int
        lib.adamas_decode_step_stages.argtypes = lib.adamas_decode_step.argtypes + [ctypes.c_uint32]
        _lib = lib
    return _lib


def adamas_status_string(status: int) -> str:
    return library().adamas_status_string(int(status)).decode()


def build_id() -> str:
    """Hash of the sources the loaded library was built from."""
    return library().adamas_build_id().decode()


def adamas_workspace_bytes(cfg: Config, batch: int, max_seq_len: int, k: int) -> int:
    return int(library().adamas_workspace_bytes(ctypes.byref(cfg), batch, max_seq_len, k))


# ------------------------------------------------------------------ tensor marshalling

def _ptr(t, dtype, name, shape=None, optional=False):
    import torch
    if t is None:
        if optional:
            return None
        raise TypeError("%s must not be None" % name)
    if not isinstance(t, torch.Tensor):
        raise TypeError("%s must be a torch.Tensor" % name)
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if t.dtype != dtype:
        raise ValueError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    return t.data_ptr()


def _stream(stream):
    import torch
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(rc, where):
    if rc != 0:
        raise AdamasError(rc, where)


def adamas_encode_keys(cfg: Config, K, codes, row_begin: int, n_rows: int, stream=None) -> None:
    import torch
    hkv, pool = cfg.num_kv_heads, cfg.pool_tokens
    rc = library().adamas_encode_keys(
        ctypes.byref(cfg), _ptr(K, torch.bfloat16, "K", (hkv, pool, cfg.head_dim)),
        _ptr(codes, torch.uint8, "codes", (hkv, pool, cfg.code_row_bytes)), row_begin, n_rows,
        _stream(stream))
    _check(rc, "adamas_encode_keys")


def adamas_encode_query(cfg: Config, q, qcodes, stream=None) -> None:
    import torch
    batch = q.shape[0]
    rc = library().adamas_encode_query(
        ctypes.byref(cfg), _ptr(q, torch.bfloat16, "q", (batch, cfg.num_q_heads, cfg.head_dim)),
        _ptr(qcodes, torch.uint8, "qcodes", (batch, cfg.num_q_heads, cfg.code_row_bytes)), batch,
        _stream(stream))
    _check(rc, "adamas_encode_query")


def adamas_decode_step_paged(cfg: Config, q, K, V, codes, page_table, page_tokens: int, seq_len,
                             k: int, out, max_seq_len: int, workspace, k_new=None, v_new=None,
                             idx_out=None, stream=None, stages=STAGE_ALL) -> None:
    import torch
    batch = q.shape[0]
    hkv, pool = cfg.num_kv_heads, cfg.pool_tokens
    if page_table.dim() != 2 or page_table.shape[0] != batch:
        raise ValueError("page_table must have shape (batch, max_pages)")
    rc = library().adamas_decode_step_paged(
        ctypes.byref(cfg), _ptr(q, torch.bfloat16, "q", (batch, cfg.num_q_heads, cfg.head_dim)),
        _ptr(k_new, torch.bfloat16, "k_new", (batch, hkv, cfg.head_dim), optional=True),
        _ptr(v_new, torch.bfloat16, "v_new", (batch, hkv, cfg.head_dim), optional=True),
        _ptr(K, torch.bfloat16, "K", (hkv, pool, cfg.head_dim)),
        _ptr(V, torch.bfloat16, "V", (hkv, pool, cfg.head_dim)),
        _ptr(codes, torch.uint8, "codes", (hkv, pool, cfg.code_row_bytes)),
        _ptr(page_table, torch.int32, "page_table"), page_table.shape[1], int(page_tokens),
        _ptr(seq_len, torch.int32, "seq_len", (batch,)), batch, k,
        _ptr(out, torch.float32, "out", (batch, cfg.num_q_heads, cfg.head_dim)),
        _ptr(idx_out, torch.int32, "idx_out", (batch, cfg.num_q_heads, k), optional=True),
        max_seq_len, _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream),
        int(stages))
    _check(rc, "adamas_decode_step_paged")


def adamas_full_attn_workspace_bytes(cfg: Config, batch: int, max_seq_len: int) -> int:
    return int(library().adamas_full_attn_workspace_bytes(ctypes.byref(cfg), batch, max_seq_len))


def adamas_full_attn(cfg: Config, q, K, V, seq_start, seq_len, out, max_seq_len: int, workspace,
                     stream=None) -> None:
    import torch
    batch = q.shape[0]
    hkv, pool = cfg.num_kv_heads, cfg.pool_tokens
    rc = library().adamas_full_attn(
        ctypes.byref(cfg), _ptr(q, torch.bfloat16, "q", (batch, cfg.num_q_heads, cfg.head_dim)),
        _ptr(K, torch.bfloat16, "K", (hkv, pool, cfg.head_dim)),
        _ptr(V, torch.bfloat16, "V", (hkv, pool, cfg.head_dim)),
        _ptr(seq_start, torch.int64, "seq_start", (batch,)),
        _ptr(seq_len, torch.int32, "seq_len", (batch,)), batch,
        _ptr(out, torch.float32, "out", (batch, cfg.num_q_heads, cfg.head_dim)),
        max_seq_len, _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    _check(rc, "adamas_full_attn")


def adamas_stream_read(src, sink, stream=None) -> None:
    """Reads every byte of the uint8 tensor `src` once (measurement aid); `sink` int32, >= 1 element."""
    import torch
    rc = library().adamas_stream_read(_ptr(src, torch.uint8, "src"), src.numel(),
                                      _ptr(sink, torch.int32, "sink"), _stream(stream))
    _check(rc, "adamas_stream_read")


def adamas_manhattan_distance(cfg: Config, qcodes, codes, seq_start, seq_len, dist_out,
                              stream=None) -> None:
    import torch
    batch = qcodes.shape[0]
    max_seq_len = dist_out.shape[2]
    rc = library().adamas_manhattan_distance(
        ctypes.byref(cfg),
        _ptr(qcodes, torch.uint8, "qcodes", (batch, cfg.num_q_heads, cfg.code_row_bytes)),
        _ptr(codes, torch.uint8, "codes", (cfg.num_kv_heads, cfg.pool_tokens, cfg.code_row_bytes)),
        _ptr(seq_start, torch.int64, "seq_start", (batch,)),
        _ptr(seq_len, torch.int32, "seq_len", (batch,)), batch,
        _ptr(dist_out, torch.uint16, "dist_out", (batch, cfg.num_q_heads, max_seq_len)),
        max_seq_len, _stream(stream))
    _check(rc, "adamas_manhattan_distance")


def adamas_select_topk(cfg: Config, qcodes, codes, seq_start, seq_len, k: int, idx_out,
                       max_seq_len: int, workspace, dist_out=None, stream=None) -> None:
    import torch
    batch = qcodes.shape[0]
    rc = library().adamas_select_topk(
        ctypes.byref(cfg),
        _ptr(qcodes, torch.uint8, "qcodes", (batch, cfg.num_q_heads, cfg.code_row_bytes)),
        _ptr(codes, torch.uint8, "codes", (cfg.num_kv_heads, cfg.pool_tokens, cfg.code_row_bytes)),
        _ptr(seq_start, torch.int64, "seq_start", (batch,)),
        _ptr(seq_len, torch.int32, "seq_len", (batch,)), batch, k,
        _ptr(idx_out, torch.int32, "idx_out", (batch, cfg.num_q_heads, k)),
        _ptr(dist_out, torch.uint16, "dist_out", (batch, cfg.num_q_heads, max_seq_len),
             optional=True),
        max_seq_len, _ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _stream(stream))
    _check(rc, "adamas_select_topk")


def adamas_sparse_attn(cfg: Config, q, K, V, seq_start, idx, out, max_seq_len: int, workspace,
                       stream=None) -> None:
    import torch
    batch, _, k = idx.shape
    hkv, pool = cfg.num_kv_heads, cfg.pool_tokens
    rc = library().adamas_sparse_attn(
        ctypes.byref(cfg), _ptr(q, torch.bfloat16, "q", (batch, cfg.num_q_heads, cfg.head_dim)),
        _ptr(K, torch.bfloat16, "K", (hkv, pool, cfg.head_dim)),
        _ptr(V, torch.bfloat16, "V", (hkv, pool, cfg.head_dim)),
        _ptr(seq_start, torch.int64, "seq_start", (batch,)),
        _ptr(idx, torch.int32, "idx", (batch, cfg.num_q_heads, k)), batch, k,
        _ptr(out, torch.float32, "out", (batch, cfg.num_q_heads, cfg.head_dim)), max_seq_len,
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    _check(rc, "adamas_sparse_attn")




def adamas_decode_step(cfg: Config, q, K, V, codes, seq_start, seq_len, k: int, out,
                       max_seq_len: int, workspace, k_new=None, v_new=None, idx_out=None,
                       stream=None) -> None:
    adamas_decode_step_stages(cfg, q, K, V, codes, seq_start, seq_len, k, out, max_seq_len,
                              workspace, k_new=k_new, v_new=v_new, idx_out=idx_out, stream=stream,
                              stages=None)


TRACE_SLOTS = 16


def adamas_phase_trace(scan_records, select_records) -> None:
    """Profiling builds only: int64 tensors [n_records, TRACE_SLOTS] on the GPU that receive the
    kernels' phase stamps (None, None switches them off)."""
    import torch
    n = 0
    for t in (scan_records, select_records):
        if t is not None:
            if t.dim() != 2 or t.shape[1] != TRACE_SLOTS:
                raise ValueError("trace buffers must have shape (n_records, %d)" % TRACE_SLOTS)
            n = t.shape[0] if n == 0 else n
            if t.shape[0] != n:
                raise ValueError("both trace buffers must hold the same number of records")
    rc = library().adamas_phase_trace(_ptr(scan_records, torch.int64, "scan_records", optional=True),
                                      _ptr(select_records, torch.int64, "select_records",
                                           optional=True), n)
    _check(rc, "adamas_phase_trace")


def adamas_decode_step_static(cfg: Config, q, K, V, codes, seq_start, seq_len, k: int, out,
                              max_seq_len: int, k_new=None, v_new=None, idx_out=None,
                              stream=None) -> None:
    """adamas_decode_step on the library's own static scratch array: no workspace argument."""
    import torch
    batch = q.shape[0]
    hkv, pool = cfg.num_kv_heads, cfg.pool_tokens
    rc = library().adamas_decode_step_static(
        ctypes.byref(cfg), _ptr(q, torch.bfloat16, "q", (batch, cfg.num_q_heads, cfg.head_dim)),
        _ptr(k_new, torch.bfloat16, "k_new", (batch, hkv, cfg.head_dim), optional=True),
        _ptr(v_new, torch.bfloat16, "v_new", (batch, hkv, cfg.head_dim), optional=True),
        _ptr(K, torch.bfloat16, "K", (hkv, pool, cfg.head_dim)),
        _ptr(V, torch.bfloat16, "V", (hkv, pool, cfg.head_dim)),
        _ptr(codes, torch.uint8, "codes", (hkv, pool, cfg.code_row_bytes)),
        _ptr(seq_start, torch.int64, "seq_start", (batch,)),
        _ptr(seq_len, torch.int32, "seq_len", (batch,)), batch, k,
        _ptr(out, torch.float32, "out", (batch, cfg.num_q_heads, cfg.head_dim)),
        _ptr(idx_out, torch.int32, "idx_out", (batch, cfg.num_q_heads, k), optional=True),
        max_seq_len, _stream(stream))
    _check(rc, "adamas_decode_step_static")


def adamas_decode_step_stages(cfg: Config, q, K, V, codes, seq_start, seq_len, k: int, out,
                              max_seq_len: int, workspace, k_new=None, v_new=None, idx_out=None,
                              stream=None, stages=STAGE_ALL) -> None:
    """stages=None calls the plain adamas_decode_step entry point."""
    import torch
    batch = q.shape[0]
    hkv, pool = cfg.num_kv_heads, cfg.pool_tokens
    fn = library().adamas_decode_step if stages is None else library().adamas_decode_step_stages
    extra = () if stages is None else (int(stages),)
    rc = fn(
        ctypes.byref(cfg), _ptr(q, torch.bfloat16, "q", (batch, cfg.num_q_heads, cfg.head_dim)),
        _ptr(k_new, torch.bfloat16, "k_new", (batch, hkv, cfg.head_dim), optional=True),
        _ptr(v_new, torch.bfloat16, "v_new", (batch, hkv, cfg.head_dim), optional=True),
        _ptr(K, torch.bfloat16, "K", (hkv, pool, cfg.head_dim)),
        _ptr(V, torch.bfloat16, "V", (hkv, pool, cfg.head_dim)),
        _ptr(codes, torch.uint8, "codes", (hkv, pool, cfg.code_row_bytes)),
        _ptr(seq_start, torch.int64, "seq_start", (batch,)),
        _ptr(seq_len, torch.int32, "seq_len", (batch,)), batch, k,
        _ptr(out, torch.float32, "out", (batch, cfg.num_q_heads, cfg.head_dim)),
        _ptr(idx_out, torch.int32, "idx_out", (batch, cfg.num_q_heads, k), optional=True),
        max_seq_len, _ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _stream(stream), *extra)
    _check(rc, "adamas_decode_step")
