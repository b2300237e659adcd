"""ctypes binding of the CPU oracle (adamas_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The GPU library and its Python binding never import
this package, and this package never imports them.

Every function takes and returns numpy arrays; bf16 data travels as uint16 bit
patterns.  The shared object is built on first use with gcc (see build()).
"""

from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "adamas_oracle.c"
_LIB = _HERE / "libadamas_oracle.so"

D = 128
ROW_BYTES = 32

OK, BAD_ARG, PRECONDITION, NOMEM = 0, -1, -2, -3


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc -O2 -fopenmp (scalar loops; no tuning flags)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", str(tmp), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(str(_LIB))
        for name in ("oracle_hadamard_matrix", "oracle_hadamard_transform", "oracle_bucketize",
                     "oracle_pack_row", "oracle_unpack_row", "oracle_encode", "oracle_manhattan",
                     "oracle_topk", "oracle_sparse_attention", "oracle_full_attention",
                     "oracle_decode_step", "oracle_max_threads", "oracle_encode_variant",
                     "oracle_squared_distance", "oracle_decode_step_variant",
                     "oracle_decode_step_paged", "oracle_bucketize_n", "oracle_pack_row_bits",
                     "oracle_unpack_row_bits", "oracle_encode_bits", "oracle_decode_step_bits"):
            getattr(_lib, name).restype = ctypes.c_int
        _lib.oracle_set_threads.restype = None
        _lib.oracle_sparse_attention.argtypes = [ctypes.c_void_p] * 4 + [
            ctypes.c_int32, ctypes.c_double, ctypes.c_void_p]
        _lib.oracle_full_attention.argtypes = [ctypes.c_void_p] * 3 + [
            ctypes.c_int64, ctypes.c_double, ctypes.c_void_p]
        _lib.oracle_decode_step.argtypes = [
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_double] + [ctypes.c_void_p] * 8 + [ctypes.c_int32, ctypes.c_int32] + [
            ctypes.c_void_p] * 3 + [ctypes.c_int64]
        _lib.oracle_decode_step_variant.argtypes = _lib.oracle_decode_step.argtypes + [
            ctypes.c_int, ctypes.c_int]
        _lib.oracle_decode_step_paged.argtypes = [
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_double] + [ctypes.c_void_p] * 7 + [ctypes.c_int32, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int]
        _lib.oracle_encode_bits.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                            ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                            ctypes.c_void_p]
        _lib.oracle_decode_step_bits.argtypes = [
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_double] + [ctypes.c_void_p] * 8 + [
            ctypes.c_int32, ctypes.c_int32] + [ctypes.c_void_p] * 3 + [
            ctypes.c_int64, ctypes.c_int, ctypes.c_int]
        _lib.oracle_encode_variant.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                               ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    return _lib


class OracleError(RuntimeError):
    pass


def _check(rc: int, what: str) -> None:
    if rc != OK:
        names = {BAD_ARG: "bad argument", PRECONDITION: "exactness precondition violated",
                 NOMEM: "out of memory"}
        raise OracleError("%s: %s (%d)" % (what, names.get(rc, "error"), rc))


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _thr(thr, bits: int = 2) -> np.ndarray:
    t = np.ascontiguousarray(np.asarray(thr, dtype=np.float32))
    assert t.shape == ((1 << bits) - 1,)
    return t


class head_dim:
    """`with oracle.head_dim(64): ...` runs the calls inside with d = 64 (or 96, 160, 192, 256:
    a multiple of 32 of the form 2^n, 2^n * 12 or 2^n * 20); 128 is the default and is restored on
    exit.  Process-wide state of the oracle library."""

    def __init__(self, d: int):
        self.d = int(d)

    def __enter__(self):
        global D, ROW_BYTES
        self.prev = D
        if lib().oracle_set_head_dim(ctypes.c_int(self.d)) != 0:
            raise OracleError("head dimension must be a multiple of 32 up to 256 of the form "
                              "2^n, 2^n * 12 or 2^n * 20")
        D, ROW_BYTES = self.d, self.d // 4
        return self

    def __exit__(self, *exc):
        global D, ROW_BYTES
        lib().oracle_set_head_dim(ctypes.c_int(self.prev))
        D, ROW_BYTES = self.prev, self.prev // 4
        return False


def max_threads() -> int:
    return int(lib().oracle_max_threads())


def set_threads(n: int) -> None:
    lib().oracle_set_threads(ctypes.c_int(int(n)))


def hadamard_matrix(d: int) -> np.ndarray:
    """+-1 Hadamard matrix of order d = 2^n (Sylvester, Eq. 2), 2^n * 12 or 2^n * 20 (the same
    Kronecker recursion started from Paley's matrix of order 12 / 20)."""
    H = np.empty((d, d), dtype=np.int8)
    _check(lib().oracle_hadamard_matrix(ctypes.c_int(d), _p(H)), "hadamard_matrix")
    return H


def hadamard_transform(x: np.ndarray) -> np.ndarray:
    """Unnormalised y = x H for one vector of float64 (Eq. 4, dense sums)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty_like(x)
    _check(lib().oracle_hadamard_transform(ctypes.c_int(x.shape[0]), _p(x), _p(y)),
           "hadamard_transform")
    return y


def bucketize(y: np.ndarray, thr, d: int = D) -> np.ndarray:
    """Codes 0..3 of unnormalised order-d coefficients y against orthonormal-scale thresholds
    (Eq. 5)."""
    y = np.ascontiguousarray(y, dtype=np.float64)
    code = np.empty(y.shape[0], dtype=np.uint8)
    _check(lib().oracle_bucketize(ctypes.c_int64(y.shape[0]), _p(y), ctypes.c_int(d),
                                  _p(_thr(thr)), _p(code)), "bucketize")
    return code


def pack_row(code: np.ndarray) -> np.ndarray:
    code = np.ascontiguousarray(code, dtype=np.uint8)
    assert code.shape == (D,)
    row = np.empty(ROW_BYTES, dtype=np.uint8)
    _check(lib().oracle_pack_row(_p(code), _p(row)), "pack_row")
    return row


def unpack_row(row: np.ndarray) -> np.ndarray:
    row = np.ascontiguousarray(row, dtype=np.uint8)
    assert row.shape == (ROW_BYTES,)
    code = np.empty(D, dtype=np.uint8)
    _check(lib().oracle_unpack_row(_p(row), _p(code)), "unpack_row")
    return code


def unpack_rows(rows: np.ndarray) -> np.ndarray:
    rows = np.ascontiguousarray(rows, dtype=np.uint8)
    flat = rows.reshape(-1, ROW_BYTES)
    out = np.empty((flat.shape[0], D), dtype=np.uint8)
    for i in range(flat.shape[0]):
        out[i] = unpack_row(flat[i])
    return out.reshape(rows.shape[:-1] + (D,))


def encode(x_bf16: np.ndarray, thr, hadamard: bool = True):
    """x_bf16: uint16 [..., 128].  Returns (codes uint8 [..., 128], rows uint8 [..., 32]).
    hadamard=False is the ablation that bucketizes the raw vector (Section 4.4)."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    assert x.shape[-1] == D
    n = x.size // D
    codes = np.empty(x.shape, dtype=np.uint8)
    rows = np.empty(x.shape[:-1] + (ROW_BYTES,), dtype=np.uint8)
    _check(lib().oracle_encode_variant(_p(x), ctypes.c_int64(n), _p(_thr(thr)),
                                       1 if hadamard else 0, _p(codes), _p(rows)), "encode")
    return codes, rows


def squared_distance(qcode: np.ndarray, kcodes: np.ndarray) -> np.ndarray:
    """qcode uint8 [128], kcodes uint8 [L,128] (unpacked) -> int32 [L]: sum of squared code
    differences (the L2 ablation of Section 4.4, without the monotone square root)."""
    qcode = np.ascontiguousarray(qcode, dtype=np.uint8)
    kcodes = np.ascontiguousarray(kcodes, dtype=np.uint8)
    assert qcode.shape == (D,) and kcodes.ndim == 2 and kcodes.shape[1] == D
    L = kcodes.shape[0]
    out = np.empty(L, dtype=np.int32)
    _check(lib().oracle_squared_distance(_p(qcode), _p(kcodes), ctypes.c_int64(L), _p(out)),
           "squared_distance")
    return out


def manhattan(qcode: np.ndarray, kcodes: np.ndarray) -> np.ndarray:
    """qcode uint8 [128], kcodes uint8 [L,128] (unpacked) -> int32 [L] (Eq. 6)."""
    qcode = np.ascontiguousarray(qcode, dtype=np.uint8)
    kcodes = np.ascontiguousarray(kcodes, dtype=np.uint8)
    assert qcode.shape == (D,) and kcodes.ndim == 2 and kcodes.shape[1] == D
    L = kcodes.shape[0]
    out = np.empty(L, dtype=np.int32)
    _check(lib().oracle_manhattan(_p(qcode), _p(kcodes), ctypes.c_int64(L), _p(out)), "manhattan")
    return out


def topk(dist: np.ndarray, k: int) -> np.ndarray:
    """k smallest distances, ties to the lower index; ascending indices, -1 padded."""
    dist = np.ascontiguousarray(dist, dtype=np.int32)
    idx = np.empty(k, dtype=np.int32)
    _check(lib().oracle_topk(_p(dist), ctypes.c_int64(dist.shape[0]), ctypes.c_int32(k), _p(idx)),
           "topk")
    return idx


def sparse_attention(q, K, V, idx, scale: float) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.uint16)
    K = np.ascontiguousarray(K, dtype=np.uint16)
    V = np.ascontiguousarray(V, dtype=np.uint16)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    assert q.shape == (D,) and K.shape[1] == D and V.shape == K.shape
    assert idx.size == 0 or int(idx.max()) < K.shape[0]
    out = np.empty(D, dtype=np.float32)
    _check(lib().oracle_sparse_attention(_p(q), _p(K), _p(V), _p(idx), idx.shape[0],
                                         float(scale), _p(out)), "sparse_attention")
    return out


def full_attention(q, K, V, scale: float) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.uint16)
    K = np.ascontiguousarray(K, dtype=np.uint16)
    V = np.ascontiguousarray(V, dtype=np.uint16)
    assert q.shape == (D,) and K.shape[1] == D and V.shape == K.shape
    out = np.empty(D, dtype=np.float32)
    _check(lib().oracle_full_attention(_p(q), _p(K), _p(V), K.shape[0], float(scale), _p(out)),
           "full_attention")
    return out


def decode_step(q, K, V, code_rows, seq_start, seq_len, k, thr_q, thr_k, scale,
                k_new=None, v_new=None, want_dist=False, hadamard=True, squared=False):
    """One decode step of one layer (Algorithm 1) over a ragged batch.

    q uint16 [B,Hq,128]; K, V uint16 [Hkv,pool,128] and code_rows uint8 [Hkv,pool,32] are
    UPDATED IN PLACE when k_new/v_new (uint16 [B,Hkv,128]) are given.  seq_len counts the
    appended token.  Returns (out float32 [B,Hq,128], idx int32 [B,Hq,k], dist int32
    [B,Hq,max_len] or None).  hadamard=False / squared=True select the ablation variants of
    Section 4.4 (code_rows must have been encoded with the same `hadamard`).
    """
    q = np.ascontiguousarray(q, dtype=np.uint16)
    B, Hq, _ = q.shape
    Hkv, pool, _ = K.shape
    for a, dt in ((K, np.uint16), (V, np.uint16), (code_rows, np.uint8)):
        assert a.dtype == dt and a.flags.c_contiguous
    assert V.shape == K.shape and code_rows.shape == (Hkv, pool, ROW_BYTES)
    seq_start = np.ascontiguousarray(seq_start, dtype=np.int64)
    seq_len = np.ascontiguousarray(seq_len, dtype=np.int32)
    assert seq_start.shape == (B,) and seq_len.shape == (B,)
    assert np.all(seq_start >= 0) and np.all(seq_start + seq_len <= pool)
    if k_new is not None:
        k_new = np.ascontiguousarray(k_new, dtype=np.uint16)
        v_new = np.ascontiguousarray(v_new, dtype=np.uint16)
        assert k_new.shape == (B, Hkv, D) and v_new.shape == (B, Hkv, D)
    max_len = int(seq_len.max()) if B else 0
    out = np.zeros((B, Hq, D), dtype=np.float32)
    idx = np.empty((B, Hq, k), dtype=np.int32)
    dist = np.full((B, Hq, max(max_len, 1)), -1, dtype=np.int32) if want_dist else None
    rc = lib().oracle_decode_step_variant(
        Hq, Hkv, pool, _p(_thr(thr_q)), _p(_thr(thr_k)), float(scale), _p(q), _p(k_new),
        _p(v_new), _p(K), _p(V), _p(code_rows), _p(seq_start), _p(seq_len), B, k, _p(out),
        _p(idx), _p(dist), max(max_len, 1), 1 if hadamard else 0, 1 if squared else 0)
    _check(rc, "decode_step")
    return out, idx, dist


def decode_step_paged(q, K, V, code_rows, page_table, page_tokens, seq_len, k, thr_q, thr_k, scale,
                      k_new=None, v_new=None, hadamard=True, squared=False):
    """The step on a paged cache: token t of sequence b lives in pool row
    page_table[b, t // page_tokens] * page_tokens + t % page_tokens.  K, V, code_rows are
    UPDATED IN PLACE on append.  Returns (out float32 [B,Hq,128], idx int32 [B,Hq,k])."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    B, Hq, _ = q.shape
    Hkv, pool, _ = K.shape
    for a, dt in ((K, np.uint16), (V, np.uint16), (code_rows, np.uint8)):
        assert a.dtype == dt and a.flags.c_contiguous
    page_table = np.ascontiguousarray(page_table, dtype=np.int32)
    seq_len = np.ascontiguousarray(seq_len, dtype=np.int32)
    assert page_table.ndim == 2 and page_table.shape[0] == B and seq_len.shape == (B,)
    if k_new is not None:
        k_new = np.ascontiguousarray(k_new, dtype=np.uint16)
        v_new = np.ascontiguousarray(v_new, dtype=np.uint16)
    out = np.zeros((B, Hq, D), dtype=np.float32)
    idx = np.empty((B, Hq, k), dtype=np.int32)
    rc = lib().oracle_decode_step_paged(
        Hq, Hkv, pool, _p(_thr(thr_q)), _p(_thr(thr_k)), float(scale), _p(q), _p(k_new),
        _p(v_new), _p(K), _p(V), _p(code_rows), _p(page_table), page_table.shape[1],
        int(page_tokens), _p(seq_len), B, k, _p(out), _p(idx), 1 if hadamard else 0,
        1 if squared else 0)
    _check(rc, "decode_step_paged")
    return out, idx


# ------------------------------------------------ bucketization ablation: 1-, 2-, 3-bit codes

def bucketize_n(y: np.ndarray, thr, d: int = D) -> np.ndarray:
    """Eq. 5 with len(thr) thresholds (1, 3 or 7)."""
    y = np.ascontiguousarray(y, dtype=np.float64)
    t = np.ascontiguousarray(np.asarray(thr, dtype=np.float32))
    code = np.empty(y.shape[0], dtype=np.uint8)
    _check(lib().oracle_bucketize_n(ctypes.c_int64(y.shape[0]), _p(y), ctypes.c_int(d), _p(t),
                                    ctypes.c_int(t.shape[0]), _p(code)), "bucketize_n")
    return code


def pack_row_bits(code: np.ndarray, bits: int) -> np.ndarray:
    code = np.ascontiguousarray(code, dtype=np.uint8)
    assert code.shape == (D,)
    row = np.empty((D // 8) * bits, dtype=np.uint8)
    _check(lib().oracle_pack_row_bits(_p(code), ctypes.c_int(bits), _p(row)), "pack_row_bits")
    return row


def unpack_row_bits(row: np.ndarray, bits: int) -> np.ndarray:
    row = np.ascontiguousarray(row, dtype=np.uint8)
    assert row.shape == ((D // 8) * bits,)
    code = np.empty(D, dtype=np.uint8)
    _check(lib().oracle_unpack_row_bits(_p(row), ctypes.c_int(bits), _p(code)), "unpack_row_bits")
    return code


def unpack_rows_bits(rows: np.ndarray, bits: int) -> np.ndarray:
    rows = np.ascontiguousarray(rows, dtype=np.uint8)
    flat = rows.reshape(-1, (D // 8) * bits)
    out = np.empty((flat.shape[0], D), dtype=np.uint8)
    for i in range(flat.shape[0]):
        out[i] = unpack_row_bits(flat[i], bits)
    return out.reshape(rows.shape[:-1] + (D,))


def encode_bits(x_bf16: np.ndarray, thr, bits: int, hadamard: bool = True):
    """x_bf16 uint16 [..., 128] -> (codes uint8 [..., 128] in 0..2^bits-1, rows uint8
    [..., 16*bits]); thr holds 2^bits - 1 thresholds."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    assert x.shape[-1] == D
    n = x.size // D
    codes = np.empty(x.shape, dtype=np.uint8)
    rows = np.empty(x.shape[:-1] + ((D // 8) * bits,), dtype=np.uint8)
    _check(lib().oracle_encode_bits(_p(x), ctypes.c_int64(n), _p(_thr(thr, bits)), bits,
                                    1 if hadamard else 0, _p(codes), _p(rows)), "encode_bits")
    return codes, rows


def decode_step_bits(q, K, V, code_rows, seq_start, seq_len, k, thr_q, thr_k, bits, scale,
                     k_new=None, v_new=None, want_dist=False, hadamard=True):
    """decode_step with `bits`-bit codes: code_rows uint8 [Hkv,pool,16*bits]."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    B, Hq, _ = q.shape
    Hkv, pool, _ = K.shape
    for a, dt in ((K, np.uint16), (V, np.uint16), (code_rows, np.uint8)):
        assert a.dtype == dt and a.flags.c_contiguous
    assert V.shape == K.shape and code_rows.shape == (Hkv, pool, (D // 8) * bits)
    seq_start = np.ascontiguousarray(seq_start, dtype=np.int64)
    seq_len = np.ascontiguousarray(seq_len, dtype=np.int32)
    assert np.all(seq_start >= 0) and np.all(seq_start + seq_len <= pool)
    if k_new is not None:
        k_new = np.ascontiguousarray(k_new, dtype=np.uint16)
        v_new = np.ascontiguousarray(v_new, dtype=np.uint16)
    max_len = int(seq_len.max()) if B else 0
    out = np.zeros((B, Hq, D), dtype=np.float32)
    idx = np.empty((B, Hq, k), dtype=np.int32)
    dist = np.full((B, Hq, max(max_len, 1)), -1, dtype=np.int32) if want_dist else None
    rc = lib().oracle_decode_step_bits(
        Hq, Hkv, pool, _p(_thr(thr_q, bits)), _p(_thr(thr_k, bits)), bits, float(scale), _p(q),
        _p(k_new), _p(v_new), _p(K), _p(V), _p(code_rows), _p(seq_start), _p(seq_len), B, k,
        _p(out), _p(idx), _p(dist), max(max_len, 1), 1 if hadamard else 0, 0)
    _check(rc, "decode_step_bits")
    return out, idx, dist
