"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Loads ``oracle/liboracle.so`` (built from ``swiftprune_oracle.c`` by
:func:`build`) and exposes its functions on numpy arrays.  bf16 tensors are
numpy ``uint16`` arrays holding the raw bits; fp32 tensors are ``float32``,
IEEE half tensors ``float16``.

Only the tests, the smoke check and the CPU-baseline leg of the benchmark may
import this package.  It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "swiftprune_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

F32, BF16, F16 = 0, 1, 2

CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c11", "-Wall", "-Wextra",
          "-shared", "-fPIC"]


def build(extra_flags=(), out_path: str | None = None) -> str:
    """Compile the oracle with gcc; returns the path of the shared object."""
    out_path = out_path or _LIB
    cmd = ["gcc", *CFLAGS, *extra_flags, _SRC, "-o", out_path, "-lm"]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return out_path


_lib = None


def _stale() -> bool:
    if not os.path.exists(_LIB):
        return True
    t = os.path.getmtime(_LIB)
    return any(os.path.getmtime(os.path.join(_HERE, f)) > t
               for f in ("swiftprune_oracle.c", "ewma_body.inc"))


def lib(path: str | None = None) -> C.CDLL:
    """The loaded oracle library (built on first use if missing or out of date)."""
    global _lib
    if path is not None:
        return _declare(C.CDLL(path))
    if _lib is None:
        if _stale():
            build()
        _lib = _declare(C.CDLL(_LIB))
    return _lib


_vp, _i64, _i32, _f, _d = C.c_void_p, C.c_int64, C.c_int, C.c_float, C.c_double


def _declare(L: C.CDLL) -> C.CDLL:
    L.oracle_stats_accumulate.argtypes = [_vp, _i64, _i64, _i64, _i32, _vp]
    L.oracle_stats_accumulate_partials.argtypes = [_vp, _i64, _i64, _i64, _vp]
    L.oracle_stats_finalize.argtypes = [_vp, _i64, _vp, _vp]
    L.oracle_channel_factor_f32.argtypes = [_vp, _f, _i64, _vp]
    L.oracle_channel_factor_f64.argtypes = [_vp, _i64, _vp]
    L.oracle_score_f32.argtypes = [_vp, _i64, _i64, _i64, _i32, _vp, _vp]
    L.oracle_score_f64.argtypes = [_vp, _i64, _i64, _i64, _i32, _vp, _vp]
    L.oracle_ewma_row_f32.argtypes = [_vp, _i64, _f, _f, _f, _vp, _vp, _vp]
    L.oracle_ewma_row_f64.argtypes = [_vp, _i64, _d, _d, _d, _vp, _vp, _vp]
    L.oracle_ewma_select_f32.argtypes = [_vp, _i64, _i64, _i64, _i32, _vp, _f, _f, _f, _vp, _vp, _vp]
    L.oracle_ewma_select_f64.argtypes = [_vp, _i64, _i64, _i64, _i32, _vp, _d, _d, _d, _vp, _vp, _vp]
    L.oracle_nm_select_f32.argtypes = [_vp, _i64, _i64, _i64, _i32, _vp, _i32, _i32, _vp, _vp]
    L.oracle_nm_select_f64.argtypes = [_vp, _i64, _i64, _i64, _i32, _vp, _i32, _i32, _vp, _vp]
    L.oracle_ewma_select_literal_f32.argtypes = [_vp, _i64, _i64, _i64, _i32, _vp, _f, _f, _f, _f,
                                                 _vp, _vp, _vp, _vp, _vp]
    L.oracle_topk_select_f32.argtypes = [_vp, _i64, _i64, _i64, _i32, _vp, _vp, _i64, _vp]
    L.oracle_compact_nm.argtypes = [_vp, _i64, _i64, _i64, _i32, _vp, _i32, _i32, _vp, _vp]
    L.oracle_expand_nm.argtypes = [_vp, _vp, _i64, _i64, _i32, _i32, _i32, _vp]
    L.oracle_apply.argtypes = [_vp, _i64, _i64, _i64, _i32, _vp]
    for name in ("oracle_stats_accumulate", "oracle_stats_accumulate_partials", "oracle_stats_finalize", "oracle_channel_factor_f32",
                 "oracle_channel_factor_f64", "oracle_score_f32", "oracle_score_f64",
                 "oracle_ewma_row_f32", "oracle_ewma_row_f64", "oracle_ewma_select_f32",
                 "oracle_ewma_select_f64", "oracle_nm_select_f32", "oracle_nm_select_f64",
                 "oracle_ewma_select_literal_f32", "oracle_topk_select_f32", "oracle_compact_nm", "oracle_expand_nm", "oracle_apply"):
        getattr(L, name).restype = None
    return L


# ---------------------------------------------------------------- helpers
def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float16:
        return F16
    raise TypeError(f"tensor must be float32, float16 or uint16 (bf16 bits), got {a.dtype}")


def _mat(a: np.ndarray):
    """(pointer, rows, cols, pitch-in-elements, dtype code) of a 2-D row-major view."""
    if a.ndim != 2 or a.strides[1] != a.itemsize or a.strides[0] % a.itemsize:
        raise ValueError("expected a 2-D array with unit column stride")
    return a.ctypes.data, a.shape[0], a.shape[1], a.strides[0] // a.itemsize, _dtype_code(a)


def _p(a):
    return None if a is None else a.ctypes.data


def _real(precision: str):
    if precision == "f32":
        return np.float32, "_f32"
    if precision == "f64":
        return np.float64, "_f64"
    raise ValueError(precision)


# ---------------------------------------------------------------- step 1
def stats_accumulate(X: np.ndarray, acc: np.ndarray | None = None, L=None) -> np.ndarray:
    """acc[q] += sum_t X[t,q]^2 in double; returns acc (created when None)."""
    ptr, tokens, n, ld, dt = _mat(X)
    if acc is None:
        acc = np.zeros(n, dtype=np.float64)
    assert acc.dtype == np.float64 and acc.shape == (n,) and acc.flags.c_contiguous
    (L or lib()).oracle_stats_accumulate(ptr, tokens, n, ld, dt, acc.ctypes.data)
    return acc


def stats_accumulate_partials(P: np.ndarray, acc: np.ndarray | None = None, L=None) -> np.ndarray:
    """acc[q] += sum_p P[p,q] in double, P float32 [parts, in] (row pitch allowed): the sums of squares that the
    producer of X formed over its own pieces of the tokens.  Returns acc (created when None)."""
    assert P.dtype == np.float32 and P.ndim == 2 and P.strides[1] == 4 and P.strides[0] % 4 == 0
    parts, n = P.shape
    if acc is None:
        acc = np.zeros(n, dtype=np.float64)
    assert acc.dtype == np.float64 and acc.shape == (n,) and acc.flags.c_contiguous
    (L or lib()).oracle_stats_accumulate_partials(P.ctypes.data, parts, n, P.strides[0] // 4, acc.ctypes.data)
    return acc


def stats_finalize(acc: np.ndarray, L=None):
    """(xsq float32[in], S float32 scalar) from the double accumulators."""
    n = acc.shape[0]
    xsq = np.empty(n, dtype=np.float32)
    S = np.empty(1, dtype=np.float32)
    (L or lib()).oracle_stats_finalize(acc.ctypes.data, n, xsq.ctypes.data, S.ctypes.data)
    return xsq, S[0]


def channel_factor_f32(xsq: np.ndarray, S, L=None) -> np.ndarray:
    xsq = np.ascontiguousarray(xsq, dtype=np.float32)
    hr = np.empty_like(xsq)
    (L or lib()).oracle_channel_factor_f32(xsq.ctypes.data, float(np.float32(S)), xsq.shape[0],
                                           hr.ctypes.data)
    return hr


def channel_factor_f64(acc: np.ndarray, L=None) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.float64)
    hr = np.empty_like(acc)
    (L or lib()).oracle_channel_factor_f64(acc.ctypes.data, acc.shape[0], hr.ctypes.data)
    return hr


def layer_stats(X: np.ndarray, L=None):
    """Whole of step 1 in float outputs: (xsq, S, hr)."""
    acc = stats_accumulate(X, L=L)
    xsq, S = stats_finalize(acc, L=L)
    return xsq, S, channel_factor_f32(xsq, S, L=L)


# ---------------------------------------------------------------- steps 2-4
def score(W: np.ndarray, hr: np.ndarray, precision: str = "f32", L=None) -> np.ndarray:
    ptr, out, n, ld, dt = _mat(W)
    real, sfx = _real(precision)
    hr = np.ascontiguousarray(hr, dtype=real)
    assert hr.shape == (n,)
    scores = np.empty((out, n), dtype=real)
    getattr(L or lib(), "oracle_score" + sfx)(ptr, out, n, ld, dt, hr.ctypes.data, scores.ctypes.data)
    return scores


def ewma_row(Lrow: np.ndarray, alpha, beta, la, precision: str = "f32", L=None):
    """EWMA walk over one row of scores: (prune uint8[n], est[n], dev[n]) (state after each element)."""
    real, sfx = _real(precision)
    Lrow = np.ascontiguousarray(Lrow, dtype=real)
    n = Lrow.shape[0]
    prune = np.zeros(n, dtype=np.uint8)
    est = np.empty(n, dtype=real)
    dev = np.empty(n, dtype=real)
    getattr(L or lib(), "oracle_ewma_row" + sfx)(Lrow.ctypes.data, n, float(alpha), float(beta),
                                                 float(la), prune.ctypes.data, est.ctypes.data,
                                                 dev.ctypes.data)
    return prune, est, dev


def ewma_select(W: np.ndarray, hr: np.ndarray, alpha, beta, la, precision: str = "f32",
                want_scores: bool = False, L=None):
    """Unstructured selection: (keep_mask uint32[out, ceil(in/32)], row_pruned int32[out], scores|None)."""
    ptr, out, n, ld, dt = _mat(W)
    real, sfx = _real(precision)
    hr = np.ascontiguousarray(hr, dtype=real)
    assert hr.shape == (n,)
    mask = np.empty((out, (n + 31) // 32), dtype=np.uint32)
    cnt = np.empty(out, dtype=np.int32)
    sc = np.empty((out, n), dtype=real) if want_scores else None
    getattr(L or lib(), "oracle_ewma_select" + sfx)(ptr, out, n, ld, dt, hr.ctypes.data, float(alpha),
                                                    float(beta), float(la), mask.ctypes.data,
                                                    cnt.ctypes.data, _p(sc))
    return mask, cnt, sc


def ewma_select_literal(W: np.ndarray, xsq: np.ndarray, S, alpha, beta, la, details: bool = False, L=None):
    """Algorithm 1 as printed (S updated when pruning): (keep_mask, row_pruned, n_effective_S_updates);
    with details also (scores float32[out, in], S of every row after its last element)."""
    ptr, out, n, ld, dt = _mat(W)
    xsq = np.ascontiguousarray(xsq, dtype=np.float32)
    mask = np.empty((out, (n + 31) // 32), dtype=np.uint32)
    cnt = np.empty(out, dtype=np.int32)
    eff = np.zeros(1, dtype=np.int64)
    sc = np.empty((out, n), dtype=np.float32) if details else None
    S_rows = np.empty(out, dtype=np.float32) if details else None
    (L or lib()).oracle_ewma_select_literal_f32(ptr, out, n, ld, dt, xsq.ctypes.data,
                                                float(np.float32(S)), float(alpha), float(beta),
                                                float(la), mask.ctypes.data, cnt.ctypes.data,
                                                eff.ctypes.data, _p(sc), _p(S_rows))
    if details:
        return mask, cnt, int(eff[0]), sc, S_rows
    return mask, cnt, int(eff[0])


def nm_select(W: np.ndarray, hr: np.ndarray, n_keep: int, m_group: int, precision: str = "f32",
              want_scores: bool = False, L=None):
    """N:M selection: (keep_mask, scores|None).  Requires in % m_group == 0."""
    ptr, out, n, ld, dt = _mat(W)
    if n % m_group or not (0 < n_keep < m_group):
        raise ValueError("in must be a multiple of m_group and 0 < n_keep < m_group")
    real, sfx = _real(precision)
    hr = np.ascontiguousarray(hr, dtype=real)
    mask = np.empty((out, (n + 31) // 32), dtype=np.uint32)
    sc = np.empty((out, n), dtype=real) if want_scores else None
    getattr(L or lib(), "oracle_nm_select" + sfx)(ptr, out, n, ld, dt, hr.ctypes.data, n_keep, m_group,
                                                  mask.ctypes.data, _p(sc))
    return mask, sc


def topk_select(W: np.ndarray, hr: np.ndarray, k, L=None) -> np.ndarray:
    """Exact sort-based selection: prune the k smallest scores of every row (k: int or int32[out])."""
    ptr, out, n, ld, dt = _mat(W)
    hr = np.ascontiguousarray(hr, dtype=np.float32)
    mask = np.empty((out, (n + 31) // 32), dtype=np.uint32)
    if np.isscalar(k):
        kp, ku = None, int(k)
    else:
        karr = np.ascontiguousarray(k, dtype=np.int32)
        assert karr.shape == (out,)
        kp, ku = karr.ctypes.data, 0
    (L or lib()).oracle_topk_select_f32(ptr, out, n, ld, dt, hr.ctypes.data, kp, ku, mask.ctypes.data)
    return mask


def nm_meta_words(n: int, n_keep: int, m_group: int) -> int:
    bits = 2 if m_group == 4 else 4
    return (n // m_group * n_keep * bits + 31) // 32


def compact_nm(W: np.ndarray, keep_mask: np.ndarray, n_keep: int, m_group: int, L=None):
    """(values [out, in/M*N] in W's dtype, meta uint32 [out, meta_words]) of an N:M-masked matrix."""
    ptr, out, n, ld, dt = _mat(W)
    keep_mask = np.ascontiguousarray(keep_mask, dtype=np.uint32)
    values = np.empty((out, n // m_group * n_keep), dtype=W.dtype)
    meta = np.empty((out, nm_meta_words(n, n_keep, m_group)), dtype=np.uint32)
    (L or lib()).oracle_compact_nm(ptr, out, n, ld, dt, keep_mask.ctypes.data, n_keep, m_group,
                                   values.ctypes.data, meta.ctypes.data)
    return values, meta


def expand_nm(values: np.ndarray, meta: np.ndarray, n: int, n_keep: int, m_group: int, L=None) -> np.ndarray:
    """Dense [out, n] matrix from the compact form."""
    values = np.ascontiguousarray(values)
    meta = np.ascontiguousarray(meta, dtype=np.uint32)
    out = values.shape[0]
    W = np.empty((out, n), dtype=values.dtype)
    (L or lib()).oracle_expand_nm(values.ctypes.data, meta.ctypes.data, out, n, _dtype_code(values),
                                  n_keep, m_group, W.ctypes.data)
    return W


# ---------------------------------------------------------------- step 5
def apply(W: np.ndarray, keep_mask: np.ndarray, L=None) -> np.ndarray:
    """Zero the pruned entries of W in place; returns W."""
    ptr, out, n, ld, dt = _mat(W)
    keep_mask = np.ascontiguousarray(keep_mask, dtype=np.uint32)
    assert keep_mask.shape == (out, (n + 31) // 32)
    (L or lib()).oracle_apply(ptr, out, n, ld, dt, keep_mask.ctypes.data)
    return W


def unpack_mask(keep_mask: np.ndarray, n: int) -> np.ndarray:
    """bool[out, n] view of a bit-packed keep mask (format helper, no method arithmetic)."""
    bits = np.unpackbits(keep_mask.view(np.uint8), axis=1, bitorder="little")
    return bits[:, :n].astype(bool)
