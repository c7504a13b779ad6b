"""ctypes binding of libswiftprune.so: argument marshalling only.

Each function has the name and the argument order of its C entry point
(include/swiftprune.h) and takes torch tensors living on the GPU; torch is used
for device memory and for the current stream, nothing else.  Every step of the
path runs in the HIP kernels.  There is no fallback: a missing library raises
at first use.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libswiftprune.so")

SP_F32, SP_BF16, SP_F16 = 0, 1, 2
SP_OK, SP_EINVAL, SP_ENOSPC, SP_EHIP, SP_ERANGE = 0, -1, -2, -3, -4
SP_SEQUENTIAL_ORDER, SP_APPLY_INPLACE = 1, 2

EXPORTS = ("swiftprune_layer_stats", "swiftprune_layer_stats_static", "swiftprune_score_select", "swiftprune_nm_select",
           "swiftprune_apply", "swiftprune_score_select_group", "swiftprune_nm_select_group", "swiftprune_channel_factor", "swiftprune_layer_stats_from_partials", "swiftprune_ewma_trace", "swiftprune_count_pruned", "swiftprune_calibrate_la", "swiftprune_calibrate_la_device", "swiftprune_la_workspace_bytes", "swiftprune_score_select_la", "swiftprune_topk_select", "swiftprune_compact_nm", "swiftprune_expand_nm", "swiftprune_nm_meta_words", "swiftprune_la_for_sparsity", "swiftprune_stats_workspace_bytes",
           "swiftprune_strerror", "swiftprune_version")


class SwiftPruneError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {swiftprune_strerror(code)} ({code})")


class sp_ewma_params(C.Structure):
    _fields_ = [("alpha", C.c_float), ("beta", C.c_float), ("la", C.c_float)]


class sp_matrix(C.Structure):
    _fields_ = [("W", C.c_void_p), ("out", C.c_int64), ("ldw", C.c_int64), ("keep_mask", C.c_void_p),
                ("row_pruned", C.c_void_p)]


SP_MAX_GROUP = 8


_lib = None


def load_library(path: str | None = None) -> C.CDLL:
    """Load the C-ABI library (no build is attempted here)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise ImportError(f"{p} is missing: build it with `python -m paper_2501_16376_amd.build` "
                          "(or __graft_entry__.build()); there is no CPU fallback")
    L = C.CDLL(p)
    vp, i64, i32, u32, f = C.c_void_p, C.c_int64, C.c_int, C.c_uint32, C.c_float
    L.swiftprune_layer_stats.argtypes = [vp, i64, i64, i64, i32, vp, vp, vp, i32, i32, vp, C.c_size_t, vp]
    L.swiftprune_layer_stats.restype = i32
    L.swiftprune_layer_stats_static.argtypes = [vp, i64, i64, i64, i32, vp, vp, vp, i32, i32, vp]
    L.swiftprune_layer_stats_static.restype = i32
    L.swiftprune_score_select.argtypes = [vp, i64, i64, i64, i32, vp, f, C.POINTER(sp_ewma_params),
                                          vp, vp, vp, u32, vp]
    L.swiftprune_score_select.restype = i32
    L.swiftprune_score_select_group.argtypes = [C.POINTER(sp_matrix), i32, i64, i32, vp, f,
                                                C.POINTER(sp_ewma_params), u32, vp]
    L.swiftprune_score_select_group.restype = i32
    L.swiftprune_nm_select_group.argtypes = [C.POINTER(sp_matrix), i32, i64, i32, vp, i32, i32, u32, vp]
    L.swiftprune_nm_select_group.restype = i32
    L.swiftprune_nm_select.argtypes = [vp, i64, i64, i64, i32, vp, i32, i32, vp, vp, u32, vp]
    L.swiftprune_nm_select.restype = i32
    L.swiftprune_apply.argtypes = [vp, i64, i64, i64, i32, vp, vp]
    L.swiftprune_apply.restype = i32
    L.swiftprune_channel_factor.argtypes = [vp, vp, i64, vp, vp]
    L.swiftprune_channel_factor.restype = i32
    L.swiftprune_layer_stats_from_partials.argtypes = [vp, i64, i64, i64, vp, vp, vp, i32, i32, vp]
    L.swiftprune_layer_stats_from_partials.restype = i32
    L.swiftprune_ewma_trace.argtypes = [vp, i64, i64, i64, i32, vp, f, f, vp, vp, vp]
    L.swiftprune_ewma_trace.restype = i32
    L.swiftprune_count_pruned.argtypes = [vp, i64, i64, i64, i32, vp, f, f, C.POINTER(C.c_float), i32, vp, vp]
    L.swiftprune_count_pruned.restype = i32
    L.swiftprune_calibrate_la.argtypes = [vp, i64, i64, i64, i32, vp, f, f, f, f, f, f, vp,
                                          C.POINTER(C.c_float), C.POINTER(C.c_float), vp]
    L.swiftprune_calibrate_la.restype = i32
    L.swiftprune_la_workspace_bytes.argtypes = []
    L.swiftprune_la_workspace_bytes.restype = C.c_size_t
    L.swiftprune_calibrate_la_device.argtypes = [vp, i64, i64, i64, i32, vp, f, f, f, vp, C.c_size_t, vp, vp, vp, vp]
    L.swiftprune_calibrate_la_device.restype = i32
    L.swiftprune_score_select_la.argtypes = [vp, i64, i64, i64, i32, vp, f, f, vp, vp, vp, u32, vp]
    L.swiftprune_score_select_la.restype = i32
    L.swiftprune_topk_select.argtypes = [vp, i64, i64, i64, i32, vp, vp, i64, vp, u32, vp]
    L.swiftprune_topk_select.restype = i32
    L.swiftprune_compact_nm.argtypes = [vp, i64, i64, i64, i32, vp, i32, i32, vp, vp, vp]
    L.swiftprune_compact_nm.restype = i32
    L.swiftprune_expand_nm.argtypes = [vp, vp, i64, i64, i32, i32, i32, vp, i64, vp]
    L.swiftprune_expand_nm.restype = i32
    L.swiftprune_nm_meta_words.argtypes = [i64, i32, i32]
    L.swiftprune_nm_meta_words.restype = C.c_size_t
    L.swiftprune_la_for_sparsity.argtypes = [f, C.POINTER(C.c_float)]
    L.swiftprune_la_for_sparsity.restype = i32
    L.swiftprune_stats_workspace_bytes.argtypes = [i64, i64]
    L.swiftprune_stats_workspace_bytes.restype = C.c_size_t
    L.swiftprune_strerror.argtypes = [i32]
    L.swiftprune_strerror.restype = C.c_char_p
    L.swiftprune_version.argtypes = []
    L.swiftprune_version.restype = C.c_char_p
    if path is None:
        _lib = L
    return L


# ------------------------------------------------------------------ marshalling helpers
def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return SP_BF16
    if t.dtype == torch.float32:
        return SP_F32
    if t.dtype == torch.float16:
        return SP_F16
    raise TypeError(f"tensor must be bfloat16, float16 or float32, got {t.dtype}")


def _matrix(t):
    """(pointer, rows, cols, pitch in elements, dtype code) of a 2-D device tensor with unit column stride."""
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("expected a 2-D tensor with unit column stride")
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU (there is no CPU path)")
    return t.data_ptr(), t.shape[0], t.shape[1], t.stride(0), _dtype_code(t)


def _vec(t, dtype, n, name):
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous() or t.numel() < n:
        raise ValueError(f"{name}: expected a contiguous {dtype} GPU tensor with at least {n} elements")
    return t.data_ptr()


def _stream(stream):
    import torch
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _check(code: int, where: str):
    if code != SP_OK:
        raise SwiftPruneError(code, where)


# ------------------------------------------------------------------ host helpers
def swiftprune_version() -> str:
    return load_library().swiftprune_version().decode()


def swiftprune_strerror(code: int) -> str:
    return load_library().swiftprune_strerror(int(code)).decode()


def swiftprune_la_for_sparsity(sparsity: float) -> float:
    la = C.c_float()
    _check(load_library().swiftprune_la_for_sparsity(float(sparsity), C.byref(la)),
           "swiftprune_la_for_sparsity")
    return la.value


def swiftprune_stats_workspace_bytes(tokens: int, n_in: int) -> int:
    return int(load_library().swiftprune_stats_workspace_bytes(int(tokens), int(n_in)))


# ------------------------------------------------------------------ entry points
def swiftprune_layer_stats(X, xsq, S, hr, accumulate: bool = False, finalize: bool = True,
                           workspace=None, stream=None):
    """X[tokens, in] -> xsq[in], S[1], hr[in] (all fp32 GPU tensors, written in place)."""
    import torch
    ptr, tokens, n_in, ldx, dt = _matrix(X)
    need = swiftprune_stats_workspace_bytes(tokens, n_in)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    code = load_library().swiftprune_layer_stats(
        ptr, tokens, n_in, ldx, dt, _vec(xsq, torch.float32, n_in, "xsq"),
        _vec(S, torch.float32, 1, "S"), _vec(hr, torch.float32, n_in, "hr"),
        int(bool(accumulate)), int(bool(finalize)), workspace.data_ptr(),
        workspace.numel() * workspace.element_size(), _stream(stream))
    _check(code, "swiftprune_layer_stats")
    return workspace


def swiftprune_layer_stats_static(X, xsq, S, hr, accumulate: bool = False, finalize: bool = True, stream=None):
    """swiftprune_layer_stats with the partial sums in the library's own device array (no workspace)."""
    import torch
    ptr, tokens, n_in, ldx, dt = _matrix(X)
    code = load_library().swiftprune_layer_stats_static(
        ptr, tokens, n_in, ldx, dt, _vec(xsq, torch.float32, n_in, "xsq"),
        _vec(S, torch.float32, 1, "S"), _vec(hr, torch.float32, n_in, "hr"),
        int(bool(accumulate)), int(bool(finalize)), _stream(stream))
    _check(code, "swiftprune_layer_stats_static")


def swiftprune_channel_factor(xsq, S, hr, stream=None):
    """hr[q] = 1/2 / (1 - xsq[q]/S) from given statistics (fp32 GPU tensors; hr is written)."""
    import torch
    n_in = xsq.numel()
    code = load_library().swiftprune_channel_factor(
        _vec(xsq, torch.float32, n_in, "xsq"), _vec(S, torch.float32, 1, "S"), n_in,
        _vec(hr, torch.float32, n_in, "hr"), _stream(stream))
    _check(code, "swiftprune_channel_factor")


def swiftprune_layer_stats_from_partials(partials, xsq, S, hr=None, accumulate: bool = False, finalize: bool = True,
                                         stream=None):
    """Step 1 from partials[parts, in] (fp32 GPU tensor, unit column stride): per-piece sums of X^2 that the
    producer of X formed over its own share of the tokens.  Writes xsq, S and (finalize) hr."""
    import torch
    ptr, parts, n_in, ld, dt = _matrix(partials)
    if dt != SP_F32:
        raise ValueError("partials must be float32")
    code = load_library().swiftprune_layer_stats_from_partials(
        ptr, parts, n_in, ld, _vec(xsq, torch.float32, n_in, "xsq"), _vec(S, torch.float32, 1, "S"),
        _vec(hr, torch.float32, n_in, "hr"), int(bool(accumulate)), int(bool(finalize)), _stream(stream))
    _check(code, "swiftprune_layer_stats_from_partials")


def swiftprune_score_select(W, hr, keep_mask, sparsity: float = 0.5, alpha: float = 0.125,
                            beta: float = 0.125, la: float | None = None, row_pruned=None,
                            scores=None, flags: int = 0, stream=None):
    """EWMA selection of W[out, in]; keep_mask is int32/uint32 [out, ceil(in/32)]."""
    import torch
    ptr, out, n_in, ldw, dt = _matrix(W)
    words = (n_in + 31) // 32
    params = sp_ewma_params(float(alpha), float(beta), float("nan") if la is None else float(la))
    code = load_library().swiftprune_score_select(
        ptr, out, n_in, ldw, dt, _vec(hr, torch.float32, n_in, "hr"), float(sparsity),
        C.byref(params), _vec(keep_mask, torch.int32, out * words, "keep_mask"),
        _vec(row_pruned, torch.int32, out, "row_pruned"),
        _vec(scores, torch.float32, out * n_in, "scores"), int(flags), _stream(stream))
    _check(code, "swiftprune_score_select")


def swiftprune_nm_select(W, hr, n_keep: int, m_group: int, keep_mask, scores=None, flags: int = 0,
                         stream=None):
    import torch
    ptr, out, n_in, ldw, dt = _matrix(W)
    words = (n_in + 31) // 32
    code = load_library().swiftprune_nm_select(
        ptr, out, n_in, ldw, dt, _vec(hr, torch.float32, n_in, "hr"), int(n_keep), int(m_group),
        _vec(keep_mask, torch.int32, out * words, "keep_mask"),
        _vec(scores, torch.float32, out * n_in, "scores"), int(flags), _stream(stream))
    _check(code, "swiftprune_nm_select")


def _group(Ws, keep_masks, row_pruned):
    """Marshals a list of matrices into an sp_matrix array: (array, n, columns, dtype code)."""
    import torch
    n = len(Ws)
    if not 1 <= n <= SP_MAX_GROUP or len(keep_masks) != n or (row_pruned is not None and len(row_pruned) != n):
        raise ValueError(f"a group holds 1..{SP_MAX_GROUP} matrices with one mask (and count vector) each")
    arr = (sp_matrix * n)()
    n_in, dt = None, None
    for j, W in enumerate(Ws):
        ptr, out, cols, ldw, code = _matrix(W)
        if n_in is None:
            n_in, dt = cols, code
        elif (cols, code) != (n_in, dt):
            raise ValueError("the matrices of a group share the number of columns and the dtype")
        words = (cols + 31) // 32
        arr[j] = sp_matrix(ptr, out, ldw, _vec(keep_masks[j], torch.int32, out * words, "keep_mask"),
                           None if row_pruned is None else _vec(row_pruned[j], torch.int32, out, "row_pruned"))
    return arr, n, n_in, dt


def swiftprune_score_select_group(Ws, hr, keep_masks, sparsity: float = 0.5, alpha: float = 0.125,
                                  beta: float = 0.125, la: float | None = None, row_pruned=None, flags: int = 0,
                                  stream=None):
    """EWMA selection of several matrices that share one layer input (one hr) in one launch."""
    import torch
    arr, n, n_in, dt = _group(Ws, keep_masks, row_pruned)
    params = sp_ewma_params(float(alpha), float(beta), float("nan") if la is None else float(la))
    code = load_library().swiftprune_score_select_group(
        arr, n, n_in, dt, _vec(hr, torch.float32, n_in, "hr"), float(sparsity), C.byref(params), int(flags),
        _stream(stream))
    _check(code, "swiftprune_score_select_group")


def swiftprune_nm_select_group(Ws, hr, n_keep: int, m_group: int, keep_masks, flags: int = 0, stream=None):
    """N:M selection of several matrices that share one layer input (one hr) in one launch."""
    import torch
    arr, n, n_in, dt = _group(Ws, keep_masks, None)
    code = load_library().swiftprune_nm_select_group(
        arr, n, n_in, dt, _vec(hr, torch.float32, n_in, "hr"), int(n_keep), int(m_group), int(flags),
        _stream(stream))
    _check(code, "swiftprune_nm_select_group")


def swiftprune_ewma_trace(W, hr, est=None, dev=None, alpha: float = 0.125, beta: float = 0.125, stream=None):
    """est[out, in], dev[out, in] (fp32 GPU tensors, either may be None) = EWMA state after each weight."""
    import torch
    ptr, out, n_in, ldw, dt = _matrix(W)
    code = load_library().swiftprune_ewma_trace(
        ptr, out, n_in, ldw, dt, _vec(hr, torch.float32, n_in, "hr"), float(alpha), float(beta),
        _vec(est, torch.float32, out * n_in, "est"), _vec(dev, torch.float32, out * n_in, "dev"),
        _stream(stream))
    _check(code, "swiftprune_ewma_trace")


def swiftprune_count_pruned(W, hr, la_candidates, counts, alpha: float = 0.125, beta: float = 0.125,
                            stream=None):
    """counts[i] (int64 GPU tensor, >= len(la_candidates)) = weights pruned with la_candidates[i]."""
    import torch
    ptr, out, n_in, ldw, dt = _matrix(W)
    n = len(la_candidates)
    arr = (C.c_float * n)(*[float(x) for x in la_candidates])
    code = load_library().swiftprune_count_pruned(
        ptr, out, n_in, ldw, dt, _vec(hr, torch.float32, n_in, "hr"), float(alpha), float(beta), arr, n,
        _vec(counts, torch.int64, n, "counts"), _stream(stream))
    _check(code, "swiftprune_count_pruned")


def swiftprune_calibrate_la(W, hr, target_sparsity: float, tolerance: float = 1e-3, la_lo: float = -8.0,
                            la_hi: float = 8.0, alpha: float = 0.125, beta: float = 0.125, counts_ws=None,
                            stream=None):
    """(la, achieved, reached) with the pruned fraction of W within `tolerance` of the target when
    reached is True.  Synchronises the stream."""
    import torch
    ptr, out, n_in, ldw, dt = _matrix(W)
    if counts_ws is None:
        counts_ws = torch.empty(16, dtype=torch.int64, device=W.device)
    la, ach = C.c_float(), C.c_float()
    code = load_library().swiftprune_calibrate_la(
        ptr, out, n_in, ldw, dt, _vec(hr, torch.float32, n_in, "hr"), float(alpha), float(beta),
        float(target_sparsity), float(tolerance), float(la_lo), float(la_hi),
        _vec(counts_ws, torch.int64, 16, "counts_ws"), C.byref(la), C.byref(ach), _stream(stream))
    if code not in (SP_OK, SP_ERANGE):
        _check(code, "swiftprune_calibrate_la")
    return la.value, ach.value, code == SP_OK


def swiftprune_la_workspace_bytes() -> int:
    return int(load_library().swiftprune_la_workspace_bytes())


def swiftprune_calibrate_la_device(W, hr, target_sparsity: float, la_out, pruned_out=None, status_out=None,
                                   alpha: float = 0.125, beta: float = 0.125, workspace=None, stream=None):
    """la for a target pruned fraction, computed on the stream and left in la_out (float32 GPU tensor [1]);
    pruned_out (int64 [1]) and status_out (int32 [1]) are optional GPU tensors.  No synchronisation."""
    import torch
    ptr, out, n_in, ldw, dt = _matrix(W)
    need = swiftprune_la_workspace_bytes()
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=W.device)
    code = load_library().swiftprune_calibrate_la_device(
        ptr, out, n_in, ldw, dt, _vec(hr, torch.float32, n_in, "hr"), float(alpha), float(beta),
        float(target_sparsity), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
        _vec(la_out, torch.float32, 1, "la_out"), _vec(pruned_out, torch.int64, 1, "pruned_out"),
        _vec(status_out, torch.int32, 1, "status_out"), _stream(stream))
    _check(code, "swiftprune_calibrate_la_device")
    return workspace


def swiftprune_score_select_la(W, hr, la_dev, keep_mask, alpha: float = 0.125, beta: float = 0.125,
                               row_pruned=None, flags: int = 0, stream=None):
    """swiftprune_score_select with la read from a float32 GPU tensor [1] when the kernel runs."""
    import torch
    ptr, out, n_in, ldw, dt = _matrix(W)
    words = (n_in + 31) // 32
    code = load_library().swiftprune_score_select_la(
        ptr, out, n_in, ldw, dt, _vec(hr, torch.float32, n_in, "hr"), float(alpha), float(beta),
        _vec(la_dev, torch.float32, 1, "la_dev"), _vec(keep_mask, torch.int32, out * words, "keep_mask"),
        _vec(row_pruned, torch.int32, out, "row_pruned"), int(flags), _stream(stream))
    _check(code, "swiftprune_score_select_la")


def swiftprune_topk_select(W, hr, keep_mask, k_per_row=None, k_uniform: int = 0, flags: int = 0, stream=None):
    """Prune the k smallest scores of every row (k_per_row: int32 GPU tensor [out], or k_uniform)."""
    import torch
    ptr, out, n_in, ldw, dt = _matrix(W)
    words = (n_in + 31) // 32
    code = load_library().swiftprune_topk_select(
        ptr, out, n_in, ldw, dt, _vec(hr, torch.float32, n_in, "hr"),
        _vec(k_per_row, torch.int32, out, "k_per_row"), int(k_uniform),
        _vec(keep_mask, torch.int32, out * words, "keep_mask"), int(flags), _stream(stream))
    _check(code, "swiftprune_topk_select")


def swiftprune_nm_meta_words(n_in: int, n_keep: int, m_group: int) -> int:
    return int(load_library().swiftprune_nm_meta_words(int(n_in), int(n_keep), int(m_group)))


def swiftprune_compact_nm(W, keep_mask, n_keep: int, m_group: int, values, meta, stream=None):
    """values [out, in/M*N] (W's dtype) and meta int32 [out, meta_words] from an N:M-masked W."""
    import torch
    ptr, out, n_in, ldw, dt = _matrix(W)
    words = (n_in + 31) // 32
    mw = swiftprune_nm_meta_words(n_in, n_keep, m_group)
    if mw == 0:
        raise SwiftPruneError(SP_EINVAL, "swiftprune_compact_nm")
    code = load_library().swiftprune_compact_nm(
        ptr, out, n_in, ldw, dt, _vec(keep_mask, torch.int32, out * words, "keep_mask"), int(n_keep),
        int(m_group), _vec(values, W.dtype, out * (n_in // m_group * n_keep), "values"),
        _vec(meta, torch.int32, out * mw, "meta"), _stream(stream))
    _check(code, "swiftprune_compact_nm")


def swiftprune_expand_nm(values, meta, n_in: int, n_keep: int, m_group: int, W_out, stream=None):
    import torch
    ptr, out, n2, ldw, dt = _matrix(W_out)
    if n2 != n_in:
        raise ValueError("W_out must have n_in columns")
    mw = swiftprune_nm_meta_words(n_in, n_keep, m_group)
    if mw == 0:
        raise SwiftPruneError(SP_EINVAL, "swiftprune_expand_nm")
    code = load_library().swiftprune_expand_nm(
        _vec(values, W_out.dtype, out * (n_in // m_group * n_keep), "values"),
        _vec(meta, torch.int32, out * mw, "meta"), out, n_in, dt, int(n_keep), int(m_group), ptr, ldw,
        _stream(stream))
    _check(code, "swiftprune_expand_nm")


def swiftprune_apply(W, keep_mask, stream=None):
    import torch
    ptr, out, n_in, ldw, dt = _matrix(W)
    words = (n_in + 31) // 32
    code = load_library().swiftprune_apply(ptr, out, n_in, ldw, dt,
                                           _vec(keep_mask, torch.int32, out * words, "keep_mask"),
                                           _stream(stream))
    _check(code, "swiftprune_apply")


# ------------------------------------------------------------------ convenience: one layer
class LayerBuffers:
    """Device buffers one layer's calls need (allocated once, reused across layers of the same size)."""

    def __init__(self, out: int, n_in: int, tokens: int, device="cuda"):
        import torch
        self.xsq = torch.empty(n_in, dtype=torch.float32, device=device)
        self.S = torch.empty(1, dtype=torch.float32, device=device)
        self.hr = torch.empty(n_in, dtype=torch.float32, device=device)
        self.keep_mask = torch.empty((out, (n_in + 31) // 32), dtype=torch.int32, device=device)
        self.row_pruned = torch.empty(out, dtype=torch.int32, device=device)
        self.workspace = torch.empty(swiftprune_stats_workspace_bytes(tokens, n_in), dtype=torch.uint8,
                                     device=device)


def prune_layer(W, X, buffers: LayerBuffers | None = None, sparsity: float = 0.5, nm=None,
                alpha: float = 0.125, beta: float = 0.125, la: float | None = None, stream=None):
    """The whole path for one layer, in place on W: statistics, score + selection, apply (fused).

    nm = (n_keep, m_group) selects the structured variant.  Returns the buffers (mask, counts)."""
    b = buffers or LayerBuffers(W.shape[0], W.shape[1], X.shape[0], W.device)
    swiftprune_layer_stats(X, b.xsq, b.S, b.hr, workspace=b.workspace, stream=stream)
    if nm is None:
        swiftprune_score_select(W, b.hr, b.keep_mask, sparsity=sparsity, alpha=alpha, beta=beta, la=la,
                                row_pruned=b.row_pruned, flags=SP_APPLY_INPLACE, stream=stream)
    else:
        swiftprune_nm_select(W, b.hr, nm[0], nm[1], b.keep_mask, flags=SP_APPLY_INPLACE, stream=stream)
    return b


def prune_group(Ws, X, buffers, sparsity: float = 0.5, nm=None, alpha: float = 0.125, beta: float = 0.125,
                la: float | None = None, stream=None):
    """Matrices that share the layer input X (q / k / v, gate / up), in place: ONE statistics pass, then one
    selection + apply launch over all of them.  buffers: one LayerBuffers per matrix; the statistics land
    in buffers[0] (xsq, S, hr, workspace), masks and counts in each matrix's own."""
    b0 = buffers[0]
    swiftprune_layer_stats(X, b0.xsq, b0.S, b0.hr, workspace=b0.workspace, stream=stream)
    masks = [b.keep_mask for b in buffers]
    if nm is None:
        swiftprune_score_select_group(Ws, b0.hr, masks, sparsity=sparsity, alpha=alpha, beta=beta, la=la,
                                      row_pruned=[b.row_pruned for b in buffers], flags=SP_APPLY_INPLACE,
                                      stream=stream)
    else:
        swiftprune_nm_select_group(Ws, b0.hr, nm[0], nm[1], masks, flags=SP_APPLY_INPLACE, stream=stream)
    return buffers
