"""Helpers of the GPU parity tests: host<->device movement and the mask-difference rule."""
from __future__ import annotations

import numpy as np


def to_device(a: np.ndarray, device="cuda"):
    """numpy float32 / float16 / uint16 (bf16 bits) -> torch tensor on the GPU with the same bits."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def same_bits(a: np.ndarray, b: np.ndarray) -> bool:
    """Bit-for-bit equality of two arrays of one dtype (so that -0 and +0 differ)."""
    if a.dtype != b.dtype or a.shape != b.shape:
        return False
    u = {2: np.uint16, 4: np.uint32}[a.dtype.itemsize]
    return np.array_equal(np.ascontiguousarray(a).view(u), np.ascontiguousarray(b).view(u))


def mask_to_host(t) -> np.ndarray:
    return t.detach().cpu().numpy().view(np.uint32)


def differing_bits(mask_a: np.ndarray, mask_b: np.ndarray, n: int):
    """(row, q) positions where two bit-packed masks differ."""
    x = np.ascontiguousarray(mask_a ^ mask_b)
    bits = np.unpackbits(x.view(np.uint8), axis=1, bitorder="little")[:, :n]
    return np.argwhere(bits != 0)


TOL = 1e-5   # relative distance between a score and its threshold within which a decision may differ
ULPS = 8     # ... or this many fp32 units in the last place of the larger of the threshold's two terms


def decision_open(L, thr, est_prev, dev_prev, la):
    """True where the rounding-level rule leaves a decision open.  The threshold is est - la*dev; the scan
    kernels evaluate est and dev in another addition order than the sequential fp32 walk, which moves each
    by a few units in the last place.  Where the two terms do not cancel (every la of the paper's table:
    thr is a good part of est) that is far inside TOL relative to the threshold; where they nearly cancel
    (la around 1 and above, the ratios below 50 % that the paper's table does not cover) the threshold is
    small against its terms and the same absolute error is a larger relative one, so the band is stated in
    units of the terms themselves."""
    L = np.asarray(L, dtype=np.float64)
    thr = np.asarray(thr, dtype=np.float64)
    gap = np.abs(L - thr)
    rel_ok = gap <= TOL * np.maximum(np.abs(L), np.abs(thr))
    terms = np.maximum(np.abs(np.asarray(est_prev, dtype=np.float32)),
                       np.abs(np.float32(la) * np.asarray(dev_prev, dtype=np.float32)))
    ulp_ok = gap <= ULPS * np.spacing(terms.astype(np.float32)).astype(np.float64)
    return rel_ok | ulp_ok


def check_ewma_mask(orc, W_host, hr, alpha, beta, la, mask_gpu, cnt_gpu=None):
    """Compare a GPU EWMA mask with the oracle's.  A bit may differ only where the oracle's score is
    within TOL (relative) of the oracle's threshold for that element, or within ULPS units in the last
    place of the threshold's terms (decision_open).  Returns the number of such differences; raises on
    any other difference."""
    n = W_host.shape[1]
    mask_o, cnt_o, _ = orc.ewma_select(W_host, hr, alpha, beta, la)
    diffs = differing_bits(mask_gpu, mask_o, n)
    per_row = {}
    for r, q in diffs:
        per_row.setdefault(int(r), []).append(int(q))
    for r, qs in per_row.items():
        L = orc.score(np.ascontiguousarray(W_host[r:r + 1]), hr)[0]
        _, est, dev = orc.ewma_row(L, alpha, beta, la, precision="f32")
        for q in qs:
            if q == 0:
                raise AssertionError(f"row {r}: element 0 differs (it is never pruned)")
            thr = np.float32(est[q - 1]) - np.float32(la) * np.float32(dev[q - 1])
            if not decision_open(L[q], thr, est[q - 1], dev[q - 1], la):
                raise AssertionError(f"mask differs at ({r},{q}): L={L[q]!r} thr={thr!r} est={est[q - 1]!r}, "
                                     f"not within {TOL} relative nor {ULPS} ulp of the threshold's terms")
        if cnt_gpu is not None:
            assert abs(int(cnt_gpu[r]) - int(cnt_o[r])) <= len(qs)
    if cnt_gpu is not None:
        same = np.ones(W_host.shape[0], dtype=bool)
        same[list(per_row.keys())] = False
        assert np.array_equal(np.asarray(cnt_gpu)[same], cnt_o[same])
    return len(diffs)


def near_threshold_count(orc, W_host, hr, alpha, beta, la):
    """How many decisions of the whole matrix the rounding-level rule leaves open: elements (other than a
    row's first) whose oracle score lies within TOL (relative) of the oracle's threshold for them."""
    total = 0
    sc = orc.score(np.ascontiguousarray(W_host), hr)
    for r in range(W_host.shape[0]):
        L = sc[r]
        _, est, dev = orc.ewma_row(L, alpha, beta, la, precision="f32")
        thr = est[:-1] - np.float32(la) * dev[:-1]
        total += int(np.sum(decision_open(L[1:], thr, est[:-1], dev[:-1], la)))
    return total
