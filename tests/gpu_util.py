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


def check_ewma_mask(orc, W_host, hr, alpha, beta, la, mask_gpu, cnt_gpu=None):
    """Compare a GPU EWMA mask with the oracle's.  A bit may differ only where the oracle's score is
    within TOL (relative) of the oracle's threshold for that element.  Returns the number of such
    differences; raises on any other difference."""
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
            scale = max(abs(float(L[q])), abs(float(thr)))
            if not abs(float(L[q]) - float(thr)) <= TOL * scale:
                raise AssertionError(f"mask differs at ({r},{q}): L={L[q]!r} thr={thr!r}, not within {TOL} relative")
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
        scale = np.maximum(np.abs(L[1:]), np.abs(thr))
        total += int(np.sum(np.abs(L[1:].astype(np.float64) - thr.astype(np.float64)) <= TOL * scale))
    return total
