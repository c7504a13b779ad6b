"""Pins of the CPU oracle: checks against what the paper and the mathematics fix.

Every pin is a function ``pin_xxx(orc, L)`` where ``orc`` is the oracle package
and ``L`` an (optionally different) loaded oracle library; it raises
AssertionError when the library under test violates the pinned fact.  The same
functions are run on the real oracle (must pass) and on deliberately broken
copies of it (each must be caught by at least one pin).

None of the pins restates the recurrence loop; they use closed forms, special
inputs, invariants, library routines (numpy sort / inverse / sum) and a
hand-worked example.
"""
from __future__ import annotations

import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ EWMA walk
def pin_worked_rows(orc, L=None):
    """Hand-worked rows (tests/golden/ewma_worked_rows.txt): bit-exact in both precisions."""
    cases, cur = [], None
    with open(os.path.join(GOLDEN, "ewma_worked_rows.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            tok = line.split()
            if tok[0] == "case":
                cur = {"p": tuple(float(x) for x in tok[1:4]), "rows": []}
                cases.append(cur)
            else:
                cur["rows"].append([float(x) for x in tok])
    assert len(cases) >= 2
    for c in cases:
        rows = np.array(c["rows"])
        a, b, la = c["p"]
        for prec in ("f32", "f64"):
            prune, est, dev = orc.ewma_row(rows[:, 0], a, b, la, precision=prec, L=L)
            assert prune.tolist() == rows[:, 2].astype(int).tolist(), (c["p"], prec, prune)
            assert np.array_equal(est.astype(np.float64), rows[:, 3]), (c["p"], prec, est)
            assert np.array_equal(dev.astype(np.float64), rows[:, 4]), (c["p"], prec, dev)


def closed_form_states(Lrow, alpha, beta):
    """est/dev after each element from the closed-form sums (float64, no recurrence):
       e_q = A^q L_0 + alpha * sum_{j=1..q} A^(q-j) L_j
       d_q = beta * sum_{j=1..q} B^(q-j) |e_j - L_j|          (e_0 = L_0, d_0 = 0)
    """
    Lrow = np.asarray(Lrow, dtype=np.float64)
    n = Lrow.shape[0]
    A, B = 1.0 - alpha, 1.0 - beta
    q = np.arange(n)
    expo = q[:, None] - q[None, :]                      # q - j
    lower = expo >= 0
    PA = np.where(lower, np.power(A, np.where(lower, expo, 0)), 0.0)
    PB = np.where(lower, np.power(B, np.where(lower, expo, 0)), 0.0)
    src = alpha * Lrow
    src[0] = Lrow[0]                                    # A^q L_0 term carries weight 1, not alpha
    e = PA @ src
    a = np.abs(e - Lrow)
    a[0] = 0.0                                          # sum starts at j = 1
    d = beta * (PB @ a)
    return e, d


def pin_closed_form(orc, L=None):
    """Recurrence vs closed-form sums, and the decisions they imply."""
    rng = _rng(11)
    for (alpha, beta, la, n) in [(0.125, 0.125, 0.5, 96), (0.3, 0.07, -0.9, 64), (0.125, 0.25, 1.3, 130)]:
        Lrow = rng.chisquare(1, size=n) * 3.0 + 1e-3
        e, d = closed_form_states(Lrow, alpha, beta)
        prune, est, dev = orc.ewma_row(Lrow, alpha, beta, la, precision="f64", L=L)
        assert np.allclose(est, e, rtol=1e-12, atol=0), np.abs(est - e).max()
        assert np.allclose(dev, d, rtol=1e-11, atol=1e-15), np.abs(dev - d).max()
        # identity |e_j - L_j| = A |e_{j-1} - L_j|
        assert np.allclose(np.abs(est[1:] - Lrow[1:]), (1 - alpha) * np.abs(est[:-1] - Lrow[1:]), rtol=1e-9)
        # decisions from the closed-form state BEFORE each element
        e_prev = np.concatenate([[Lrow[0]], e[:-1]])
        d_prev = np.concatenate([[0.0], d[:-1]])
        thr = e_prev - la * d_prev
        safe = np.abs(Lrow - thr) > 1e-9 * np.maximum(np.abs(Lrow), np.abs(thr))
        assert safe[1:].all()                         # element 0 sits exactly on its threshold (kept)
        assert np.array_equal(prune.astype(bool), Lrow < thr)
        assert 0 < prune.sum() < n
        # float walk stays within rounding of the closed form
        _, est32, dev32 = orc.ewma_row(Lrow, alpha, beta, la, precision="f32", L=L)
        assert np.allclose(est32, e, rtol=2e-6), np.abs(est32 / e - 1).max()
        assert np.allclose(dev32, d, rtol=1e-5, atol=1e-7)
    # the whole-layer walk in double: masks, counts and scores of a small matrix against the closed-form
    # decisions on scores formed with numpy
    out, n, alpha, beta, la = 5, 70, 0.125, 0.25, 0.4
    W = rng.standard_normal((out, n)).astype(np.float32)
    hr = 0.5 / (1.0 - rng.uniform(0, 0.4, n))
    mask, cnt, sc = orc.ewma_select(W, hr, alpha, beta, la, precision="f64", want_scores=True, L=L)
    ref_sc = W.astype(np.float64) ** 2 * hr
    assert np.allclose(sc, ref_sc, rtol=1e-15)
    keep = orc.unpack_mask(mask, n)
    assert mask.shape == (out, 3) and np.all((mask[:, 2] >> (n - 64)) == 0)
    for r in range(out):
        e, d = closed_form_states(ref_sc[r], alpha, beta)
        thr = np.concatenate([[ref_sc[r, 0]], e[:-1]]) - la * np.concatenate([[0.0], d[:-1]])
        assert (np.abs(ref_sc[r] - thr)[1:] > 1e-9 * np.abs(thr[1:])).all()
        assert np.array_equal(~keep[r], ref_sc[r] < thr), r
        assert cnt[r] == int((ref_sc[r] < thr).sum())


def pin_constant_row(orc, L=None):
    """L constant -> est stays at it, dev stays 0, nothing is pruned whatever la is."""
    for la in (-3.0, -0.2, 0.0, 0.5, 4.0):
        for prec in ("f32", "f64"):
            prune, est, dev = orc.ewma_row(np.full(50, 0.75), 0.125, 0.125, la, precision=prec, L=L)
            assert prune.sum() == 0
            assert np.all(est == 0.75) and np.all(dev == 0.0)


def pin_first_two_elements(orc, L=None):
    """Element 0 is never pruned; element 1 is pruned iff L_1 < L_0 for any la (dev is still 0)."""
    rng = _rng(5)
    for _ in range(200):
        Lrow = rng.random(6) + 0.1
        la = rng.uniform(-5, 5)
        prune, _, _ = orc.ewma_row(Lrow, 0.125, 0.125, la, precision="f64", L=L)
        assert prune[0] == 0
        assert bool(prune[1]) == bool(Lrow[1] < Lrow[0])
    # exact tie at element 1 is kept (strict inequality)
    prune, _, _ = orc.ewma_row(np.array([2.0, 2.0, 1.0]), 0.125, 0.125, 0.0, precision="f32", L=L)
    assert prune.tolist() == [0, 0, 1]


def pin_monotone_in_la(orc, L=None):
    """With S fixed the state does not depend on la: a larger la prunes a subset; la -> +inf prunes none
    beyond what dev == 0 allows; la -> -inf prunes all elements after the first non-zero dev."""
    rng = _rng(7)
    Lrow = rng.chisquare(1, size=400)
    prev = None
    for la in (-4.0, -1.5, -0.9, -0.2, 0.2, 0.5, 1.0, 2.0, 8.0):
        prune, _, _ = orc.ewma_row(Lrow, 0.125, 0.125, la, precision="f64", L=L)
        p = prune.astype(bool)
        if prev is not None:
            assert not (p & ~prev).any(), la          # pruned(la2) subset of pruned(la1), la1 < la2
        prev = p
    big, _, _ = orc.ewma_row(Lrow, 0.125, 0.125, 1e9, precision="f64", L=L)
    assert big[2:].sum() == 0                          # dev > 0 from element 1 on for generic input
    small, _, _ = orc.ewma_row(Lrow, 0.125, 0.125, -1e9, precision="f64", L=L)
    assert small[2:].sum() == Lrow.shape[0] - 2


def pin_step_response(orc, L=None):
    """L = c1 for q < k, c2 afterwards:  e_{k+m} = c2 + (c1 - c2) A^(m+1)."""
    c1, c2, k, alpha = 5.0, 1.0, 10, 0.125
    Lrow = np.concatenate([np.full(k, c1), np.full(40, c2)])
    _, est, dev = orc.ewma_row(Lrow, alpha, 0.3, 0.5, precision="f64", L=L)
    m = np.arange(40)
    assert np.allclose(est[k:], c2 + (c1 - c2) * (1 - alpha) ** (m + 1), rtol=1e-13)
    assert np.all(est[:k] == c1) and np.all(dev[:k] == 0)
    # first deviation sample after the step: dev_k = beta * |e_k - c2|
    assert np.isclose(dev[k], 0.3 * abs(est[k] - c2), rtol=1e-14)


def pin_tracks_mean_and_deviation(orc, L=None):
    """The tracking figure of Sec. 4.2: on a long stationary row est follows the mean of the scores and
    dev the mean absolute gap between est and the scores (both are unbiased EWMAs of those quantities)."""
    rng = _rng(13)
    Lrow = rng.chisquare(1, size=40000) * 2.5
    for alpha, beta in ((0.125, 0.125), (0.05, 0.2)):
        _, est, dev = orc.ewma_row(Lrow, alpha, beta, 4.0, precision="f64", L=L)
        warm = 500
        assert abs(est[warm:].mean() / Lrow[warm:].mean() - 1) < 0.02
        gap = np.abs(est[warm:] - Lrow[warm:]).mean()
        assert abs(dev[warm:].mean() / gap - 1) < 0.02
        # a slower est (smaller alpha) is smoother
    _, e_fast, _ = orc.ewma_row(Lrow, 0.5, 0.125, 4.0, precision="f64", L=L)
    _, e_slow, _ = orc.ewma_row(Lrow, 0.02, 0.125, 4.0, precision="f64", L=L)
    assert e_slow[500:].std() < 0.3 * e_fast[500:].std()


# ------------------------------------------------------------------ statistics and score
def pin_stats_library_sum(orc, L=None):
    """Step 1 against numpy's float64 column sum; bf16 and fp32 inputs, with a row pitch."""
    from paper_2501_16376_amd import synth
    rng = _rng(3)
    X = (rng.standard_normal((300, 72)) * rng.lognormal(0, 0.5, 72)).astype(np.float32)
    Xp = np.zeros((300, 80), dtype=np.float32)
    Xp[:, :72] = X
    Xp[:, 72:] = 1e6                                    # must be ignored (pitch > in)
    acc = orc.stats_accumulate(Xp[:, :72], L=L)
    ref = np.square(X.astype(np.float64)).sum(0)
    assert np.allclose(acc, ref, rtol=1e-14)
    # chunked accumulation continues the same sums
    acc2 = orc.stats_accumulate(Xp[:100, :72], L=L)
    acc2 = orc.stats_accumulate(Xp[100:, :72], acc2, L=L)
    assert np.allclose(acc2, ref, rtol=1e-14)
    xsq, S = orc.stats_finalize(acc, L=L)
    assert np.array_equal(xsq, ref.astype(np.float32)) or np.allclose(xsq, ref, rtol=1e-7)
    assert np.isclose(S, ref.sum(), rtol=1e-7)
    # bf16 bits are widened exactly
    Xb = synth.f32_to_bf16_bits(X)
    accb = orc.stats_accumulate(Xb, L=L)
    refb = np.square(synth.bf16_bits_to_f32(Xb).astype(np.float64)).sum(0)
    assert np.allclose(accb, refb, rtol=1e-14)
    # all-ones input: xsq = T, S = T*in, hr = 0.5/(1 - 1/in) (all exactly representable for in = 64)
    ones = np.ones((128, 64), dtype=np.float32)
    xsq1, S1, hr1 = orc.layer_stats(ones, L=L)
    assert np.all(xsq1 == 128.0) and S1 == 128.0 * 64
    assert np.all(hr1 == np.float32(0.5) / (np.float32(1) - np.float32(1 / 64)))


def pin_stats_from_partials(orc, L=None):
    """Statistics from sums that the producer of X formed over its own pieces of the tokens: the column sum
    of the pieces (numpy, float64), with a row pitch, continued over two calls; and the property that makes
    the entry point useful - cutting the tokens of X into pieces (of unequal length), squaring and summing
    each piece exactly, and combining the pieces gives the statistics of X itself."""
    rng = _rng(31)
    P = rng.lognormal(0.0, 1.0, (7, 40)).astype(np.float32)
    Pp = np.full((7, 48), 1e9, dtype=np.float32)              # pitch > in: the padding must be ignored
    Pp[:, :40] = P
    acc = orc.stats_accumulate_partials(Pp[:, :40], L=L)
    ref = P.astype(np.float64).sum(0)
    assert np.allclose(acc, ref, rtol=1e-15)
    acc2 = orc.stats_accumulate_partials(Pp[:3, :40], L=L)
    acc2 = orc.stats_accumulate_partials(Pp[3:, :40], acc2, L=L)
    assert np.allclose(acc2, ref, rtol=1e-15)
    one = orc.stats_accumulate_partials(np.ascontiguousarray(P[2:3]), L=L)   # a single piece is returned as it is
    assert np.array_equal(one, P[2].astype(np.float64))
    # pieces of X: small integers, so that every square and every sum is exact in float and in double
    X = rng.integers(-8, 9, size=(90, 24)).astype(np.float32)
    cuts = [0, 13, 14, 50, 90]
    pieces = np.stack([np.square(X[a:b].astype(np.float64)).sum(0) for a, b in zip(cuts[:-1], cuts[1:])]).astype(np.float32)
    xsq_p, S_p = orc.stats_finalize(orc.stats_accumulate_partials(pieces, L=L), L=L)
    xsq_x, S_x, _ = orc.layer_stats(X, L=L)
    assert np.array_equal(xsq_p, xsq_x) and S_p == S_x


def pin_inverse_identity(orc, L=None):
    """The score's denominator is the paper's surrogate for the diagonal of the damped inverse Hessian.

    For one activation vector x (n entries), H = 2 x x^T + (2S/n) I.  Sec. 3.1 derives
        inv(H)_qq = (S/n + S - x_q^2) / ((2S/n)(S/n + S))
                  = (1 - x_q^2/S) * G_q,   G_q = n/(2(1+n)) / (S - x_q^2) + n^2 / (2 S (1+n)).
    So  0.5 * G_q / inv(H)_qq  must equal the oracle's channel factor 0.5/(1 - x_q^2/S), with inv(H)
    from numpy.linalg.inv.  Also G_q -> n/(2S) when S >> x_q^2.
    """
    rng = _rng(9)
    for n in (4, 9, 16):
        x = rng.standard_normal(n) * rng.lognormal(0, 0.5, n)
        S = float(np.sum(x * x))
        H = 2.0 * np.outer(x, x) + (2.0 * S / n) * np.eye(n)
        Hinv_qq = np.diag(np.linalg.inv(H))
        closed = (S / n + S - x * x) / ((2 * S / n) * (S / n + S))
        assert np.allclose(Hinv_qq, closed, rtol=1e-10)
        G = n / (2.0 * (1 + n)) / (S - x * x) + n * n / (2.0 * S * (1 + n))
        acc = orc.stats_accumulate(np.ascontiguousarray(x[None, :], dtype=np.float32), L=L)
        x32 = x.astype(np.float32).astype(np.float64)
        S32 = float(np.sum(x32 * x32))
        H32 = 2.0 * np.outer(x32, x32) + (2.0 * S32 / n) * np.eye(n)
        G32 = n / (2.0 * (1 + n)) / (S32 - x32 * x32) + n * n / (2.0 * S32 * (1 + n))
        hr64 = orc.channel_factor_f64(acc, L=L)
        assert np.allclose(hr64, 0.5 * G32 / np.diag(np.linalg.inv(H32)), rtol=1e-9)
        # score = w^2 * hr
        w = rng.standard_normal((3, n)).astype(np.float32)
        sc = orc.score(w, hr64, precision="f64", L=L)
        assert np.allclose(sc, 0.5 * w.astype(np.float64) ** 2 / (1.0 - x32 * x32 / S32), rtol=1e-12)
    # large n: G_q / (n/(2S)) -> 1
    n = 4096
    x = rng.standard_normal(n)
    S = float(np.sum(x * x))
    G = n / (2.0 * (1 + n)) / (S - x * x) + n * n / (2.0 * S * (1 + n))
    assert np.abs(G / (n / (2 * S)) - 1).max() < 5e-3


def pin_float_factor_matches_double(orc, L=None):
    """Float channel factor and float scores are the double ones to rounding; degenerate conventions."""
    from paper_2501_16376_amd import synth
    W, X = synth.config1()
    acc = orc.stats_accumulate(X, L=L)
    xsq, S = orc.stats_finalize(acc, L=L)
    hr32 = orc.channel_factor_f32(xsq, S, L=L)
    hr64 = orc.channel_factor_f64(acc, L=L)
    assert np.allclose(hr32, hr64, rtol=3e-7)
    assert hr32.min() >= 0.5 and hr32.max() > 0.6       # outlier channels raise the factor
    s32 = orc.score(W, hr32, precision="f32", L=L)
    s64 = orc.score(W, hr64, precision="f64", L=L)
    assert np.allclose(s32, s64, rtol=5e-7)
    # conventions where the paper is silent
    assert np.all(orc.channel_factor_f32(np.zeros(8, np.float32), 0.0, L=L) == 0.5)
    one_hot = np.zeros(8, np.float32)
    one_hot[3] = 4.0
    hr = orc.channel_factor_f32(one_hot, 4.0, L=L)
    assert hr[3] == np.float32(0.5) / np.finfo(np.float32).eps and np.all(np.delete(hr, 3) == 0.5)


# ------------------------------------------------------------------ whole-layer selection
def pin_select_metamorphic(orc, L=None):
    """Scaling W or X by a power of two, permuting rows: masks follow exactly."""
    from paper_2501_16376_amd import synth
    W, X = synth.layer_inputs(24, 160, 64, seed=4, dtype="f32", n_outlier=2)
    _, _, hr = orc.layer_stats(X, L=L)
    m0, c0, s0 = orc.ewma_select(W, hr, 0.125, 0.125, 0.5, want_scores=True, L=L)
    assert 0.3 < c0.sum() / W.size < 0.7
    # W * 2^k: scores scale by 4^k exactly, decisions unchanged
    m1, c1, s1 = orc.ewma_select(W * np.float32(8.0), hr, 0.125, 0.125, 0.5, want_scores=True, L=L)
    assert np.array_equal(m0, m1) and np.array_equal(s1, s0 * np.float32(64.0))
    # X * 2^k: xsq and S scale by 4^k, the ratio (and hr) is unchanged bit for bit
    _, _, hr2 = orc.layer_stats(X * np.float32(4.0), L=L)
    assert np.array_equal(hr, hr2)
    # row permutation
    perm = _rng(1).permutation(W.shape[0])
    m2, c2, _ = orc.ewma_select(np.ascontiguousarray(W[perm]), hr, 0.125, 0.125, 0.5, L=L)
    assert np.array_equal(m2, m0[perm]) and np.array_equal(c2, c0[perm])
    # token permutation leaves the statistics unchanged up to double rounding
    xsq_a, S_a, _ = orc.layer_stats(X, L=L)
    xsq_b, S_b, _ = orc.layer_stats(np.ascontiguousarray(X[_rng(2).permutation(X.shape[0])]), L=L)
    assert np.allclose(xsq_a, xsq_b, rtol=1e-7) and np.isclose(S_a, S_b, rtol=1e-7)
    # mask format: bit (q & 31) of word q >> 5; row counts match the mask; pad bits are zero
    keep = orc.unpack_mask(m0, W.shape[1])
    assert np.array_equal((~keep).sum(1), c0)
    assert keep[:, 0].all()
    row0 = s0[0]
    prune0, _, _ = orc.ewma_row(row0, 0.125, 0.125, 0.5, precision="f32", L=L)
    for q in (0, 1, 31, 32, 33, 100, 159):
        assert ((int(m0[0, q >> 5]) >> (q & 31)) & 1) == (0 if prune0[q] else 1)
    W2, X2 = synth.layer_inputs(3, 40, 16, seed=8, dtype="f32", n_outlier=1)
    _, _, hrb = orc.layer_stats(X2, L=L)
    mb, _, _ = orc.ewma_select(W2, hrb, 0.125, 0.125, 0.5, L=L)
    assert mb.shape == (3, 2) and np.all((mb[:, 1] >> 8) == 0)
    # pitch: a wider parent array gives the same result
    Wp = np.full((24, 200), 7.0, dtype=np.float32)
    Wp[:, :160] = W
    m3, _, _ = orc.ewma_select(Wp[:, :160], hr, 0.125, 0.125, 0.5, L=L)
    assert np.array_equal(m3, m0)


def pin_uniform_energy_reduces_to_magnitude(orc, L=None):
    """Equal channel energies -> score proportional to w^2: N:M equals per-group top-N of |w|, and the
    EWMA selection equals the walk over c*w^2."""
    rng = _rng(21)
    n, out = 64, 12
    X = rng.choice([-1.0, 1.0], size=(32, n)).astype(np.float32)       # xsq[q] = 32 for all q
    xsq, S, hr = orc.layer_stats(X, L=L)
    assert np.all(xsq == 32.0) and np.all(hr == hr[0])
    W = rng.standard_normal((out, n)).astype(np.float32)
    for (nk, m) in [(2, 4), (4, 8), (1, 4), (3, 4), (2, 8), (8, 16)]:
        mask, _ = orc.nm_select(W, hr, nk, m, L=L)
        keep = orc.unpack_mask(mask, n)
        mag = np.abs(W).reshape(out, n // m, m)
        order = np.argsort(mag, axis=2, kind="stable")                 # library sort: ascending |w|
        ref = np.ones_like(mag, dtype=bool)
        np.put_along_axis(ref, order[:, :, : m - nk], False, axis=2)
        assert np.array_equal(keep, ref.reshape(out, n)), (nk, m)
    mask, cnt, sc = orc.ewma_select(W, hr, 0.125, 0.125, 0.2, want_scores=True, L=L)
    for r in range(out):
        prune, _, _ = orc.ewma_row((W[r] * W[r]) * hr[0], 0.125, 0.125, 0.2, precision="f32", L=L)
        assert np.array_equal(~orc.unpack_mask(mask, n)[r], prune.astype(bool))


def pin_nm_invariants(orc, L=None):
    """Exactly M-N pruned per group; every kept score >= every pruned one; equals a per-group
    lexicographic sort on (score, index); ties prune the lower index first."""
    from paper_2501_16376_amd import synth
    Wb, Xb = synth.layer_inputs(16, 96, 64, seed=6, dtype="bf16", n_outlier=3)
    _, _, hr = orc.layer_stats(Xb, L=L)
    for (nk, m) in [(2, 4), (4, 8), (1, 4), (3, 4), (6, 8), (4, 16)]:
        mask, sc = orc.nm_select(Wb, hr, nk, m, want_scores=True, L=L)
        keep = orc.unpack_mask(mask, 96).reshape(16, 96 // m, m)
        assert np.all(keep.sum(2) == nk)
        g = sc.reshape(16, 96 // m, m)
        kept_min = np.where(keep, g, np.inf).min(2)
        pruned_max = np.where(~keep, g, -np.inf).max(2)
        assert np.all(kept_min >= pruned_max)
        idx = np.broadcast_to(np.arange(m), g.shape)
        ref = np.ones_like(keep)
        for r in range(16):
            for j in range(96 // m):
                order = np.lexsort((idx[r, j], g[r, j]))               # by score, then index
                ref[r, j, order[: m - nk]] = False
        assert np.array_equal(keep, ref), (nk, m)
        # the double-precision instantiation: same rule on double scores (per-group lexsort again)
        hr64 = hr.astype(np.float64) * (1.0 + 1e-9 * np.arange(96))      # not representable in float
        mask64, sc64 = orc.nm_select(Wb, hr64, nk, m, precision="f64", want_scores=True, L=L)
        w64 = synth.bf16_bits_to_f32(Wb).astype(np.float64)
        assert np.allclose(sc64, w64 * w64 * hr64, rtol=1e-15)
        g64 = sc64.reshape(16, 96 // m, m)
        ref64 = np.ones_like(keep)
        for r in range(16):
            for j in range(96 // m):
                ref64[r, j, np.lexsort((idx[r, j], g64[r, j]))[: m - nk]] = False
        assert np.array_equal(orc.unpack_mask(mask64, 96).reshape(16, 96 // m, m), ref64), (nk, m)
    # ties: all-equal weights, equal energies -> the first M-N of each group go
    X = np.ones((4, 16), dtype=np.float32)
    _, _, hr1 = orc.layer_stats(X, L=L)
    mask, _ = orc.nm_select(np.full((2, 16), 0.5, np.float32), hr1, 2, 4, L=L)
    assert np.array_equal(orc.unpack_mask(mask, 16), np.tile([False, False, True, True], (2, 4)))
    mask, _ = orc.nm_select(np.full((1, 16), 0.5, np.float32), hr1, 3, 8, L=L)
    assert np.array_equal(orc.unpack_mask(mask, 16)[0], np.tile([False] * 5 + [True] * 3, 2))


def pin_channel_energy_changes_ranking(orc, L=None):
    """A weight on a high-energy channel outranks a slightly larger weight on a quiet channel."""
    X = np.ones((8, 4), dtype=np.float32)
    X[:, 2] = 3.0                                        # xsq = [8, 8, 72, 8], S = 96
    _, _, hr = orc.layer_stats(X, L=L)
    assert hr[2] == np.float32(0.5) / (np.float32(1) - np.float32(72) / np.float32(96))   # = 2.0
    W = np.array([[1.0, 1.2, 0.9, 1.1]], dtype=np.float32)
    mask, sc = orc.nm_select(W, hr, 2, 4, want_scores=True, L=L)
    # quiet channels: 0.5/(1 - 8/96) = 6/11; loud channel: 2 -> scores [6/11, 1.44*6/11, 1.62, 1.21*6/11]
    assert orc.unpack_mask(mask, 4)[0].tolist() == [False, True, True, False]
    assert np.allclose(sc[0], [6 / 11, 1.44 * 6 / 11, 1.62, 1.21 * 6 / 11], rtol=1e-6)


def _literal_golden():
    params, rows = None, []
    with open(os.path.join(GOLDEN, "literal_worked_row.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            tok = line.split()
            if tok[0] == "params":
                params = tuple(float(x) for x in tok[1:5])
            else:
                rows.append([float(x) for x in tok])
    return params, np.array(rows)


def pin_literal_form(orc, L=None):
    """Algorithm 1 as printed (S shrinks by w^2 on pruning) vs the fixed-S form: identical for
    calibration-sized sums, different when S is comparable to w^2; and a hand-worked row
    (tests/golden/literal_worked_row.txt) that fixes the direction, the amount and the timing of the update."""
    from paper_2501_16376_amd import synth
    W, X = synth.config1()
    xsq, S, hr = orc.layer_stats(X, L=L)
    m0, c0, _ = orc.ewma_select(W, hr, 0.125, 0.125, 0.5, L=L)
    m1, c1, eff = orc.ewma_select_literal(W, xsq, S, 0.125, 0.125, 0.5, L=L)
    assert eff == 0 and np.array_equal(m0, m1) and np.array_equal(c0, c1)
    assert float(np.max(W * W)) < float(np.spacing(np.float32(S))) / 2
    # tiny activations: S ~ w^2, so the update matters and the sum really moves
    Xs = (X * np.float32(1e-4))[:4]
    xsq_s, S_s, hr_s = orc.layer_stats(Xs, L=L)
    m2, _, _ = orc.ewma_select(W, hr_s, 0.125, 0.125, 0.5, L=L)
    m3, _, eff3 = orc.ewma_select_literal(W, xsq_s, S_s, 0.125, 0.125, 0.5, L=L)
    assert eff3 > 1000 and not np.array_equal(m2, m3)

    # the hand-worked row, twice (two rows of one matrix: every row starts again from S)
    (alpha, beta, la, S0), g = _literal_golden()
    n = g.shape[0]
    Wg = np.ascontiguousarray(np.tile(g[:, 0].astype(np.float32), (2, 1)))
    xg = g[:, 1].astype(np.float32)
    mask, cnt, eff, sc, S_rows = orc.ewma_select_literal(Wg, xg, S0, alpha, beta, la, details=True, L=L)
    keep = orc.unpack_mask(mask, n)
    for r in range(2):
        assert np.array_equal(sc[r].astype(np.float64), g[:, 3]), (r, sc[r])
        assert np.array_equal(~keep[r], g[:, 5].astype(bool)), (r, keep[r])
        assert float(S_rows[r]) == g[-1, 8], S_rows
    assert cnt.tolist() == [int(g[:, 5].sum())] * 2
    assert eff == 2 * int(np.sum(g[:, 8] != g[:, 2]))
    # the table's own bookkeeping: S_r moves exactly when an element is pruned, by exactly w^2
    assert np.array_equal(g[:, 2] - g[:, 8], g[:, 5] * g[:, 0] ** 2)
    assert np.array_equal(g[1:, 2], g[:-1, 8]) and g[0, 2] == S0
    # est / dev columns of the table follow from its scores through the fixed-S walk (pinned separately)
    prune_w, est_w, dev_w = orc.ewma_row(g[:, 3], alpha, beta, la, precision="f32", L=L)
    assert np.array_equal(est_w.astype(np.float64), g[:, 6]) and np.array_equal(dev_w.astype(np.float64), g[:, 7])
    assert np.array_equal(prune_w.astype(bool), g[:, 5].astype(bool))
    # and on this row holding S fixed gives other scores (the row exists to tell the two apart)
    hr_fixed = orc.channel_factor_f32(xg, S0, L=L)
    assert not np.array_equal(orc.score(Wg, hr_fixed, L=L)[0], sc[0])


def pin_apply(orc, L=None):
    from paper_2501_16376_amd import synth
    Wb, Xb = synth.layer_inputs(8, 72, 32, seed=12, dtype="bf16", n_outlier=1)
    _, _, hr = orc.layer_stats(Xb, L=L)
    mask, cnt, _ = orc.ewma_select(Wb, hr, 0.125, 0.125, 0.5, L=L)
    keep = orc.unpack_mask(mask, 72)
    out = orc.apply(Wb.copy(), mask, L=L)
    assert np.array_equal(out[keep], Wb[keep]) and np.all(out[~keep] == 0)
    Wf = synth.bf16_bits_to_f32(Wb)
    Wf[0, 0] = -0.0
    outf = orc.apply(Wf.copy(), mask, L=L)
    assert np.array_equal(outf[keep].view(np.uint32), Wf[keep].view(np.uint32))
    assert np.all(outf[~keep].view(np.uint32) == 0)
    # pitch is honoured and the padding is untouched
    Wp = np.full((8, 80), 0x3F80, dtype=np.uint16)
    Wp[:, :72] = Wb
    orc.apply(Wp[:, :72], mask, L=L)
    assert np.all(Wp[:, 72:] == 0x3F80) and np.array_equal(Wp[:, :72], out)


def pin_sort_comparator(orc, L=None):
    """The EWMA rule stands in for sorting the scores and dropping the lowest (Sec. 3.1): with k = the
    number EWMA prunes in a row, most of them are among the k smallest scores; and the la table of the
    paper orders the achieved sparsity.  Returns the measured numbers for reporting."""
    from paper_2501_16376_amd import synth
    W, X = synth.config1()
    _, _, hr = orc.layer_stats(X, L=L)
    report = {}
    prev = 1.0
    for ratio, la in [(0.9, -1.5), (0.8, -0.9), (0.7, -0.2), (0.6, 0.2), (0.5, 0.5)]:
        mask, cnt, sc = orc.ewma_select(W, hr, 0.125, 0.125, la, want_scores=True, L=L)
        pruned = ~orc.unpack_mask(mask, W.shape[1])
        inter = 0
        for r in range(W.shape[0]):
            k = int(cnt[r])
            smallest = np.argsort(sc[r], kind="stable")[:k]
            inter += int(pruned[r, smallest].sum())
        overlap = inter / max(1, int(cnt.sum()))
        achieved = cnt.sum() / W.size
        report[ratio] = (la, float(achieved), float(overlap))
        assert achieved < prev                        # lower table ratio -> fewer pruned
        assert abs(achieved - ratio) < 0.1            # synthetic Gaussian weights land near the table
        assert overlap > 0.85
        prev = achieved
    return report


def rng_weights_with_nan():
    """2 x 32 float32 weights with a few NaNs of different payloads and signs, and infinities."""
    W = _rng(41).standard_normal((2, 32)).astype(np.float32)
    bits = W.view(np.uint32)
    bits[0, 5] = 0x7fc00001
    bits[0, 9] = 0xffc00000          # negative quiet NaN
    bits[0, 17] = 0x7f800001         # smallest payload
    bits[0, 2] = 0x7f800000          # +inf: squared it stays +inf and ranks below the NaNs
    bits[1, 0] = 0x7fffffff
    bits[1, 31] = 0x7fc00000
    bits[1, 30] = 0xff800000         # -inf -> score +inf
    return W


def pin_topk_is_library_sort(orc, L=None):
    """The sort-based comparator equals numpy's lexsort on (score, index): the k smallest go, ties by
    the lower index, k = 0 and k = in behave, per-row k is honoured."""
    from paper_2501_16376_amd import synth
    Wb, Xb = synth.layer_inputs(10, 96, 64, seed=31, dtype="bf16", n_outlier=2)
    Wb[3, 10:20] = Wb[3, 10]                       # exact ties inside a row
    Wb[4, :] = Wb[4, 0]                            # a whole row of ties
    _, _, hr = orc.layer_stats(Xb, L=L)
    hr[:] = np.float32(hr[0])                      # ties in w must be ties in score
    sc = orc.score(Wb, hr, L=L)
    ks = np.array([0, 1, 5, 7, 40, 48, 95, 96, 200, -3], dtype=np.int32)
    mask = orc.topk_select(Wb, hr, ks, L=L)
    keep = orc.unpack_mask(mask, 96)
    for r in range(10):
        k = int(np.clip(ks[r], 0, 96))
        order = np.lexsort((np.arange(96), sc[r]))
        ref = np.ones(96, dtype=bool)
        ref[order[:k]] = False
        assert np.array_equal(keep[r], ref), r
    keep4 = orc.unpack_mask(orc.topk_select(Wb, hr, 40, L=L), 96)
    assert np.array_equal(keep4[4], np.arange(96) >= 40)          # all-tie row: the first 40 go
    assert np.all((~keep4).sum(1) == 40)
    # NaN scores rank above every number, +inf included, and among themselves in index order whatever
    # their payload: the same as sorting on (is-NaN, score, index)
    Wn = rng_weights_with_nan()
    hr1 = np.ones(Wn.shape[1], dtype=np.float32)
    scn = Wn.astype(np.float64) ** 2
    for k in (3, 20, 27, 28, 29, 30, 31, 32):
        keepn = orc.unpack_mask(orc.topk_select(Wn, hr1, k, L=L), Wn.shape[1])
        for r in range(Wn.shape[0]):
            isn = np.isnan(scn[r])
            order = np.lexsort((np.arange(Wn.shape[1]), np.where(isn, 0.0, scn[r]), isn))
            ref = np.ones(Wn.shape[1], dtype=bool)
            ref[order[:k]] = False
            assert np.array_equal(keepn[r], ref), (k, r)


def pin_compact_nm(orc, L=None):
    """Compact N:M storage: a hand-made example, and expand(compact(W)) == apply(W, mask) for masks from
    the N:M selection (2:4, 4:8, 1:4, 6:8, 8:16); values are the kept entries in column order."""
    from paper_2501_16376_amd import synth
    # one row, two groups of four: keep columns {1,3} and {4,6}
    W = np.array([[10, 11, 12, 13, 14, 15, 16, 17]], dtype=np.float32)
    mask = np.array([[0b01011010]], dtype=np.uint32)
    vals, meta = orc.compact_nm(W, mask, 2, 4, L=L)
    assert vals.tolist() == [[11, 13, 14, 16]]
    assert meta.tolist() == [[1 | 3 << 2 | 0 << 4 | 2 << 6]]       # positions 1,3,0,2 in 2-bit fields
    assert np.array_equal(orc.expand_nm(vals, meta, 8, 2, 4, L=L), [[0, 11, 0, 13, 14, 0, 16, 0]])
    # 4:8 uses 4-bit fields: keep {0,2,5,7}
    mask8 = np.array([[0b10100101]], dtype=np.uint32)
    vals8, meta8 = orc.compact_nm(W, mask8, 4, 8, L=L)
    assert vals8.tolist() == [[10, 12, 15, 17]] and meta8.tolist() == [[0 | 2 << 4 | 5 << 8 | 7 << 12]]
    Wb, Xb = synth.layer_inputs(12, 192, 64, seed=17, dtype="bf16", n_outlier=2)
    _, _, hr = orc.layer_stats(Xb, L=L)
    for nk, m in ((2, 4), (4, 8), (1, 4), (6, 8), (8, 16)):
        nm, _ = orc.nm_select(Wb, hr, nk, m, L=L)
        vals, meta = orc.compact_nm(Wb, nm, nk, m, L=L)
        assert vals.shape == (12, 192 // m * nk) and meta.shape == (12, orc.nm_meta_words(192, nk, m))
        keep = orc.unpack_mask(nm, 192)
        assert np.array_equal(vals, Wb[keep].reshape(12, -1))
        dense = orc.expand_nm(vals, meta, 192, nk, m, L=L)
        assert np.array_equal(dense, orc.apply(Wb.copy(), nm, L=L)), (nk, m)
    # a group with fewer kept entries than N is padded with +0 and still round-trips
    sparse_mask = np.array([[0b00000010]], dtype=np.uint32)         # group 0 keeps only column 1, group 1 nothing
    vals, meta = orc.compact_nm(W, sparse_mask, 2, 4, L=L)
    assert vals.tolist() == [[11, 0, 0, 0]]
    assert np.array_equal(orc.expand_nm(vals, meta, 8, 2, 4, L=L), [[0, 11, 0, 0, 0, 0, 0, 0]])


def pin_binary16_storage(orc, L=None):
    """IEEE binary16 storage (IEEE 754-2008 Sec. 3.6): the oracle's decoder against numpy's float16 for
    all 65536 bit patterns (through the sum of squares of a one-token activation matrix, which is exact
    in double), and every step on a float16 matrix against the same values widened to float32."""
    bits = np.arange(65536, dtype=np.uint16)
    X = bits.view(np.float16).reshape(1, -1)
    acc = orc.stats_accumulate(X, None, L=L)
    with np.errstate(invalid="ignore", over="ignore"):
        ref = X[0].astype(np.float64) ** 2
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(acc), nan)
    assert np.array_equal(acc[~nan], ref[~nan])
    # subnormals, the largest finite value and one ordinary value by hand
    hand = np.array([0x0001, 0x03ff, 0x0400, 0x7bff, 0x3555, 0xc000], dtype=np.uint16).view(np.float16).reshape(1, -1)
    want = [2.0 ** -24, 1023 * 2.0 ** -24, 2.0 ** -14, 65504.0, (1 + 0x155 / 1024) * 0.25, -2.0]
    assert np.array_equal(orc.stats_accumulate(hand, None, L=L), np.array(want) ** 2)

    rng = _rng(16)
    out, n = 6, 96
    W16 = rng.normal(0, 0.02, size=(out, n)).astype(np.float16)
    W16[0, :4] = np.array([6.0e-8, -6.1e-5, 0.0, 1.5], dtype=np.float16)      # subnormal, smallest normal, zero, large
    W32 = W16.astype(np.float32)
    hr = (0.5 / (1.0 - rng.uniform(0, 0.3, n))).astype(np.float32)
    assert np.array_equal(orc.score(W16, hr, L=L), orc.score(W32, hr, L=L))
    m16, c16, _ = orc.ewma_select(W16, hr, 0.125, 0.125, 0.2, L=L)
    m32, c32, _ = orc.ewma_select(W32, hr, 0.125, 0.125, 0.2, L=L)
    assert np.array_equal(m16, m32) and np.array_equal(c16, c32)
    for nk, m in ((2, 4), (4, 8)):
        k16, _ = orc.nm_select(W16, hr, nk, m, L=L)
        k32, _ = orc.nm_select(W32, hr, nk, m, L=L)
        assert np.array_equal(k16, k32)
        a16 = orc.apply(W16.copy(), k16, L=L)
        assert a16.dtype == np.float16
        assert np.array_equal(a16.astype(np.float32), orc.apply(W32.copy(), k32, L=L))
        kept = orc.unpack_mask(k16, n)
        assert np.array_equal(a16.view(np.uint16)[kept], W16.view(np.uint16)[kept])       # kept: bit for bit
        assert np.all(a16.view(np.uint16)[~kept] == 0)                                    # pruned: +0
        vals, meta = orc.compact_nm(W16, k16, nk, m, L=L)
        assert vals.dtype == np.float16
        assert np.array_equal(orc.expand_nm(vals, meta, n, nk, m, L=L).view(np.uint16), a16.view(np.uint16))
    assert np.array_equal(orc.topk_select(W16, hr, 40, L=L), orc.topk_select(W32, hr, 40, L=L))


ALL_PINS = [pin_binary16_storage, pin_topk_is_library_sort, pin_compact_nm, pin_tracks_mean_and_deviation, pin_worked_rows, pin_closed_form, pin_constant_row, pin_first_two_elements,
            pin_monotone_in_la, pin_step_response, pin_stats_library_sum, pin_stats_from_partials, pin_inverse_identity,
            pin_float_factor_matches_double, pin_select_metamorphic,
            pin_uniform_energy_reduces_to_magnitude, pin_nm_invariants,
            pin_channel_energy_changes_ranking, pin_literal_form, pin_apply, pin_sort_comparator]
