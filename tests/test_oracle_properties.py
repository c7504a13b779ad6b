"""CPU-only, property-based (hypothesis): invariants of the oracle's EWMA walk and N:M rule on random
small inputs.  These complement the fixed pins in tests/pins.py."""
import numpy as np
from hypothesis import given, settings, strategies as st

rows = st.lists(st.floats(min_value=2.0 ** -20, max_value=2.0 ** 20, allow_nan=False, width=32),
                min_size=2, max_size=80)
alphas = st.sampled_from([0.125, 0.25, 0.5, 0.3, 0.9, 1.0, 0.01])


@settings(max_examples=150, deadline=None, derandomize=True, database=None)
@given(L=rows, alpha=alphas, beta=alphas, la=st.floats(min_value=-4, max_value=4, allow_nan=False))
def test_walk_invariants(orc, L, alpha, beta, la):
    L = np.asarray(L, dtype=np.float64)
    prune, est, dev = orc.ewma_row(L, alpha, beta, la, precision="f64")
    assert prune[0] == 0                                   # the first element is never pruned
    assert bool(prune[1]) == bool(L[1] < L[0])             # dev is still 0 at the second element
    assert np.all(dev >= 0)
    lo, hi = np.minimum.accumulate(L), np.maximum.accumulate(L)
    assert np.all(est >= lo * (1 - 1e-12)) and np.all(est <= hi * (1 + 1e-12))   # est is a convex combination
    # scaling all scores by a power of two scales the state exactly and leaves the decisions alone
    p2, e2, d2 = orc.ewma_row(L * 4.0, alpha, beta, la, precision="f64")
    assert np.array_equal(p2, prune) and np.array_equal(e2, est * 4.0) and np.array_equal(d2, dev * 4.0)
    # a larger la never prunes more
    p3, _, _ = orc.ewma_row(L, alpha, beta, la + 0.75, precision="f64")
    assert not np.any(p3.astype(bool) & ~prune.astype(bool))


@settings(max_examples=100, deadline=None, derandomize=True, database=None)
@given(data=st.data())
def test_nm_invariants(orc, data):
    m = data.draw(st.sampled_from([4, 8, 16]))
    nk = data.draw(st.integers(min_value=1, max_value=m - 1))
    groups = data.draw(st.integers(min_value=1, max_value=6))
    out = data.draw(st.integers(min_value=1, max_value=4))
    n = groups * m
    vals = data.draw(st.lists(st.sampled_from([-2.0, -1.0, -0.5, 0.0, 0.25, 0.5, 1.0, 3.0]),
                              min_size=out * n, max_size=out * n))          # few distinct values: many ties
    W = np.asarray(vals, dtype=np.float32).reshape(out, n)
    hr = np.full(n, 0.5, dtype=np.float32)
    mask, sc = orc.nm_select(W, hr, nk, m, want_scores=True)
    keep = orc.unpack_mask(mask, n).reshape(out, groups, m)
    assert np.all(keep.sum(2) == nk)
    g = sc.reshape(out, groups, m)
    for r in range(out):
        for j in range(groups):
            order = np.lexsort((np.arange(m), g[r, j]))
            ref = np.ones(m, dtype=bool)
            ref[order[: m - nk]] = False
            assert np.array_equal(keep[r, j], ref)
    # top-k with k = M - N on a single group is the same selection
    if groups == 1:
        assert np.array_equal(orc.topk_select(W, hr, m - nk), mask)
