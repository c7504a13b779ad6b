"""GPU: swiftprune_layer_stats_static (partial sums in the library's own device array, no allocation)
against swiftprune_layer_stats on the same inputs, called twice in a row with the second input smaller,
so that whatever the first call left in the shared array is still there when the second one runs."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _pair(sp, torch, X):
    n = X.shape[1]
    dev = X.device
    a = [torch.full((n,), -1.0, dtype=torch.float32, device=dev) for _ in range(2)]
    b = [torch.full((n,), -1.0, dtype=torch.float32, device=dev) for _ in range(2)]
    Sa = torch.full((1,), -1.0, dtype=torch.float32, device=dev)
    Sb = torch.full((1,), -1.0, dtype=torch.float32, device=dev)
    return a, Sa, b, Sb


def test_static_workspace_matches_workspace_call(orc):
    import torch
    from paper_2501_16376_amd import binding as sp, synth
    from gpu_util import to_device

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    L = sp.load_library()
    # large first (several strips, every split used), then a smaller ragged one, then an accumulate pair
    shapes = [(20000, 4096, "bf16"), (777, 1000, "bf16"), (300, 250, "f32")]
    for tokens, n, dt in shapes:
        _, Xh = synth.layer_inputs(1, n, tokens, seed=tokens + n, dtype=dt)
        X = to_device(Xh, dev)
        (xsq_a, hr_a), Sa, (xsq_b, hr_b), Sb = _pair(sp, torch, X)
        held_before = torch.cuda.memory_allocated()
        sp.swiftprune_layer_stats_static(X, xsq_a, Sa, hr_a)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == held_before          # the binding asked torch for no workspace
        sp.swiftprune_layer_stats(X, xsq_b, Sb, hr_b)
        torch.cuda.synchronize()
        # same kernels, same launch geometry, fixed summation order: bit for bit
        assert torch.equal(xsq_a, xsq_b) and torch.equal(hr_a, hr_b) and torch.equal(Sa, Sb)
        # and both agree with the oracle to the statistics tolerance
        xsq_o, S_o, hr_o = orc.layer_stats(Xh)
        assert np.allclose(xsq_a.cpu().numpy(), xsq_o, rtol=1e-5, atol=0)
        assert np.allclose(hr_a.cpu().numpy(), hr_o, rtol=1e-5, atol=0)
        assert np.isclose(float(Sa.item()), float(S_o), rtol=1e-5)

    # token chunks through accumulate / finalize, still on the shared array
    _, Xh = synth.layer_inputs(1, 520, 1500, seed=5, dtype="bf16")
    X = to_device(Xh, dev)
    (xsq_a, hr_a), Sa, _, _ = _pair(sp, torch, X)
    sp.swiftprune_layer_stats_static(X[:1000], xsq_a, Sa, None, accumulate=False, finalize=False)
    sp.swiftprune_layer_stats_static(X[1000:], xsq_a, Sa, hr_a, accumulate=True, finalize=True)
    torch.cuda.synchronize()
    xsq_o, S_o, hr_o = orc.layer_stats(Xh)
    assert np.allclose(xsq_a.cpu().numpy(), xsq_o, rtol=1e-5, atol=0)
    assert np.allclose(hr_a.cpu().numpy(), hr_o, rtol=1e-5, atol=0)

    # a shape whose partial sums do not fit the array is refused on the host, nothing is enqueued
    need = sp.swiftprune_stats_workspace_bytes(8, 4_000_000)
    assert need > (8 << 20)
    big = torch.zeros((1, 8), dtype=torch.float32, device=dev)       # never read: the call must fail first
    rc = L.swiftprune_layer_stats_static(big.data_ptr(), 8, 4_000_000, 4_000_000, sp.SP_F32, xsq_a.data_ptr(),
                                         Sa.data_ptr(), hr_a.data_ptr(), 0, 1, None)
    assert rc == sp.SP_ENOSPC
