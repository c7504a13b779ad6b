"""GPU parity: every entry point of the C-ABI library against the CPU oracle, element by element,
on the same seeded inputs.

Bars:
  * masks from the strict-order EWMA kernel and from N:M selection, scores, apply: bit-exact when
    both sides are given the same channel factor;
  * statistics (xsq, S, hr): 1e-5 relative (fp32 partial sums on the GPU, fp64 in the oracle);
  * masks from the scan kernel (or from GPU statistics): a bit may differ only where the oracle's
    score is within 1e-5 relative of the oracle's threshold for that element (gpu_util.TOL).
"""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

A, B = 0.125, 0.125


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2501_16376_amd import binding
    binding.load_library()
    return torch.device("cuda:0")


def _stats_gpu(X_dev, n, accumulate_chunks=None):
    import torch
    from paper_2501_16376_amd import binding as b
    xsq = torch.empty(n, dtype=torch.float32, device=X_dev.device)
    S = torch.empty(1, dtype=torch.float32, device=X_dev.device)
    hr = torch.empty(n, dtype=torch.float32, device=X_dev.device)
    if accumulate_chunks is None:
        b.swiftprune_layer_stats(X_dev, xsq, S, hr)
    else:
        bounds = accumulate_chunks
        for i in range(len(bounds) - 1):
            b.swiftprune_layer_stats(X_dev[bounds[i]:bounds[i + 1]], xsq, S, hr, accumulate=(i > 0),
                                     finalize=(i == len(bounds) - 2))
    torch.cuda.synchronize()
    return xsq.cpu().numpy(), float(S.cpu().numpy()[0]), hr.cpu().numpy()


def _select_gpu(W_dev, hr_dev, la, flags=0, want_scores=False, alpha=A, beta=B):
    import torch
    from paper_2501_16376_amd import binding as b
    from gpu_util import mask_to_host
    out, n = W_dev.shape
    mask = torch.full((out, (n + 31) // 32), -1, dtype=torch.int32, device=W_dev.device)
    cnt = torch.full((out,), -7, dtype=torch.int32, device=W_dev.device)
    sc = torch.empty((out, n), dtype=torch.float32, device=W_dev.device) if want_scores else None
    b.swiftprune_score_select(W_dev, hr_dev, mask, alpha=alpha, beta=beta, la=la, row_pruned=cnt,
                              scores=sc, flags=flags)
    torch.cuda.synchronize()
    return mask_to_host(mask), cnt.cpu().numpy(), (None if sc is None else sc.cpu().numpy())


def _nm_gpu(W_dev, hr_dev, nk, m, flags=0, want_scores=False):
    import torch
    from paper_2501_16376_amd import binding as b
    from gpu_util import mask_to_host
    out, n = W_dev.shape
    mask = torch.full((out, (n + 31) // 32), -1, dtype=torch.int32, device=W_dev.device)
    sc = torch.empty((out, n), dtype=torch.float32, device=W_dev.device) if want_scores else None
    b.swiftprune_nm_select(W_dev, hr_dev, nk, m, mask, scores=sc, flags=flags)
    torch.cuda.synchronize()
    return mask_to_host(mask), (None if sc is None else sc.cpu().numpy())


def _layer_case(orc, gpu, out, n, tokens, dtype, seed, las=(0.5,), nms=((2, 4), (4, 8)), pitch_pad=0,
                n_outlier=None):
    """Full parity of one layer shape; returns the number of tolerated scan-vs-oracle differences."""
    import torch
    from paper_2501_16376_amd import binding as b, synth
    from gpu_util import to_device, check_ewma_mask, mask_to_host, same_bits
    say(f"[case] out={out} in={n} tokens={tokens} dtype={dtype} seed={seed} pad={pitch_pad}")
    Wh, Xh = synth.layer_inputs(out, n, tokens, seed=seed, dtype=dtype, n_outlier=n_outlier)
    if pitch_pad:
        Wp = np.zeros((out, n + pitch_pad), dtype=Wh.dtype)
        Wp[:, :n] = Wh
        Xp = np.full((tokens, n + pitch_pad), 0x4000 if dtype == "bf16" else 2.0, dtype=Xh.dtype)
        Xp[:, :n] = Xh
        W_dev = to_device(Wp, gpu)[:, :n]
        X_dev = to_device(Xp, gpu)[:, :n]
    else:
        W_dev, X_dev = to_device(Wh, gpu), to_device(Xh, gpu)

    # --- step 1
    xsq_o, S_o, hr_o = orc.layer_stats(Xh)
    xsq_g, S_g, hr_g = _stats_gpu(X_dev, n)
    assert np.allclose(xsq_g, xsq_o, rtol=1e-5, atol=0), np.abs(xsq_g / xsq_o - 1).max()
    assert abs(S_g - S_o) <= 1e-5 * abs(S_o)
    assert np.allclose(hr_g, hr_o, rtol=1e-5, atol=0)
    hr_dev = to_device(hr_o, gpu)

    tolerated = 0
    for la in las:
        # --- strict order, same factor: bit-exact masks, counts and scores
        mask_o, cnt_o, sc_o = orc.ewma_select(Wh, hr_o, A, B, la, want_scores=True)
        m_seq, c_seq, sc_seq = _select_gpu(W_dev, hr_dev, la, flags=b.SP_SEQUENTIAL_ORDER, want_scores=True)
        assert np.array_equal(m_seq, mask_o), f"strict-order mask differs, la={la}"
        assert np.array_equal(c_seq, cnt_o)
        assert np.array_equal(sc_seq.view(np.uint32), sc_o.view(np.uint32))
        # --- scan path, same factor: rounding-level differences only
        m_scan, c_scan, sc_scan = _select_gpu(W_dev, hr_dev, la, want_scores=True)
        assert np.array_equal(sc_scan.view(np.uint32), sc_o.view(np.uint32))
        tolerated += check_ewma_mask(orc, Wh, hr_o, A, B, la, m_scan, c_scan)
        # --- the same call without the scores output: aligned layouts take the fast kernel here
        m_fast, c_fast, _ = _select_gpu(W_dev, hr_dev, la)
        tolerated += check_ewma_mask(orc, Wh, hr_o, A, B, la, m_fast, c_fast)
        # --- scan path on the GPU's own statistics (end to end)
        m_e2e, c_e2e, sc_e2e = _select_gpu(W_dev, to_device(hr_g, gpu), la, want_scores=True)
        assert np.allclose(sc_e2e, sc_o, rtol=1e-5, atol=0)
        tolerated += check_ewma_mask(orc, Wh, hr_o, A, B, la, m_e2e, c_e2e)

    # --- N:M: bit-exact with the same factor
    for nk, m in nms:
        if n % m:
            continue
        nm_o, nsc_o = orc.nm_select(Wh, hr_o, nk, m, want_scores=True)
        nm_g, nsc_g = _nm_gpu(W_dev, hr_dev, nk, m, want_scores=True)
        assert np.array_equal(nm_g, nm_o), f"{nk}:{m} mask differs"
        assert np.array_equal(nsc_g.view(np.uint32), nsc_o.view(np.uint32))

    # --- apply, separate and fused
    mask_o, _, _ = orc.ewma_select(Wh, hr_o, A, B, las[0])
    ref = orc.apply(Wh.copy(), mask_o)
    W1 = W_dev.clone() if not pitch_pad else to_device(Wp, gpu)[:, :n]
    b.swiftprune_apply(W1, to_device(mask_o.view(np.int32), gpu))
    torch.cuda.synchronize()
    assert same_bits(synth.torch_to_host_bits(W1), ref)
    W2 = W_dev.clone() if not pitch_pad else to_device(Wp, gpu)[:, :n]
    mk = torch.empty((out, (n + 31) // 32), dtype=torch.int32, device=gpu)
    b.swiftprune_score_select(W2, hr_dev, mk, la=las[0], flags=b.SP_APPLY_INPLACE | b.SP_SEQUENTIAL_ORDER)
    torch.cuda.synchronize()
    assert same_bits(synth.torch_to_host_bits(W2), ref)
    W3 = W_dev.clone() if not pitch_pad else to_device(Wp, gpu)[:, :n]
    b.swiftprune_score_select(W3, hr_dev, mk, la=las[0], flags=b.SP_APPLY_INPLACE)
    torch.cuda.synchronize()
    # the fused mask against the oracle's under the threshold rule, and the zeroed weights against the
    # oracle's apply of that mask: together they tie the fused result to the oracle, not to itself
    check_ewma_mask(orc, Wh, hr_o, A, B, las[0], mask_to_host(mk))
    assert same_bits(synth.torch_to_host_bits(W3), orc.apply(Wh.copy(), mask_to_host(mk)))
    if n % 4 == 0:
        nm_o, _ = orc.nm_select(Wh, hr_o, 2, 4)
        W4 = W_dev.clone() if not pitch_pad else to_device(Wp, gpu)[:, :n]
        b.swiftprune_nm_select(W4, hr_dev, 2, 4, mk, flags=b.SP_APPLY_INPLACE)
        torch.cuda.synchronize()
        assert same_bits(synth.torch_to_host_bits(W4), orc.apply(Wh.copy(), nm_o))
    if pitch_pad:                                                     # padding columns untouched
        for Wt in (W1, W2, W3):
            full = synth.torch_to_host_bits(Wt._base if Wt._base is not None else Wt)
            assert np.all(full[:, n:] == 0)
    return tolerated


def test_config1_fp32(orc, gpu):
    """The small case: W 256x256 fp32, X 128x256 fp32, 4 outlier channels, every la of the paper's table."""
    t = _layer_case(orc, gpu, 256, 256, 128, "f32", seed=0, las=(0.5, 0.2, -0.2, -0.9, -1.5),
                    nms=((2, 4), (4, 8), (1, 4), (3, 4), (8, 16)), n_outlier=4)
    say(f"config 1: {t} tolerated scan differences")


@pytest.mark.parametrize("out,n,tokens,dtype,pad", [
    (300, 1376, 5000, "bf16", 0),      # several 512-column segments + ragged tail; rows not a multiple of 4/8
    (70, 2056, 1111, "bf16", 0),       # in % 8 == 0 but not % 32
    (33, 1001, 777, "bf16", 0),        # odd width: element-wise path
    (65, 1000, 300, "bf16", 24),       # row pitch > columns (strided view), vector path
    (19, 999, 300, "f32", 5),          # fp32, odd width and odd pitch
    (129, 520, 2100, "f32", 0),        # fp32 vector path
    (5, 8, 3, "bf16", 0),              # one chunk
    (3, 1, 1, "f32", 0),               # a single column, a single token
    (1, 4096, 64, "bf16", 0),          # a single row
    (300, 1376, 5000, "f16", 0),       # IEEE half storage: vector path
    (33, 1001, 777, "f16", 0),         # IEEE half, element-wise path
    (65, 1000, 300, "f16", 24),        # IEEE half, padded pitch
    (1300, 4104, 64, "bf16", 0),       # two wavefronts per row, three spans, the last one ragged
    (40, 9000, 64, "bf16", 0),         # four wavefronts per row, three spans, rows not a multiple of 4
    (1100, 1032, 64, "f32", 8),        # two wavefronts per row, fp32, padded pitch
])
def test_shapes(orc, gpu, out, n, tokens, dtype, pad):
    t = _layer_case(orc, gpu, out, n, tokens, dtype, seed=out + n, pitch_pad=pad,
                    nms=((2, 4), (4, 8), (1, 4), (6, 8), (4, 16)))
    say(f"  tolerated scan differences: {t}")


def test_random_small_shapes(orc, gpu):
    """Forty-eight seeded random shapes (1-40 rows, 1-1500 columns, 1-200 tokens, three storage types, random row pitch):
    statistics to 1e-5, strict-order / N:M / apply bit-exact, scan path under the rounding rule."""
    import torch
    from paper_2501_16376_amd import binding as b, synth
    from gpu_util import to_device, check_ewma_mask, mask_to_host, same_bits
    rng = np.random.default_rng(2024)
    for case in range(48):
        out = int(rng.integers(1, 41))
        n = int(rng.integers(1, 1501))
        if case % 3 == 0:
            n = max(8, n // 8 * 8)                                    # exercise the vector path too
        tokens = int(rng.integers(1, 201))
        dtype = ("bf16", "f32", "f16")[(case // 3 + case) % 3]
        pad = int(rng.choice([0, 0, 8, 3]))
        la = float(rng.choice([0.5, 0.2, -0.2, -0.9, 1.1]))
        say(f"[case {case}] out={out} in={n} tokens={tokens} {dtype} pad={pad} la={la}")
        Wh, Xh = synth.layer_inputs(out, n, tokens, seed=5000 + case, dtype=dtype)
        Wp = np.zeros((out, n + pad), dtype=Wh.dtype)
        Wp[:, :n] = Wh
        Xp = np.zeros((tokens, n + pad), dtype=Xh.dtype)
        Xp[:, :n] = Xh
        W_dev, X_dev = to_device(Wp, gpu)[:, :n], to_device(Xp, gpu)[:, :n]
        xsq_o, S_o, hr_o = orc.layer_stats(Xh)
        xsq_g, S_g, hr_g = _stats_gpu(X_dev, n)
        assert np.allclose(xsq_g, xsq_o, rtol=1e-5, atol=0) and abs(S_g - S_o) <= 1e-5 * abs(S_o)
        assert np.allclose(hr_g, hr_o, rtol=1e-5, atol=0)
        hr_dev = to_device(hr_o, gpu)
        mask_o, cnt_o, _ = orc.ewma_select(Wh, hr_o, A, B, la)
        m_seq, c_seq, _ = _select_gpu(W_dev, hr_dev, la, flags=b.SP_SEQUENTIAL_ORDER)
        assert np.array_equal(m_seq, mask_o) and np.array_equal(c_seq, cnt_o)
        m_scan, c_scan, _ = _select_gpu(W_dev, hr_dev, la)
        check_ewma_mask(orc, Wh, hr_o, A, B, la, m_scan, c_scan)
        for nk, m in ((2, 4), (4, 8), (5, 16)):
            if n % m == 0:
                nm_g, _ = _nm_gpu(W_dev, hr_dev, nk, m)
                assert np.array_equal(nm_g, orc.nm_select(Wh, hr_o, nk, m)[0]), (nk, m)
        W2 = to_device(Wp, gpu)[:, :n]
        mk = torch.empty((out, (n + 31) // 32), dtype=torch.int32, device=gpu)
        b.swiftprune_score_select(W2, hr_dev, mk, la=la, flags=b.SP_APPLY_INPLACE)
        torch.cuda.synchronize()
        assert same_bits(synth.torch_to_host_bits(W2), orc.apply(Wh.copy(), mask_to_host(mk)))
        assert np.all(synth.torch_to_host_bits(W2._base)[:, n:] == 0)


def test_other_alpha_beta(orc, gpu):
    """alpha != beta, large and small decay, negative and large la."""
    from paper_2501_16376_amd import binding as b, synth
    from gpu_util import to_device, check_ewma_mask
    Wh, Xh = synth.layer_inputs(64, 1536, 256, seed=77, dtype="bf16")
    _, _, hr_o = orc.layer_stats(Xh)
    W_dev, hr_dev = to_device(Wh, gpu), to_device(hr_o, gpu)
    for alpha, beta, la in [(0.3, 0.07, -0.9), (0.02, 0.5, 0.4), (1.0, 1.0, 0.1), (0.9, 0.01, 2.0),
                            (0.125, 0.25, 4.0), (0.001, 0.001, 0.0)]:
        say(f"[case] alpha={alpha} beta={beta} la={la}")
        mask_o, cnt_o, _ = orc.ewma_select(Wh, hr_o, alpha, beta, la)
        m_seq, c_seq, _ = _select_gpu(W_dev, hr_dev, la, flags=b.SP_SEQUENTIAL_ORDER, alpha=alpha, beta=beta)
        assert np.array_equal(m_seq, mask_o) and np.array_equal(c_seq, cnt_o)
        m_scan, c_scan, _ = _select_gpu(W_dev, hr_dev, la, alpha=alpha, beta=beta)
        check_ewma_mask(orc, Wh, hr_o, alpha, beta, la, m_scan, c_scan)


def test_la_from_sparsity(orc, gpu):
    """la = NaN -> looked up from the sparsity argument (paper's table)."""
    import torch
    from paper_2501_16376_amd import binding as b, synth
    from gpu_util import to_device, mask_to_host
    Wh, Xh = synth.layer_inputs(32, 512, 128, seed=5, dtype="bf16")
    _, _, hr_o = orc.layer_stats(Xh)
    W_dev, hr_dev = to_device(Wh, gpu), to_device(hr_o, gpu)
    mask = torch.empty((32, 16), dtype=torch.int32, device=gpu)
    b.swiftprune_score_select(W_dev, hr_dev, mask, sparsity=0.7, la=None, flags=b.SP_SEQUENTIAL_ORDER)
    torch.cuda.synchronize()
    mask_o, _, _ = orc.ewma_select(Wh, hr_o, A, B, -0.2)
    assert np.array_equal(mask_to_host(mask), mask_o)


def test_stats_chunked_and_deterministic(orc, gpu):
    """Token chunks accumulate to the one-shot result; repeated runs are bit-identical."""
    from paper_2501_16376_amd import synth
    from gpu_util import to_device
    Wh, Xh = synth.layer_inputs(1, 2048, 9000, seed=9, dtype="bf16")
    X_dev = to_device(Xh, gpu)
    xsq_o, S_o, hr_o = orc.layer_stats(Xh)
    one = _stats_gpu(X_dev, 2048)
    two = _stats_gpu(X_dev, 2048)
    assert np.array_equal(one[0], two[0]) and one[1] == two[1] and np.array_equal(one[2], two[2])
    chunked = _stats_gpu(X_dev, 2048, accumulate_chunks=[0, 1000, 4097, 9000])
    assert np.allclose(chunked[0], xsq_o, rtol=1e-5, atol=0)
    assert abs(chunked[1] - S_o) <= 1e-5 * S_o
    assert np.allclose(chunked[2], hr_o, rtol=1e-5, atol=0)


@pytest.mark.parametrize("tokens,n,dtype", [(37, 40000, "bf16"), (5, 70001, "f32"), (4099, 8, "bf16"),
                                             (100000, 64, "f32"), (9, 2049, "bf16")])
def test_stats_wide_and_tall(orc, gpu, tokens, n, dtype):
    """Statistics on shapes far from the Llama ones: many strips with one token range, a single narrow
    strip with many ranges, odd widths on the element-wise path."""
    from paper_2501_16376_amd import synth
    from gpu_util import to_device
    say(f"[case] stats tokens={tokens} in={n} {dtype}")
    _, Xh = synth.layer_inputs(1, n, tokens, seed=tokens + n, dtype=dtype)
    xsq_o, S_o, hr_o = orc.layer_stats(Xh)
    xsq_g, S_g, hr_g = _stats_gpu(to_device(Xh, gpu), n)
    assert np.allclose(xsq_g, xsq_o, rtol=1e-5, atol=0)
    assert abs(S_g - S_o) <= 1e-5 * S_o
    assert np.allclose(hr_g, hr_o, rtol=1e-5, atol=0)


def test_graph_capture_replays(orc, gpu):
    """The whole layer path (statistics, selection + apply) records into a HIP graph - the library
    allocates nothing and never synchronises - and every replay reproduces the eager result, with eager
    work and synchronisations between the replays."""
    import torch
    from paper_2501_16376_amd import binding as b, synth
    from gpu_util import mask_to_host, same_bits
    out, n, tokens = 512, 2048, 4096
    X = synth.device_activations(tokens, n, seed=21, device=gpu)
    W0 = synth.device_weights(out, n, seed=22, device=gpu)
    bufs = b.LayerBuffers(out, n, tokens, gpu)
    # eager reference
    W = W0.clone()
    b.prune_layer(W, X, bufs, la=0.5)
    torch.cuda.synchronize()
    ref_W, ref_mask = synth.torch_to_host_bits(W), mask_to_host(bufs.keep_mask).copy()
    ref_hr = bufs.hr.cpu().numpy().copy()
    # capture
    Wg = W0.clone()
    side = torch.cuda.Stream(device=gpu)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        b.prune_layer(Wg, X, bufs, la=0.5)                 # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        b.prune_layer(Wg, X, bufs, la=0.5)
    for rep in range(3):
        Wg.copy_(W0)                                       # eager work between replays
        bufs.keep_mask.zero_()
        bufs.hr.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(bufs.hr.cpu().numpy(), ref_hr), rep
        assert np.array_equal(mask_to_host(bufs.keep_mask), ref_mask), rep
        assert same_bits(synth.torch_to_host_bits(Wg), ref_W), rep


def test_degenerate_statistics(orc, gpu):
    """All-zero activations -> S = 0, factor 1/2; one channel holding all the energy -> clamped denominator."""
    import torch
    X = torch.zeros((64, 256), dtype=torch.bfloat16, device=gpu)
    xsq, S, hr = _stats_gpu(X, 256)
    assert np.all(xsq == 0) and S == 0 and np.all(hr == 0.5)
    X[:, 7] = 3.0
    xsq, S, hr = _stats_gpu(X, 256)
    xsq_o, S_o, hr_o = orc.layer_stats(X.cpu().view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(xsq, xsq_o) and S == S_o and np.array_equal(hr, hr_o)
    assert hr[7] == np.float32(0.5) / np.finfo(np.float32).eps


def test_all_ones_exact(orc, gpu):
    """All-ones input: xsq = T, S = T*in, factor exactly 0.5/(1 - 1/in) - exact in fp32."""
    import torch
    X = torch.ones((4096, 1024), dtype=torch.bfloat16, device=gpu)
    xsq, S, hr = _stats_gpu(X, 1024)
    assert np.all(xsq == 4096.0) and S == 4096.0 * 1024
    assert np.all(hr == np.float32(0.5) / (np.float32(1) - np.float32(1 / 1024)))


def _full_size_layer(orc, gpu, out, n, seed, las=(0.5,), dtype="bf16"):
    """A Llama-sized layer at the full 128x2048 calibration tokens, in the launch configuration the
    benchmark times.  The oracle sees the same bits (copied to the host in token chunks) and computes
    everything itself; nothing it is given comes from the GPU path."""
    import torch
    from paper_2501_16376_amd import binding as b, synth
    from gpu_util import to_device, check_ewma_mask, same_bits
    tokens = synth.CALIB_TOKENS
    say(f"[full] out={out} in={n} tokens={tokens}: generating")
    X = synth.device_activations(tokens, n, seed=seed, device=gpu, dtype=dtype)
    W = synth.device_weights(out, n, seed=seed + 1, device=gpu, dtype=dtype)
    xsq_g, S_g, hr_g = _stats_gpu(X, n)
    say("[full] statistics on the oracle")
    acc = None
    for t0 in range(0, tokens, 32768):
        acc = orc.stats_accumulate(synth.torch_to_host_bits(X[t0:t0 + 32768]), acc)
    xsq_o, S_o = orc.stats_finalize(acc)
    hr_o = orc.channel_factor_f32(xsq_o, S_o)
    assert np.allclose(xsq_g, xsq_o, rtol=1e-5, atol=0), np.abs(xsq_g / xsq_o - 1).max()
    assert abs(S_g - S_o) <= 1e-5 * S_o
    assert np.allclose(hr_g, hr_o, rtol=1e-5, atol=0)
    say(f"[full] xsq max rel err {np.abs(xsq_g / xsq_o - 1).max():.2e}, S rel err {abs(S_g / S_o - 1):.2e}")
    assert np.abs(xsq_g / xsq_o - 1).max() <= 1e-6 and abs(S_g / S_o - 1) <= 1e-6   # far inside the 1e-5 bar
    del X
    torch.cuda.empty_cache()
    Wh = synth.torch_to_host_bits(W)
    hr_dev = to_device(hr_o, gpu)
    for la in las:
        say(f"[full] la={la}: strict-order selection")
        mask_o, cnt_o, _ = orc.ewma_select(Wh, hr_o, A, B, la)
        m_seq, c_seq, _ = _select_gpu(W, hr_dev, la, flags=b.SP_SEQUENTIAL_ORDER)
        assert np.array_equal(m_seq, mask_o) and np.array_equal(c_seq, cnt_o)
        say(f"[full] la={la}: scan selection")
        m_scan, c_scan, _ = _select_gpu(W, hr_dev, la)
        t = check_ewma_mask(orc, Wh, hr_o, A, B, la, m_scan, c_scan)
        say(f"[full] la={la}: scan vs oracle: {t} tolerated differences of {out * n} weights; "
            f"sparsity {cnt_o.sum() / (out * n):.4f}")
    m_scan, c_scan, _ = _select_gpu(W, hr_dev, 0.5)
    for nk, m in ((2, 4), (4, 8)):
        nm_o, _ = orc.nm_select(Wh, hr_o, nk, m)
        nm_g, _ = _nm_gpu(W, hr_dev, nk, m)
        assert np.array_equal(nm_g, nm_o)
    # fused select + apply as the benchmark runs it
    W2 = W.clone()
    bufs = b.LayerBuffers(out, n, 16, gpu)
    b.swiftprune_score_select(W2, hr_dev, bufs.keep_mask, la=0.5, row_pruned=bufs.row_pruned,
                              flags=b.SP_APPLY_INPLACE)
    torch.cuda.synchronize()
    from gpu_util import mask_to_host
    assert np.array_equal(mask_to_host(bufs.keep_mask), m_scan)
    assert same_bits(synth.torch_to_host_bits(W2), orc.apply(Wh.copy(), m_scan))


def test_full_size_q_proj(orc, gpu):
    _full_size_layer(orc, gpu, 4096, 4096, seed=100)


def test_full_size_kv_proj_8b(orc, gpu):
    _full_size_layer(orc, gpu, 1024, 4096, seed=200)


def test_full_size_gate_8b(orc, gpu):
    _full_size_layer(orc, gpu, 14336, 4096, seed=300)


def test_full_size_down_8b(orc, gpu):
    _full_size_layer(orc, gpu, 4096, 14336, seed=400)


def test_full_size_down_7b(orc, gpu):
    _full_size_layer(orc, gpu, 4096, 11008, seed=500)


def test_full_size_gate_7b(orc, gpu):
    _full_size_layer(orc, gpu, 11008, 4096, seed=600)


# Llama-2-70B-shaped layers (hidden 8192, intermediate 28672): the table's la for 50 % and 70 %
def test_full_size_q_proj_13b(orc, gpu):
    """5120 columns: three strips whose last wavefront is a third full (4 rows in flight, 512 workgroups)."""
    _full_size_layer(orc, gpu, 5120, 5120, seed=160)


def test_full_size_qkv_pythia(orc, gpu):
    """2560 columns: two strips of 160 lanes (16 rows in flight per lane)."""
    _full_size_layer(orc, gpu, 7680, 2560, seed=170)


def test_full_size_gate_8b_fp16(orc, gpu):
    _full_size_layer(orc, gpu, 14336, 4096, seed=150, dtype="f16")


def test_full_size_q_proj_70b(orc, gpu):
    _full_size_layer(orc, gpu, 8192, 8192, seed=700, las=(0.5, -0.2))


def test_full_size_kv_proj_70b(orc, gpu):
    _full_size_layer(orc, gpu, 1024, 8192, seed=800)


def test_full_size_gate_70b(orc, gpu):
    _full_size_layer(orc, gpu, 28672, 8192, seed=900)


def test_full_size_down_70b(orc, gpu):
    _full_size_layer(orc, gpu, 8192, 28672, seed=1000, las=(0.5, -0.2))


def test_matrix_beyond_4g_elements(orc, gpu):
    """Index arithmetic past 2^32 elements: a 66000 x 65536 bf16 matrix (4.3e9 weights; row 65536 starts at
    element 2^32 exactly).  Rows are independent, so rows on both sides of the boundary are checked
    against the oracle one by one: EWMA (strict order and scan), 2:4, and the in-place apply."""
    import torch
    from paper_2501_16376_amd import binding as b, synth
    from gpu_util import to_device, check_ewma_mask, mask_to_host, same_bits
    out, n = 66000, 65536
    say(f"[case] {out} x {n} bf16: generating")
    g = torch.Generator(device=gpu)
    g.manual_seed(4242)
    W = torch.empty((out, n), device=gpu, dtype=torch.bfloat16)
    buf = torch.empty((6000, n), device=gpu, dtype=torch.float32)
    for r0 in range(0, out, 6000):
        buf.normal_(0.0, synth.W_STD, generator=g)
        W[r0:r0 + 6000].copy_(buf[:min(6000, out - r0)])
    del buf
    rng = np.random.default_rng(7)
    hr = (0.5 / (1.0 - rng.uniform(0.0, 0.02, n))).astype(np.float32)
    hr_dev = to_device(hr, gpu)
    rows = [0, 1, 32767, 32768, 65535, 65536, 65537, out - 1]
    Wh = synth.torch_to_host_bits(W[rows])
    words = n // 32
    mask = torch.empty((out, words), dtype=torch.int32, device=gpu)
    cnt = torch.empty(out, dtype=torch.int32, device=gpu)

    say("[case] strict-order selection")
    b.swiftprune_score_select(W, hr_dev, mask, la=0.5, row_pruned=cnt, flags=b.SP_SEQUENTIAL_ORDER)
    torch.cuda.synchronize()
    mask_o, cnt_o, _ = orc.ewma_select(Wh, hr, A, B, 0.5)
    assert np.array_equal(mask_to_host(mask[rows]), mask_o)
    assert np.array_equal(cnt[rows].cpu().numpy(), cnt_o)

    say("[case] 2:4 selection")
    b.swiftprune_nm_select(W, hr_dev, 2, 4, mask)
    torch.cuda.synchronize()
    nm_o, _ = orc.nm_select(Wh, hr, 2, 4)
    assert np.array_equal(mask_to_host(mask[rows]), nm_o)
    say("[case] apply of the 2:4 mask on a copy of the matrix")
    W24 = W.clone()
    b.swiftprune_apply(W24, mask)
    torch.cuda.synchronize()
    assert same_bits(synth.torch_to_host_bits(W24[rows]), orc.apply(Wh.copy(), nm_o))
    del W24

    say("[case] scan selection fused with apply")
    b.swiftprune_score_select(W, hr_dev, mask, la=0.5, row_pruned=cnt, flags=b.SP_APPLY_INPLACE)
    torch.cuda.synchronize()
    m_scan = mask_to_host(mask[rows])
    t = check_ewma_mask(orc, Wh, hr, A, B, 0.5, m_scan, cnt[rows].cpu().numpy())
    say(f"[case] scan vs oracle on {len(rows)} rows: {t} tolerated differences")
    assert same_bits(synth.torch_to_host_bits(W[rows]), orc.apply(Wh.copy(), m_scan))
    total = int(cnt.to(torch.int64).sum().item())
    assert 0.45 < total / (out * n) < 0.60, total / (out * n)


def test_fp16_all_finite_bit_patterns(orc, gpu):
    """IEEE half storage with random finite bit patterns (subnormals, +-65504, both zeros) in X and W: the
    conversions in the streaming kernel (mixed-precision multiply-add), in the vector path and in the
    element-wise path are exact, so statistics stay within 1e-5 and scores / strict-order masks bit-exact."""
    import torch
    from paper_2501_16376_amd import binding as b
    from gpu_util import to_device, check_ewma_mask
    rng = np.random.default_rng(1616)
    for out, n, tokens in ((40, 2048, 300), (9, 1003, 77)):
        say(f"[case] fp16 bit patterns out={out} in={n} tokens={tokens}")
        def patterns(shape):
            bits = rng.integers(0, 1 << 16, size=shape, dtype=np.uint16)
            bits[(bits & 0x7c00) == 0x7c00] &= 0x83ff          # infinities and NaNs become subnormals
            return bits.view(np.float16)
        Xh, Wh = patterns((tokens, n)), patterns((out, n))
        Xh[:, 0] = np.float16(0.0)                              # a dead channel
        X_dev, W_dev = to_device(Xh, gpu), to_device(Wh, gpu)
        xsq_o, S_o, hr_o = orc.layer_stats(Xh)
        xsq_g, S_g, hr_g = _stats_gpu(X_dev, n)
        assert xsq_g[0] == 0.0 and xsq_o[0] == 0.0
        assert np.allclose(xsq_g, xsq_o, rtol=1e-5, atol=0) and abs(S_g - S_o) <= 1e-5 * S_o
        assert np.allclose(hr_g, hr_o, rtol=1e-5, atol=0)
        hr_dev = to_device(hr_o, gpu)
        mask_o, cnt_o, sc_o = orc.ewma_select(Wh, hr_o, A, B, 0.5, want_scores=True)
        m_seq, c_seq, sc_seq = _select_gpu(W_dev, hr_dev, 0.5, flags=b.SP_SEQUENTIAL_ORDER, want_scores=True)
        assert np.array_equal(sc_seq.view(np.uint32), sc_o.view(np.uint32))
        assert np.array_equal(m_seq, mask_o) and np.array_equal(c_seq, cnt_o)
        m_scan, c_scan, sc_scan = _select_gpu(W_dev, hr_dev, 0.5, want_scores=True)
        assert np.array_equal(sc_scan.view(np.uint32), sc_o.view(np.uint32))
        check_ewma_mask(orc, Wh, hr_o, A, B, 0.5, m_scan, c_scan)
        m_fast, c_fast, _ = _select_gpu(W_dev, hr_dev, 0.5)
        check_ewma_mask(orc, Wh, hr_o, A, B, 0.5, m_fast, c_fast)
        if n % 4 == 0:
            nm_g, _ = _nm_gpu(W_dev, hr_dev, 2, 4)
            assert np.array_equal(nm_g, orc.nm_select(Wh, hr_o, 2, 4)[0])
