"""Seeded synthetic inputs: Llama-shaped weight matrices and calibration activations.

These stand in for the trained weights and the calibration corpus used in the
paper's experiments (Sec. 4.1), which are not redistributed here.  The module
holds data generation and the bf16 storage format only - none of the pruning
method's arithmetic - so that the GPU path and the CPU checker can be fed the
same bits.

Recipe (every tensor):
  W[out, in]  ~ N(0, std 0.02)
  X[t, q]     = z[t, q] * s[q],  z ~ N(0, 1),  s[q] ~ lognormal(mu 0, sigma 0.5),
                and `n_outlier` channels (drawn without replacement by the same
                seeded generator) have s[q] multiplied by 50.
  bf16 tensors are generated in fp32 and rounded to nearest-even.
"""
from __future__ import annotations

import numpy as np

OUTLIER_GAIN = 50.0
W_STD = 0.02
SCALE_SIGMA = 0.5

# (name, out, in) of the seven linear layers of one decoder block
LLAMA2_7B_BLOCK = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                   ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
LLAMA3_8B_BLOCK = [("q", 4096, 4096), ("k", 1024, 4096), ("v", 1024, 4096), ("o", 4096, 4096),
                   ("gate", 14336, 4096), ("up", 14336, 4096), ("down", 4096, 14336)]
LLAMA2_70B_BLOCK = [("q", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192), ("o", 8192, 8192),
                    ("gate", 28672, 8192), ("up", 28672, 8192), ("down", 8192, 28672)]
# the other two models of the paper's main table (Sec. 4.1): LLaMA-2-13B (40 blocks) and Pythia-2.8B
# (32 blocks, GPT-NeoX layout: fused query/key/value, attention output, two MLP matrices)
LLAMA2_13B_BLOCK = [("q", 5120, 5120), ("k", 5120, 5120), ("v", 5120, 5120), ("o", 5120, 5120),
                    ("gate", 13824, 5120), ("up", 13824, 5120), ("down", 5120, 13824)]
PYTHIA_2_8B_BLOCK = [("qkv", 7680, 2560), ("dense", 2560, 2560), ("h_to_4h", 10240, 2560),
                     ("4h_to_h", 2560, 10240)]
MODEL_BLOCKS = {"llama3-8b": (LLAMA3_8B_BLOCK, 32), "llama2-7b": (LLAMA2_7B_BLOCK, 32),
                "llama2-13b": (LLAMA2_13B_BLOCK, 40), "llama2-70b": (LLAMA2_70B_BLOCK, 80),
                "pythia-2.8b": (PYTHIA_2_8B_BLOCK, 32)}
CALIB_TOKENS = 128 * 2048


def default_outliers(n_in: int) -> int:
    """0.1 % of the input channels (4 of 4096, 11 of 11008, 14 of 14336, 29 of 28672)."""
    return max(1, int(round(n_in * 0.001)))


# ------------------------------------------------------------------ bf16 storage
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ------------------------------------------------------------------ host (numpy) generator
def channel_scales(n_in: int, n_outlier: int, rng: np.random.Generator) -> np.ndarray:
    s = rng.lognormal(mean=0.0, sigma=SCALE_SIGMA, size=n_in)
    if n_outlier > 0:
        idx = rng.choice(n_in, size=n_outlier, replace=False)
        s[idx] *= OUTLIER_GAIN
    return s.astype(np.float32)


def layer_inputs(out: int, n_in: int, tokens: int, seed: int = 0, dtype: str = "bf16",
                 n_outlier: int | None = None):
    """(W, X) on the host.  dtype "f32" -> float32 arrays; "bf16" -> uint16 bit patterns; "f16" -> float16."""
    rng = np.random.default_rng(seed)
    if n_outlier is None:
        n_outlier = default_outliers(n_in)
    W = rng.normal(0.0, W_STD, size=(out, n_in)).astype(np.float32)
    s = channel_scales(n_in, n_outlier, rng)
    X = rng.standard_normal(size=(tokens, n_in), dtype=np.float32) * s[None, :]
    if dtype == "f32":
        return W, X
    if dtype == "bf16":
        return f32_to_bf16_bits(W), f32_to_bf16_bits(X)
    if dtype == "f16":
        return W.astype(np.float16), X.astype(np.float16)
    raise ValueError(dtype)


def config1(seed: int = 0):
    """The small single-layer case: W 256x256 fp32, X 128x256 fp32, 4 outlier channels."""
    return layer_inputs(256, 256, 128, seed=seed, dtype="f32", n_outlier=4)


# ------------------------------------------------------------------ device (torch) generator
def _torch_dtype(dtype: str):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype]


def device_weights(out: int, n_in: int, seed: int, device="cuda", dtype: str = "bf16"):
    """W on the device from a seeded device generator (torch is used for memory and RNG only)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    W = torch.empty((out, n_in), device=device, dtype=torch.float32)
    W.normal_(0.0, W_STD, generator=g)
    return W if dtype == "f32" else W.to(_torch_dtype(dtype))


def device_activations(tokens: int, n_in: int, seed: int, device="cuda", dtype: str = "bf16",
                       n_outlier: int | None = None, chunk_tokens: int = 8192):
    """X[tokens, in] on the device, generated in token chunks to bound the fp32 scratch."""
    import torch
    if n_outlier is None:
        n_outlier = default_outliers(n_in)
    rng = np.random.default_rng(seed)
    s = torch.from_numpy(channel_scales(n_in, n_outlier, rng)).to(device)
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) + 0x5EED)
    tdt = _torch_dtype(dtype)
    X = torch.empty((tokens, n_in), device=device, dtype=tdt)
    buf = torch.empty((min(chunk_tokens, tokens), n_in), device=device, dtype=torch.float32)
    for t0 in range(0, tokens, chunk_tokens):
        t1 = min(tokens, t0 + chunk_tokens)
        z = buf[: t1 - t0]
        z.normal_(0.0, 1.0, generator=g)
        z.mul_(s[None, :])
        X[t0:t1].copy_(z)
    return X


def torch_to_host_bits(t):
    """Device/host torch tensor -> numpy array the CPU checker accepts (uint16 bits for bf16)."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
