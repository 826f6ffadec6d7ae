"""Seeded synthetic inputs shaped like the tensors of LLM linear layers.

Serves the tests, the smoke check and the benchmark.  It holds none of the HiF4
arithmetic: it only draws numbers (numpy Philox streams) and casts them to BF16
with torch's round-to-nearest-even.  The model weights and evaluation datasets the
paper measures accuracy on are not available here; these tensors stand in for
linear-layer weights (small-variance Gaussians, per-channel scale spread) and
activations (unit Gaussians or heavy tails with rare large outliers).

Every generator returns CPU ``torch.bfloat16`` tensors (row-major, K contiguous).
"""
import numpy as np
import torch

BASE_SEED = 0x48694634  # "HiF4"


def _rng(config: int, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(BASE_SEED + 16 * config + tensor))


def to_bf16(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)


def bits(t: torch.Tensor) -> np.ndarray:
    """BF16 tensor (CPU) -> numpy uint16 bit patterns, same shape, no copy."""
    assert t.dtype == torch.bfloat16 and t.device.type == "cpu"
    return t.view(torch.int16).numpy().view(np.uint16)


def from_bits(b: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(b).view(np.int16)).view(torch.bfloat16)


def gaussian_sweep(x: int, n: int = 1024) -> np.ndarray:
    """Matrix x of the quantisation-error study: n x n, N(0, (0.01 * 2^x)^2), fp64."""
    return _rng(0, x).standard_normal((n, n)) * (0.01 * 2.0 ** x)


def activation_with_outliers(rows: int = 1024, K: int = 4096, frac: float = 0.001,
                             boost: float = 64.0, config: int = 1, tensor: int = 0) -> torch.Tensor:
    """N(0,1) with floor(frac * rows * K) seeded positions multiplied by `boost`."""
    g = _rng(config, tensor)
    x = g.standard_normal((rows, K), dtype=np.float32)
    n_out = int(frac * rows * K)
    pos = g.choice(rows * K, size=n_out, replace=False)
    x.reshape(-1)[pos] *= boost
    return to_bf16(x)


def weight_gaussian(N: int, K: int, sigma: float, config: int, tensor: int = 1,
                    channel_scale: bool = False) -> torch.Tensor:
    """N(0, sigma^2); optionally each output row times a log-uniform [0.5, 2] factor."""
    g = _rng(config, tensor)
    w = g.standard_normal((N, K), dtype=np.float32) * np.float32(sigma)
    if channel_scale:
        c = np.exp(g.uniform(np.log(0.5), np.log(2.0), size=(N, 1))).astype(np.float32)
        w *= c
    return to_bf16(w)


def activation_gaussian(M: int, K: int, config: int, tensor: int = 0) -> torch.Tensor:
    return to_bf16(_rng(config, tensor).standard_normal((M, K), dtype=np.float32))


def activation_channel_outliers(M: int, K: int, frac: float = 0.001, boost: float = 64.0,
                                n_channels: int = 8, config: int = 3, tensor: int = 0) -> torch.Tensor:
    """N(0,1); floor(frac*M*K) entries, all inside `n_channels` seeded columns, times `boost`."""
    g = _rng(config, tensor)
    x = g.standard_normal((M, K), dtype=np.float32)
    cols = g.choice(K, size=n_channels, replace=False)
    n_out = min(int(frac * M * K), M * n_channels)
    pick = g.choice(M * n_channels, size=n_out, replace=False)
    x[pick // n_channels, cols[pick % n_channels]] *= boost
    return to_bf16(x)


def activation_student_t(M: int, K: int, nu: float = 4.0, config: int = 5, tensor: int = 0) -> torch.Tensor:
    """Student-t(nu) scaled to unit variance (variance of t_nu is nu / (nu - 2))."""
    g = _rng(config, tensor)
    x = g.standard_t(nu, size=(M, K)).astype(np.float32)
    x *= np.float32(1.0 / np.sqrt(nu / (nu - 2.0)))
    return to_bf16(x)


def moe_offsets(n_tokens: int = 1024, top_k: int = 8, E: int = 64, config: int = 4, tensor: int = 2) -> np.ndarray:
    """Each token picks top_k distinct experts uniformly; rows sorted by expert -> int32[E+1]."""
    g = _rng(config, tensor)
    counts = np.zeros(E, np.int64)
    for _ in range(n_tokens):
        counts[g.choice(E, size=top_k, replace=False)] += 1
    offs = np.zeros(E + 1, np.int32)
    offs[1:] = np.cumsum(counts)
    return offs
