"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the compression method: it only draws
weights with the shapes and value distributions of the paper's workloads
(Sec. 3: Llama-3 8B, Llama-3 70B; App. A: randomly initialised weights show the
same low-entropy exponents as trained ones) and hands out their raw bf16 bits.
Both the HIP path and the CPU oracle are fed from here and from nowhere else.
"""
import math

import numpy as np
import torch

BASE_SEED = 20241027


def seed_for(config: int, tensor_index: int = 0) -> int:
    return BASE_SEED + 1000 * config + tensor_index


def _generator(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def gaussian_bf16(n_or_shape, seed: int, std: float = 0.02, device="cpu") -> torch.Tensor:
    """i.i.d. N(0, std^2) drawn in fp32 and rounded to bf16 (round to nearest even)."""
    shape = (n_or_shape,) if isinstance(n_or_shape, int) else tuple(n_or_shape)
    g = _generator(seed, device)
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    return (x * std).to(torch.bfloat16)


def student_t4_bf16(n_or_shape, seed: int, std: float = 0.015, device="cpu") -> torch.Tensor:
    """Heavy-tailed weights: Student-t with 4 degrees of freedom scaled to the given std."""
    shape = (n_or_shape,) if isinstance(n_or_shape, int) else tuple(n_or_shape)
    g = _generator(seed, device)
    z = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    chi2 = torch.zeros(shape, device=device, dtype=torch.float32)
    for _ in range(4):
        chi2 += torch.randn(shape, generator=g, device=device, dtype=torch.float32) ** 2
    t = z / torch.sqrt(chi2 / 4.0)
    return (t * (std / math.sqrt(2.0))).to(torch.bfloat16)


def random_bits_bf16(n: int, seed: int, device="cpu") -> torch.Tensor:
    """Uniformly random 16-bit patterns: every exponent equally likely (worst case for the coder)."""
    g = _generator(seed, device)
    v = torch.randint(0, 65536, (n,), generator=g, device=device, dtype=torch.int32)
    return (v - 65536 * (v >= 32768)).to(torch.int16).view(torch.bfloat16)


def all_patterns_bf16(device="cpu") -> torch.Tensor:
    """All 65,536 bf16 bit patterns in ascending order (zeros, subnormals, Inf and NaN included)."""
    v = torch.arange(65536, dtype=torch.int32, device=device)
    return (v - 65536 * (v >= 32768)).to(torch.int16).view(torch.bfloat16)


def constant_bf16(n: int, value: float, device="cpu") -> torch.Tensor:
    return torch.full((n,), value, dtype=torch.bfloat16, device=device)


def synthetic_update(w: torch.Tensor, seed: int, std: float = 1e-4) -> torch.Tensor:
    """Stand-in for an optimiser step: w + N(0, std^2) in fp32, rounded back to the type of w."""
    g = _generator(seed, w.device)
    noise = torch.randn(w.shape, generator=g, device=w.device, dtype=torch.float32) * std
    return (w.float() + noise).to(w.dtype)


def gaussian_f32(n_or_shape, seed: int, std: float = 0.02, device="cpu") -> torch.Tensor:
    """i.i.d. N(0, std^2) in binary32: master weights or optimiser-side copies of the same layers."""
    shape = (n_or_shape,) if isinstance(n_or_shape, int) else tuple(n_or_shape)
    g = _generator(seed, device)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std


def all_upper_halves_f32(low: int, device="cpu") -> torch.Tensor:
    """The 65,536 binary32 words whose upper half runs over every pattern, all with the given lower half."""
    v = (torch.arange(65536, dtype=torch.int64, device=device) << 16) | int(low)
    return (v - (v >= 2 ** 31) * 2 ** 32).to(torch.int32).view(torch.float32)


def gaussian_f16(n_or_shape, seed: int, std: float = 0.02, device="cpu") -> torch.Tensor:
    """i.i.d. N(0, std^2) drawn in fp32 and rounded to binary16."""
    shape = (n_or_shape,) if isinstance(n_or_shape, int) else tuple(n_or_shape)
    g = _generator(seed, device)
    return (torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std).to(torch.float16)


def all_patterns_f16(device="cpu") -> torch.Tensor:
    """All 65,536 binary16 bit patterns in ascending order."""
    v = torch.arange(65536, dtype=torch.int32, device=device)
    return (v - 65536 * (v >= 32768)).to(torch.int16).view(torch.float16)


def bits16(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit words of a float16 tensor as a flat uint16 numpy array (host copy)."""
    assert t.dtype == torch.float16
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1)


def from_bits16(words: np.ndarray, device="cpu") -> torch.Tensor:
    w = np.ascontiguousarray(words, dtype=np.uint16).view(np.int16)
    return torch.from_numpy(w.copy()).to(device).view(torch.float16)


def bits32(t: torch.Tensor) -> np.ndarray:
    """Raw 32-bit words of a float32 tensor as a flat uint32 numpy array (host copy)."""
    assert t.dtype == torch.float32
    return t.detach().contiguous().view(torch.int32).cpu().numpy().view(np.uint32).reshape(-1)


def from_bits32(words: np.ndarray, device="cpu") -> torch.Tensor:
    w = np.ascontiguousarray(words, dtype=np.uint32).view(np.int32)
    return torch.from_numpy(w.copy()).to(device).view(torch.float32)


def bits(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit words of a bf16 tensor as a flat uint16 numpy array (host copy)."""
    assert t.dtype == torch.bfloat16
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1)


def from_bits(words: np.ndarray, device="cpu") -> torch.Tensor:
    w = np.ascontiguousarray(words, dtype=np.uint16).view(np.int16)
    return torch.from_numpy(w.copy()).to(device).view(torch.bfloat16)


# Shapes -----------------------------------------------------------------

MLP_8B = (4096, 14336)     # Llama-3 8B MLP projection
MLP_70B = (28672, 8192)    # Llama-3 70B MLP projection


def llama3_8b_tensors():
    """(name, shape) of every linear weight of a Llama-3-8B-shaped model in forward order."""
    out = [("embed", (128256, 4096))]
    per_layer = [("q", (4096, 4096)), ("k", (1024, 4096)), ("v", (1024, 4096)), ("o", (4096, 4096)),
                 ("gate", (14336, 4096)), ("up", (14336, 4096)), ("down", (4096, 14336))]
    for layer in range(32):
        for name, shape in per_layer:
            out.append((f"layers.{layer}.{name}", shape))
    return out
