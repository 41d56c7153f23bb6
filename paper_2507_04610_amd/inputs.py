"""Seeded synthetic inputs for the any-n GEMM (shared by the tests, the benchmark
and the smoke check; used by neither the HIP kernels nor the CPU oracle).

This module draws random numbers and stores them in the on-disk/in-memory dtypes
of the problem statement.  It contains none of the method's arithmetic: no
packing, no table lookup, no dequantisation, no contraction.  The one numeric
helper it owns is the fp32 -> bf16 storage conversion of the *inputs*.

Recipe (stand-in for the quantised q/k/v/o/gate/up/down linears of a Llama
model, paper section 5 "Results", first paragraph):
  codes   uniform integers in [0, 2^bits), one per weight, uint8 [N, K]
  lut     2^bits samples of N(0, 1) per row, sorted ascending, bf16 [N, 2^bits]
  scale   U(0.005, 0.02) per (row, 128-wide group along K), bf16 [N, K/128]
  offset  N(0, 0.002)     per (row, 128-wide group along K), bf16 [N, K/128]
  x       N(0, 1) activations, bf16 [M, K]
Draw order with numpy's PCG64 `default_rng(seed)`: codes, lut, scale, offset, x.
bf16 tensors are carried as uint16 bit patterns.  With f16=True the same draws are stored as fp16.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

GROUP = 128  # the paper's default group size g along the reduction dimension

# (N, K) of the fused linears of one decoder layer
LLAMA3_8B_SHAPES = {
    "qkv": (6144, 4096),
    "o": (4096, 4096),
    "gate_up": (28672, 4096),
    "down": (4096, 14336),
}
LLAMA3_70B_SHAPES = {
    "qkv": (10240, 8192),
    "o": (8192, 8192),
    "gate_up": (57344, 8192),
    "down": (8192, 28672),
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (round-to-nearest-even), return uint16 bit patterns.
    Inputs are finite by construction."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def f32_to_f16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to fp16 (numpy's conversion: round-to-nearest-even), uint16 bit patterns."""
    return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen fp16 bit patterns to fp32 (exact)."""
    return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float32)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Case:
    """One GEMM problem, everything on the host as numpy arrays."""
    M: int
    N: int
    K: int
    bits: int
    seed: int
    codes_u8: np.ndarray   # uint8  [N, K], values < 2^bits
    lut: np.ndarray        # uint16 [N, 2^bits]  (bf16 bits)
    scale: np.ndarray      # uint16 [N, K/128]   (bf16 bits)
    offset: np.ndarray     # uint16 [N, K/128]   (bf16 bits)
    x: np.ndarray          # uint16 [M, K]       (bf16 bits)


def case_seed(base_seed: int, shape_index: int = 0, m_index: int = 0) -> int:
    """Distinct stream per (base seed, shape, M) point of a sweep."""
    return base_seed * 1000 + shape_index * 10 + m_index


def make_case(M: int, N: int, K: int, bits: int = 4, seed: int = 0, f16: bool = False) -> Case:
    """f16: the same draws stored as fp16 bit patterns (the paper's other 16-bit type, section 2.4.1)"""
    if K % GROUP != 0:
        raise ValueError("K must be a multiple of 128")
    if bits not in (2, 3, 4):
        raise ValueError("bits must be 2, 3 or 4")
    rng = np.random.default_rng(seed)
    L = 1 << bits
    G = K // GROUP
    codes = rng.integers(0, L, size=(N, K), dtype=np.uint8)
    lut = np.sort(rng.standard_normal((N, L), dtype=np.float32), axis=1)
    scale = rng.uniform(0.005, 0.02, size=(N, G)).astype(np.float32)
    offset = (rng.standard_normal((N, G), dtype=np.float32) * np.float32(0.002))
    x = rng.standard_normal((M, K), dtype=np.float32)
    store = f32_to_f16_bits if f16 else f32_to_bf16_bits
    return Case(M, N, K, bits, seed, codes, store(lut), store(scale), store(offset), store(x))


def make_case_device(M: int, N: int, K: int, bits: int = 4, seed: int = 0, device="cuda", f16: bool = False):
    """Same distributions drawn with torch's generator directly in device memory,
    for the full-size benchmark shapes (hundreds of MB of codes).  Returns a dict of
    torch tensors: codes_u8 uint8 [N,K]; lut/scale/offset/x as bf16 tensors."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    L = 1 << bits
    G = K // GROUP
    codes = torch.randint(0, L, (N, K), dtype=torch.uint8, device=device, generator=g)
    lut = torch.randn((N, L), dtype=torch.float32, device=device, generator=g).sort(dim=1).values
    scale = torch.empty((N, G), dtype=torch.float32, device=device).uniform_(0.005, 0.02, generator=g)
    offset = torch.randn((N, G), dtype=torch.float32, device=device, generator=g) * 0.002
    x = torch.randn((M, K), dtype=torch.float32, device=device, generator=g)
    dt = torch.float16 if f16 else torch.bfloat16
    return {
        "codes_u8": codes,
        "lut": lut.to(dt),
        "scale": scale.to(dt),
        "offset": offset.to(dt),
        "x": x.to(dt),
    }


@dataclass
class QuantCase:
    """One quantiser problem on the host: a weight matrix, the mean absolute activation of
    every input channel, and the uniform draws the k-means++ initialisation consumes."""
    N: int
    K: int
    bits: int
    seed: int
    w: np.ndarray      # float32 [N, K]
    act: np.ndarray    # float32 [K], > 0
    u: np.ndarray      # float32 [N, 2^bits], each in [0, 1)


def make_quant_case(N: int, K: int, bits: int = 4, seed: int = 0) -> QuantCase:
    """Stand-in for one linear layer of a language model and its calibration statistics
    (paper section 3.2, last paragraphs: weights of a linear module and the mean absolute
    activation per channel from one calibration sample):
      w    0.02 * Student-t(5): bell-shaped with heavy tails, float32 [N, K]
      act  0.05 + 0.5 * |N(0, 1)| per input channel, every 97th channel 10x larger
           (a few dominant channels), float32 [K]
      u    uniform [0, 1) draws, float32 [N, 2^bits]
    Draw order with numpy's PCG64 `default_rng(seed)`: w, act, u."""
    if K % GROUP != 0:
        raise ValueError("K must be a multiple of 128")
    rng = np.random.default_rng(seed)
    w = (rng.standard_t(5, size=(N, K)) * 0.02).astype(np.float32)
    act = (0.05 + 0.5 * np.abs(rng.standard_normal(K))).astype(np.float32)
    act[::97] *= np.float32(10.0)
    u = rng.random((N, 1 << bits), dtype=np.float32)
    return QuantCase(N, K, bits, seed, w, act, u)


def make_quant_case_device(N: int, K: int, bits: int = 4, seed: int = 0, device="cuda"):
    """The quantiser recipe drawn with torch's generator directly in device memory (full-size
    benchmark matrices): Student-t(5) = normal / sqrt(chi-square(5) / 5).  Returns a dict of
    float32 tensors w [N,K], act [K], u [N, 2^bits]."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    z = torch.randn((N, K), dtype=torch.float32, device=device, generator=g)
    chi = torch.zeros((N, K), dtype=torch.float32, device=device)
    for _ in range(5):
        chi += torch.randn((N, K), dtype=torch.float32, device=device, generator=g) ** 2
    w = 0.02 * z / torch.sqrt(chi / 5.0)
    del z, chi
    act = 0.05 + 0.5 * torch.randn((K,), dtype=torch.float32, device=device, generator=g).abs()
    act[::97] *= 10.0
    u = torch.rand((N, 1 << bits), dtype=torch.float32, device=device, generator=g)
    return {"w": w.contiguous(), "act": act.contiguous(), "u": u.contiguous()}
