"""Seeded synthetic inputs with the shapes and value distributions of the benchmark configurations.

This module only draws random tensors.  It holds none of the method's arithmetic (no SVD, no
dequantisation, no sampling transform) so that the CPU oracle and the HIP library, which share
no code, can both be fed the very same arrays.

Every tensor comes from numpy's PCG64 seeded with BASE_SEED + a tensor id, so any single tensor
(one layer's weights, say) can be regenerated on its own.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20250704
PROJ_NAMES = ("q", "k", "v", "o")

# tensor kinds inside one projection
_KIND_W, _KIND_SCALE, _KIND_ZERO, _KIND_A, _KIND_B, _KIND_V = range(6)
_X_ID_BASE = 1 << 20
_MISC_ID_BASE = 1 << 21


def _rng(tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + int(tensor_id)))


def _tid(layer: int, proj: int, kind: int) -> int:
    return (layer * 4 + proj) * 8 + kind


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (ties to even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + (np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1)))
    return (u >> np.uint64(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Projection:
    """Raw inputs of one adapted projection (nothing derived from them)."""
    name: str
    d_in: int
    d_out: int
    r: int
    quant: str                  # "int8" or "int4"
    Wq: np.ndarray              # int8 [d_out,d_in]  |  uint8 packed [d_out,d_in/2], low nibble = even column
    scales: np.ndarray          # fp32 [d_out]       |  fp16 [d_out,d_in/128]
    zeros: np.ndarray | None    # None               |  fp16 [d_out,d_in/128]
    A: np.ndarray               # fp32 [r,d_in]   ~ N(0, 1/d_in)
    B: np.ndarray               # fp32 [d_out,r]  ~ N(0, 0.01)


def make_projection(name: str, d_in: int, d_out: int, r: int, quant: str, layer: int = 0, proj: int = 0) -> Projection:
    if quant == "int8":
        Wq = _rng(_tid(layer, proj, _KIND_W)).integers(-127, 128, size=(d_out, d_in), dtype=np.int8)
        scales = _rng(_tid(layer, proj, _KIND_SCALE)).uniform(0.001, 0.01, size=d_out).astype(np.float32)
        zeros = None
    elif quant == "int4":
        assert d_in % 128 == 0
        # one random byte = two independent uniform nibbles
        Wq = _rng(_tid(layer, proj, _KIND_W)).integers(0, 256, size=(d_out, d_in // 2), dtype=np.uint8)
        scales = _rng(_tid(layer, proj, _KIND_SCALE)).uniform(0.001, 0.01, size=(d_out, d_in // 128)).astype(np.float16)
        zeros = _rng(_tid(layer, proj, _KIND_ZERO)).uniform(6.0, 9.0, size=(d_out, d_in // 128)).astype(np.float16)
    else:
        raise ValueError(quant)
    A = (_rng(_tid(layer, proj, _KIND_A)).standard_normal((r, d_in)) / np.sqrt(d_in)).astype(np.float32)
    B = (_rng(_tid(layer, proj, _KIND_B)).standard_normal((d_out, r)) * 0.1).astype(np.float32)
    return Projection(name, d_in, d_out, r, quant, Wq, scales, zeros, A, B)


def make_layer(hidden: int, kv: int, r: int, quant: str, layer: int = 0) -> list[Projection]:
    """q/o hidden x hidden, k/v kv x hidden."""
    outs = (hidden, kv, kv, hidden)
    return [make_projection(PROJ_NAMES[p], hidden, outs[p], r, quant, layer, p) for p in range(4)]


def make_x_f32(R: int, d_in: int, x_id: int = 0) -> np.ndarray:
    return _rng(_X_ID_BASE + x_id).standard_normal((R, d_in), dtype=np.float32)


def make_x_bf16(R: int, d_in: int, x_id: int = 0):
    """Returns (bits uint16 [R,d_in], values fp32 [R,d_in]); the values are exactly the bf16 numbers."""
    bits = f32_to_bf16_bits(make_x_f32(R, d_in, x_id))
    return bits, bf16_bits_to_f32(bits)


def row2cand_contiguous(K: int, rows_per_cand: int) -> np.ndarray:
    return (np.arange(K * rows_per_cand) // rows_per_cand).astype(np.int32)


def row2cand_interleaved(K: int, rows_per_cand: int, map_id: int = 0) -> np.ndarray:
    base = row2cand_contiguous(K, rows_per_cand)
    return base[_rng(_MISC_ID_BASE + map_id).permutation(base.shape[0])].astype(np.int32)


def reward_vector(d_out: int, layer: int, proj: int) -> np.ndarray:
    return (_rng(_tid(layer, proj, _KIND_V)).standard_normal(d_out) / np.sqrt(d_out)).astype(np.float32)


def sigma_perturbation(K: int, P: int, r: int, step: float, pert_id: int = 0):
    """Independent N(0, step^2) offsets for sigma_A and sigma_B, [K,P,r] each (used where a
    configuration gives candidates directly instead of through the sampler)."""
    g = _rng(_MISC_ID_BASE + 1000 + pert_id)
    return ((step * g.standard_normal((K, P, r))).astype(np.float32),
            (step * g.standard_normal((K, P, r))).astype(np.float32))


def random_covariance_basis(n: int, basis_id: int = 0):
    """Orthogonal Q (QR of a Gaussian matrix) and axis lengths d ~ logU(0.5, 2): a dense C = Q d^2 Q^T."""
    g = _rng(_MISC_ID_BASE + 2000 + basis_id)
    Q, Rm = np.linalg.qr(g.standard_normal((n, n)))
    Q = Q * np.sign(np.diag(Rm))[None, :]
    d = np.exp(g.uniform(np.log(0.5), np.log(2.0), size=n))
    return Q.astype(np.float32), d.astype(np.float32)


@dataclass(frozen=True)
class Config:
    name: str
    hidden: int
    kv: int
    r: int
    K: int
    rows_per_cand: int
    layers: int
    quant: str
    x_dtype: str
    interleaved: bool
    sigma_step: float

    @property
    def R(self) -> int:
        return self.K * self.rows_per_cand


CONFIGS = {
    # c1 is a single 512x512 projection; see tests for its sampler-driven sigma.
    "c1_tiny": Config("c1_tiny", 512, 512, 8, 4, 16, 1, "int8", "f32", False, 0.1),
    "c2_7b_decode": Config("c2_7b_decode", 3584, 512, 16, 32, 8, 28, "int8", "bf16", False, 0.05),
    "c3_32b_prefill": Config("c3_32b_prefill", 5120, 1024, 32, 64, 512, 1, "int8", "bf16", False, 0.05),
    "c4_72b_decode": Config("c4_72b_decode", 8192, 1024, 32, 128, 4, 80, "int4", "bf16", True, 0.05),
    "c5_7b_es_iter": Config("c5_7b_es_iter", 3584, 512, 16, 64, 512, 28, "int8", "bf16", False, 0.32),
}
