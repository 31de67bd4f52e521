"""Seeded synthetic workloads: the shapes of the paper's LLaMA models and the value
distributions that stand in for trained tensors.

This module holds no arithmetic of the method itself (no quantiser, no products of
the layer): it only draws random tensors.  Both the tests' CPU checker and the HIP
path are fed from it, so they see identical bits.

Shapes: hidden / intermediate sizes and ranks from the paper's table of pre-training
hyper-parameters (appendix "Hyperparamters", LLaMA 60M .. 13B); the 13B rank follows
the text of the paper's introduction (1024).  Distributions:
  W  fp32  N(0, sigma=0.02)                      (quantised to NF4 by the caller)
  P  fp32  Q factor of the reduced QR of an out x r standard Gaussian
           (stands in for the first r left singular vectors of a gradient, Alg. 2)
  B  bf16  N(0, 1e-3)      x  bf16  N(0, 1)      dy bf16  N(0, 1e-2)
Every tensor has its own counter-based stream keyed by (seed, workload, layer, name).
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    T: int  # tokens per step
    r: int  # rank of the adapter
    projections: Tuple[Tuple[str, int, int], ...]  # (layer name, out, in)
    n_blocks: int = 1  # number of identical blocks swept by the merge


def _block(d: int, ffn: int) -> Tuple[Tuple[str, int, int], ...]:
    return (
        ("q", d, d), ("k", d, d), ("v", d, d), ("o", d, d),
        ("gate", ffn, d), ("up", ffn, d), ("down", d, ffn),
    )


WORKLOADS = {
    "60m_layer": Workload("60m_layer", T=256, r=128, projections=(("layer", 512, 512),)),
    "130m_block": Workload("130m_block", T=4096, r=256, projections=_block(768, 2048)),
    "1b_block": Workload("1b_block", T=8192, r=512, projections=_block(2048, 5461)),
    "7b_block": Workload("7b_block", T=8192, r=1024, projections=_block(4096, 11008)),
    "13b_block": Workload("13b_block", T=4096, r=1024, projections=_block(5120, 13824), n_blocks=40),
}


def rng_for(seed: int, *names) -> np.random.Generator:
    """Counter-based generator keyed by the seed and a tuple of names."""
    key = [seed] + [zlib.crc32(str(n).encode()) for n in names]
    return np.random.Generator(np.random.Philox(np.random.SeedSequence(key)))


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even (finite inputs)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.reshape(-1).view(np.uint32)
    out = np.empty(u.shape, dtype=np.uint16)
    step = 1 << 20  # cache-sized pieces: the conversion is several passes over its input
    for i in range(0, u.size, step):
        c = u[i:i + step]
        r = c >> 16
        r &= 1
        r += np.uint32(0x7FFF)
        r += c
        r >>= 16
        out[i:i + step] = r
    return out.reshape(x.shape)


def normal_f32(rng: np.random.Generator, shape, sigma: float) -> np.ndarray:
    out = rng.standard_normal(shape, dtype=np.float32)
    if sigma != 1.0:
        out *= np.float32(sigma)
    return out


def normal_bf16(rng: np.random.Generator, shape, sigma: float) -> np.ndarray:
    return to_bf16_bits(normal_f32(rng, shape, sigma))


def orthonormal_f32(rng: np.random.Generator, rows: int, r: int) -> np.ndarray:
    """rows x r matrix with orthonormal columns (r <= rows): Q of a Gaussian's QR."""
    g = rng.standard_normal((rows, r))
    q, _ = np.linalg.qr(g, mode="reduced")
    return np.ascontiguousarray(q, dtype=np.float32)


@dataclass
class LayerTensors:
    name: str
    out: int
    inp: int
    r: int
    W: np.ndarray  # (out, in) float32
    P: np.ndarray  # (out, r) float32
    B: np.ndarray  # (r, in) bf16 bits
    x: np.ndarray  # (T, in) bf16 bits
    dy: np.ndarray  # (T, out) bf16 bits


def make_layer(workload: str, layer: str, out: int, inp: int, r: int, T: int, seed: int = 0,
               block: int = 0) -> LayerTensors:
    key = (workload, block, layer)
    return LayerTensors(
        name=layer, out=out, inp=inp, r=r,
        W=normal_f32(rng_for(seed, *key, "W"), (out, inp), 0.02),
        P=orthonormal_f32(rng_for(seed, *key, "P"), out, r),
        B=normal_bf16(rng_for(seed, *key, "B"), (r, inp), 1e-3),
        x=normal_bf16(rng_for(seed, *key, "x"), (T, inp), 1.0),
        dy=normal_bf16(rng_for(seed, *key, "dy"), (T, out), 1e-2),
    )


def make_workload(name: str, seed: int = 0, T: int | None = None) -> List[LayerTensors]:
    """All projections of one block of the named workload (T may be reduced for tests)."""
    wl = WORKLOADS[name]
    return [make_layer(name, ln, o, i, wl.r, T or wl.T, seed) for (ln, o, i) in wl.projections]


# algorithmic cost model, factored form (the full dW is never formed)
def flops_fwd(T: int, out: int, inp: int, r: int) -> int:
    return 2 * T * out * inp + 2 * T * inp * r + 2 * T * r * out


def flops_bwd(T: int, out: int, inp: int, r: int) -> int:
    return 2 * T * out * inp + 2 * T * out * r + 4 * T * r * inp


def flops_merge(out: int, inp: int, r: int) -> int:
    return 2 * out * inp * r


def bytes_merge(out: int, inp: int, r: int) -> float:
    """Each operand touched once: W_q read + written, P_q read, B read."""
    return 2 * 0.5625 * out * inp + 0.5625 * out * r + 2.0 * r * inp
