"""Seeded synthetic inputs shaped like the paper's workloads.

The paper trains Conformer speech models (Sec. 3.1); their weights and data are
not available, so only the *shapes* are taken: a Conformer-encoder-shaped list
of variables whose matrices are drawn N(0, 1/sqrt(fan_in)).  This module serves
the CPU oracle's tests and the GPU path alike and therefore holds no arithmetic
of the method itself: no codec, no packing, no fit, no optimizer.  Sizes of
packed buffers are obtained through a callback supplied by the caller.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, List, Optional, Sequence

import numpy as np


@dataclass(frozen=True)
class VarSpec:
    name: str
    shape: tuple
    fan_in: int
    is_matrix: bool  # rank >= 2 kernels are "weight matrices" (Sec. 2.4); vectors stay fp32

    @property
    def n(self) -> int:
        return int(np.prod(self.shape))


def conformer_varset(d_model: int = 512, blocks: int = 17, ffn: int = 2048, conv_kernel: int = 32,
                     frontend: bool = True) -> List[VarSpec]:
    """Conformer-encoder-shaped variable list ([in x out] matrices, fan_in = first dimension).

    Per block: two feed-forward modules (d x ffn, ffn x d each), self-attention (q, k, v, out
    and relative-position projections, d x d), the convolution module (pointwise d x 2d,
    depthwise K x d, pointwise d x d), and the biases / layer-norm vectors that go with them.
    """
    d = d_model
    out: List[VarSpec] = []

    def mat(name, a, b, fan_in=None):
        out.append(VarSpec(name, (a, b), fan_in if fan_in is not None else a, True))

    def vec(name, a):
        out.append(VarSpec(name, (a,), a, False))

    if frontend:
        # convolutional subsampling output (20 freq bins x d channels) projected to d, plus a
        # 3x3 channel-to-channel subsampling convolution flattened to [9 d x d]
        mat("frontend/proj", 20 * d, d)
        mat("frontend/conv2", 9 * d, d)
        vec("frontend/proj_bias", d)
        vec("frontend/conv2_bias", d)
    for i in range(blocks):
        p = f"block{i}"
        for ff in ("ffn1", "ffn2"):
            vec(f"{p}/{ff}/ln_scale", d)
            vec(f"{p}/{ff}/ln_bias", d)
            mat(f"{p}/{ff}/w_in", d, ffn)
            vec(f"{p}/{ff}/b_in", ffn)
            mat(f"{p}/{ff}/w_out", ffn, d)
            vec(f"{p}/{ff}/b_out", d)
        vec(f"{p}/att/ln_scale", d)
        vec(f"{p}/att/ln_bias", d)
        for w in ("q", "k", "v", "o"):
            mat(f"{p}/att/w_{w}", d, d)
            vec(f"{p}/att/b_{w}", d)
        mat(f"{p}/att/w_pos", d, d)
        vec(f"{p}/conv/ln_scale", d)
        vec(f"{p}/conv/ln_bias", d)
        mat(f"{p}/conv/pw1", d, 2 * d)
        vec(f"{p}/conv/pw1_bias", 2 * d)
        mat(f"{p}/conv/dw", conv_kernel, d, fan_in=conv_kernel)
        vec(f"{p}/conv/dw_bias", d)
        vec(f"{p}/conv/norm_scale", d)
        vec(f"{p}/conv/norm_bias", d)
        mat(f"{p}/conv/pw2", d, d)
        vec(f"{p}/conv/pw2_bias", d)
        vec(f"{p}/final_ln_scale", d)
        vec(f"{p}/final_ln_bias", d)
    return out


def ppq_mask(specs: Sequence[VarSpec], fraction: float, seed: int) -> np.ndarray:
    """Partial parameter quantization (Sec. 2.5): a seeded subset, by count, of the weight
    matrices is marked quantized; non-matrices never are (Sec. 2.4)."""
    mat_idx = [i for i, s in enumerate(specs) if s.is_matrix]
    perm = np.random.default_rng(seed).permutation(len(mat_idx))
    take = int(np.ceil(fraction * len(mat_idx)))
    mask = np.zeros(len(specs), dtype=bool)
    for j in perm[:take]:
        mask[mat_idx[j]] = True
    return mask


@dataclass
class Layout:
    specs: List[VarSpec]
    quantized: np.ndarray          # bool per variable
    data_offset: np.ndarray        # bytes into the arena, 16-byte aligned
    aux_offset: np.ndarray         # elements into gradient / state arrays, multiple of 4
    arena_bytes: int
    aux_elems: int


def make_layout(specs: Sequence[VarSpec], quantized: Sequence[bool],
                packed_bytes: Callable[[int], int]) -> Layout:
    """Place variables back to back: packed codes (size from `packed_bytes(n)`) or fp32, each
    at a 16-byte aligned arena offset; gradients / optimizer state at 4-element aligned offsets."""
    doff, aoff = [], []
    d = a = 0
    for s, q in zip(specs, quantized):
        doff.append(d)
        aoff.append(a)
        nbytes = packed_bytes(s.n) if q else 4 * s.n
        d += (nbytes + 15) // 16 * 16
        a += (s.n + 3) // 4 * 4
    return Layout(list(specs), np.asarray(quantized, dtype=bool), np.asarray(doff, dtype=np.uint64),
                  np.asarray(aoff, dtype=np.uint64), int(d), int(a))


def normal_f32(n: int, std: float, seed: int) -> np.ndarray:
    return (np.random.default_rng(seed).standard_normal(n, dtype=np.float32) * np.float32(std))


def init_values(layout: Layout, seed: int) -> np.ndarray:
    """fp32 values for every variable in aux order: matrices N(0, 1/sqrt(fan_in)); scale vectors
    near 1, biases near 0 (small noise so that nothing is exactly constant)."""
    out = np.zeros(layout.aux_elems, dtype=np.float32)
    rng = np.random.default_rng(seed)
    for s, a in zip(layout.specs, layout.aux_offset):
        a = int(a)
        if s.is_matrix:
            x = rng.standard_normal(s.n, dtype=np.float32) * np.float32(1.0 / np.sqrt(s.fan_in))
        elif s.name.endswith("scale"):
            x = np.float32(1.0) + rng.standard_normal(s.n, dtype=np.float32) * np.float32(0.01)
        else:
            x = rng.standard_normal(s.n, dtype=np.float32) * np.float32(0.01)
        out[a:a + s.n] = x
    return out


def gradients(layout: Layout, std: float, seed: int) -> np.ndarray:
    """One synthetic gradient set N(0, std) over the whole aux range (padding stays zero)."""
    out = np.zeros(layout.aux_elems, dtype=np.float32)
    rng = np.random.default_rng(seed)
    for s, a in zip(layout.specs, layout.aux_offset):
        a = int(a)
        out[a:a + s.n] = rng.standard_normal(s.n, dtype=np.float32) * np.float32(std)
    return out


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest, ties to even) and return the 16-bit patterns.
    Input preparation for the forward GEMM's activations; finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def adversarial_values(fmt_max: float, step: float, n: int, seed: int) -> np.ndarray:
    """Values that stress a reduced float format whose largest magnitude is `fmt_max` and whose
    smallest step is `step`: ties, near-ties, the subnormal boundary, saturation, signed zeros,
    fp32 subnormals, plus log-uniform magnitudes over the whole range."""
    rng = np.random.default_rng(seed)
    special = [0.0, -0.0, step, -step, 0.5 * step, -0.5 * step, 1.5 * step, 2.5 * step,
               0.5 * step * (1 + 2 ** -20), 0.5 * step * (1 - 2 ** -20), fmt_max, -fmt_max,
               fmt_max * (1 + 2 ** -12), 2 * fmt_max, -2 * fmt_max, 1e-45, -1e-45, 1e-40, 3e38, -3e38]
    k = max(n - len(special), 0)
    lo, hi = np.log2(step) - 3, np.log2(fmt_max) + 2
    mags = np.exp2(rng.uniform(lo, hi, size=k))
    signs = rng.choice([-1.0, 1.0], size=k)
    halves = np.round(mags / (0.5 * step)) * (0.5 * step)  # many exact ties / grid points
    pick = rng.random(k) < 0.3
    vals = np.where(pick, halves, mags) * signs
    out = np.concatenate([np.asarray(special, dtype=np.float64), vals])[:n]
    with np.errstate(over="ignore"):
        return out.astype(np.float32)
