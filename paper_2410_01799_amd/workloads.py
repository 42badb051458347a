"""Seeded synthetic inputs shaped like the paper's workloads, plus the size arithmetic.

This module holds none of the method's arithmetic: it only draws matrices/tensors and computes
widths and footprints.  The same arrays are handed to the CPU oracle and to the GPU path.

The paper's own data (a 4096x4096 Gaussian matrix, Section 4.1; the Mistral-7B weight matrices,
Section 4.2; a 4000x3000x3 photograph, Section 5) is not available, so every input here is a
synthetic stand-in with the same shape, dtype and rough structure.
"""
from __future__ import annotations

from fractions import Fraction
from typing import Dict, Iterator, List, Tuple

import numpy as np

# --------------------------------------------------------------------------- size arithmetic


def width_for_compression(m: int, n: int, p, coef_bits: int = 32, elem_bits: int = 16) -> int:
    """Width w whose packed size is the fraction p of the dense matrix (Section 4.2, Table 2).

    A term costs ``coef_bits + m + n`` bits, the dense matrix ``elem_bits * m * n`` bits;
    w = floor(p * elem_bits * m * n / (coef_bits + m + n)).
    """
    p = Fraction(p).limit_denominator(1 << 20)
    return int((p * elem_bits * m * n) // (coef_bits + m + n))


def compression_rate(w: int, m: int, n: int, coef_bits: int = 32, elem_bits: int = 16) -> float:
    """p_{m,n}(w) = w (coef_bits + m + n) / (elem_bits m n)  (Section 4.1 with 64/64, 4.2 with 32/16)."""
    return w * (coef_bits + m + n) / (elem_bits * m * n)


def packed_bits(w: int, dims, coef_bits: int = 32) -> int:
    """Bits needed for w terms: one coefficient and one sign bit per index of every mode."""
    return int(w) * (coef_bits + int(sum(dims)))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stored as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    b = x.view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    return b.astype(np.uint32).view(np.float32).reshape(x.shape)


def relative_error(approx: np.ndarray, exact: np.ndarray) -> float:
    """||approx - exact||_F / ||exact||_F in float64 (the r_k of Section 4.1)."""
    d = np.asarray(approx, dtype=np.float64) - np.asarray(exact, dtype=np.float64)
    return float(np.linalg.norm(d.ravel()) / np.linalg.norm(np.asarray(exact, dtype=np.float64).ravel()))


# --------------------------------------------------------------------------- matrices


def gaussian_matrix(m: int, n: int, seed: int, dtype=np.float32) -> np.ndarray:
    """i.i.d. N(0,1) entries drawn in float64 from PCG64(seed), then cast (Section 4.1)."""
    g = np.random.Generator(np.random.PCG64(seed))
    return g.standard_normal((m, n)).astype(dtype)


def config1() -> Tuple[np.ndarray, int, int]:
    """256x256 f32 N(0,1), width 64, sign-stream seed 1."""
    return gaussian_matrix(256, 256, 1, np.float32), 64, 1


def config2(dtype=np.float32) -> Tuple[np.ndarray, int, int]:
    """4096x4096 N(0,1) (seed 2); f32 run to w=8192, f64 run to w=2048; sign-stream seed 2."""
    w = 8192 if np.dtype(dtype) == np.float32 else 2048
    return gaussian_matrix(4096, 4096, 2, dtype), w, 2


LAYER_SHAPES: List[Tuple[str, int, int]] = [
    ("q_proj", 4096, 4096),
    ("k_proj", 1024, 4096),
    ("v_proj", 1024, 4096),
    ("o_proj", 4096, 4096),
    ("gate_proj", 14336, 4096),
    ("up_proj", 14336, 4096),
    ("down_proj", 4096, 14336),
]


def weight_like_matrix(m: int, n: int, seed: int, sigma: float = 0.02, rank: int = 16,
                       lowrank_energy: float = 0.1, outlier_frac: float = 0.01,
                       outlier_scale: float = 8.0) -> np.ndarray:
    """Decoder-weight stand-in: N(0, sigma^2) noise, plus a rank-`rank` Gaussian component that
    carries `lowrank_energy` of the total squared norm, then 1% of the columns scaled x8, then
    rounded to bf16-representable float32 values."""
    g = np.random.Generator(np.random.PCG64(seed))
    G = g.standard_normal((m, n), dtype=np.float32) * np.float32(sigma)
    if rank > 0 and lowrank_energy > 0:
        U = g.standard_normal((m, rank), dtype=np.float32)
        V = g.standard_normal((n, rank), dtype=np.float32)
        L = U @ V.T
        eg = float(np.sum(G.astype(np.float64) ** 2))
        el = float(np.sum(L.astype(np.float64) ** 2))
        # ||aL||^2 = e * (||G||^2 + ||aL||^2)  (cross term ~ 0)  ->  a^2 = e/(1-e) * eg/el
        a = np.sqrt(lowrank_energy / (1.0 - lowrank_energy) * eg / el)
        G += np.float32(a) * L
        del L
    ncol = int(n * outlier_frac)
    if ncol > 0:
        cols = g.choice(n, size=ncol, replace=False)
        G[:, cols] *= np.float32(outlier_scale)
    return round_to_bf16(G)


def config3() -> Iterator[Tuple[str, np.ndarray, int, int]]:
    """One Mistral-7B-shaped decoder layer: yields (name, matrix, width at 50% of bf16, seed)."""
    for idx, (name, m, n) in enumerate(LAYER_SHAPES):
        yield name, weight_like_matrix(m, n, 300 + idx), width_for_compression(m, n, Fraction(1, 2)), 300 + idx


def config5_manifest(layers: int = 32) -> List[Dict]:
    """The 226-matrix weight set: 32 layers x 7 shapes + embedding + lm_head (shapes, seeds, widths)."""
    out = []
    idx = 0
    for layer in range(layers):
        for name, m, n in LAYER_SHAPES:
            out.append(dict(name=f"layers.{layer}.{name}", m=m, n=n, seed=5000 + idx, kind="weight"))
            idx += 1
    for name in ("embed_tokens", "lm_head"):
        out.append(dict(name=name, m=32000, n=4096, seed=5000 + idx, kind="gauss"))
        idx += 1
    for e in out:
        e["widths"] = {p: width_for_compression(e["m"], e["n"], Fraction(p)) for p in ("1/4", "3/8", "1/2")}
    return out


def config5_matrix(entry: Dict) -> np.ndarray:
    if entry["kind"] == "gauss":
        g = np.random.Generator(np.random.PCG64(entry["seed"]))
        return round_to_bf16(g.standard_normal((entry["m"], entry["n"]), dtype=np.float32) * np.float32(0.02))
    return weight_like_matrix(entry["m"], entry["n"], entry["seed"])


# --------------------------------------------------------------------------- image-like tensor


def image_like_tensor(h: int = 4000, wd: int = 3000, channels: int = 3, blobs: int = 200,
                      seed: int = 400) -> np.ndarray:
    """h x wd x channels float32 tensor of integers 0..255: per channel a sum of `blobs`
    anisotropic Gaussian blobs plus a linear gradient and an offset of 128 (Section 5 stand-in)."""
    out = np.empty((h, wd, channels), dtype=np.float32)
    y = np.arange(h, dtype=np.float32)[:, None]
    x = np.arange(wd, dtype=np.float32)[None, :]
    for ch in range(channels):
        g = np.random.Generator(np.random.PCG64(seed + ch))
        img = np.full((h, wd), 128.0, dtype=np.float32)
        gx, gy = g.uniform(-40, 40, size=2)
        img += np.float32(gy) * (y / h - 0.5) + np.float32(gx) * (x / wd - 0.5)
        for _ in range(blobs):
            cy, cx = g.uniform(0, h), g.uniform(0, wd)
            sy, sx = np.exp(g.uniform(np.log(20.0), np.log(800.0), size=2))
            th = g.uniform(0, np.pi)
            amp = g.uniform(-80, 80)
            # separable approximation of a rotated blob: rotate the axes, keep the product form
            ct, st = np.float32(np.cos(th)), np.float32(np.sin(th))
            # bounding box of 3.5 sigma keeps the cost proportional to the blob area
            rad = 3.5 * max(sy, sx)
            y0, y1 = int(max(0, cy - rad)), int(min(h, cy + rad + 1))
            x0, x1 = int(max(0, cx - rad)), int(min(wd, cx + rad + 1))
            if y0 >= y1 or x0 >= x1:
                continue
            dy = y[y0:y1] - np.float32(cy)
            dx = x[:, x0:x1] - np.float32(cx)
            a = ct * dx + st * dy
            b = -st * dx + ct * dy
            img[y0:y1, x0:x1] += np.float32(amp) * np.exp(-0.5 * ((a / np.float32(sx)) ** 2 + (b / np.float32(sy)) ** 2))
        out[:, :, ch] = np.clip(np.rint(img), 0, 255)
    return out


def config4() -> Tuple[np.ndarray, int, int]:
    """4000x3000x3 image-like tensor, width 129, sign-stream seed 4."""
    return image_like_tensor(), 129, 4
