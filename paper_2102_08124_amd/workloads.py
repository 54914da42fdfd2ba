"""Seeded synthetic inputs shaped like the paper's workloads.

This module only *generates inputs* (shapes, distributions, dtype conversion).  It holds none of
the method's arithmetic (no magnitudes, ranks, masks, flows), so both the CPU oracle's tests and
the HIP path's tests/bench may import it without sharing any logic of the method.

The paper evaluates on trained ResNet-50 / BERT-large weights (Sec. 4.1, Tables 3-4); no trained
weights or datasets are available offline, so tensors with those architectures' layer *shapes*
and an init-like *distribution* stand in for them.
"""
from __future__ import annotations

import numpy as np

F32 = "f32"
BF16 = "bf16"


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round-to-nearest-even) and return the raw 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    r[nan] = ((u[nan] >> np.uint32(16)) | np.uint32(0x0040)).astype(np.uint16)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen raw bfloat16 bit patterns to fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def resnet50_conv_shapes(include_stem: bool = False) -> list[tuple[int, int]]:
    """Every conv of ResNet-50 flattened to (Cout, Cin*kh*kw), in network order.

    The 7x7 stem (64 x 147) is not a multiple of 4 wide and is left out unless asked for.
    """
    shapes: list[tuple[int, int]] = []
    if include_stem:
        shapes.append((64, 3 * 7 * 7))
    cin = 64
    for width, n_blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        cout = 4 * width
        for b in range(n_blocks):
            shapes.append((width, cin))          # 1x1 reduce
            shapes.append((width, width * 9))    # 3x3
            shapes.append((cout, width))         # 1x1 expand
            if b == 0:
                shapes.append((cout, cin))       # 1x1 projection shortcut
            cin = cout
    return shapes


def resnet50_kernel_area(shape: tuple[int, int]) -> int:
    """kh*kw of the conv a flattened shape came from (9 for the 3x3 convs, 49 stem, else 1)."""
    cout, k = shape
    if k == 147:
        return 49
    return 9 if k == 9 * cout else 1


def bert_large_linear_shapes() -> list[tuple[int, int]]:
    """24 encoder layers x {Q, K, V, O (1024x1024), FFN-in (4096x1024), FFN-out (1024x4096)}."""
    per_layer = [(1024, 1024)] * 4 + [(4096, 1024), (1024, 4096)]
    return per_layer * 24


def gaussian_f32(rows: int, cols: int, seed: int, std: float = 1.0) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(std)).astype(np.float32)


def laplace_f32(rows: int, cols: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.laplace(0.0, 1.0, size=(rows, cols)).astype(np.float32)


def config1() -> np.ndarray:
    """64x64 fp32, i.i.d. N(0,1), seed 1."""
    return gaussian_f32(64, 64, seed=1)


def config2(limit: int | None = None) -> list[np.ndarray]:
    """ResNet-50 conv set, fp32, Kaiming-normal (std = sqrt(2/fan_out)), seed 2+layer index."""
    mats = []
    for k, shp in enumerate(resnet50_conv_shapes()[:limit]):
        fan_out = shp[0] * resnet50_kernel_area(shp)
        mats.append(gaussian_f32(shp[0], shp[1], seed=2 + k, std=float(np.sqrt(2.0 / fan_out))))
    return mats


def config3(limit: int | None = None) -> list[np.ndarray]:
    """BERT-large linear set as raw bf16 bit patterns (uint16), N(0, 0.02), seed 3+index."""
    return [f32_to_bf16_bits(gaussian_f32(r, c, seed=3 + k, std=0.02))
            for k, (r, c) in enumerate(bert_large_linear_shapes()[:limit])]


def config4(side: int = 8192) -> np.ndarray:
    """side x side fp32, Laplace(0,1), seed 4."""
    return laplace_f32(side, side, seed=4)


def config5_init(side: int = 16384) -> np.ndarray:
    """side x side bf16 bit patterns, W0 ~ N(0, 0.02), seed 5."""
    return f32_to_bf16_bits(gaussian_f32(side, side, seed=5, std=0.02))


def config5_step(w_bits: np.ndarray, step: int) -> np.ndarray:
    """One surrogate training step: add 1e-3 * N(0, 0.02) in fp32, round back to bf16."""
    rng = np.random.default_rng(np.random.SeedSequence([5, step]))
    noise = rng.standard_normal(w_bits.shape, dtype=np.float32) * np.float32(0.02e-3)
    return f32_to_bf16_bits(bf16_bits_to_f32(w_bits) + noise)


def tie_heavy_f32(rows: int, cols: int, seed: int, levels: int = 5) -> np.ndarray:
    """Few distinct magnitudes, random signs, some exact zeros: stresses the tie-break."""
    rng = np.random.default_rng(seed)
    v = rng.integers(0, levels, size=(rows, cols)).astype(np.float32)
    s = rng.integers(0, 2, size=(rows, cols)).astype(np.float32) * 2 - 1
    return (v * s).astype(np.float32)


def special_values_f32(rows: int, cols: int, seed: int) -> np.ndarray:
    """N(0,1) salted with +-0, denormals, +-Inf and NaN (magnitude order is by bit pattern)."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((rows, cols), dtype=np.float32)
    salt = rng.integers(0, 40, size=(rows, cols))
    w[salt == 0] = 0.0
    w[salt == 1] = -0.0
    w[salt == 2] = np.float32(1e-41)
    w[salt == 3] = np.float32(-3e-42)
    w[salt == 4] = np.inf
    w[salt == 5] = -np.inf
    w[salt == 6] = np.nan
    return w
