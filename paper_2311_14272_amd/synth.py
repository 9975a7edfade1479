"""Seeded synthetic inputs for the CRISP hybrid-sparse GEMM workloads.

This module only draws random tensors and describes workload shapes.  It holds
none of the method's arithmetic (no saliency, no selection, no packing, no
products), so the CPU oracle's tests and the HIP path's tests can both feed
from it without sharing any code that is under test.

The five workloads mirror the layer shapes the paper evaluates (ResNet-50,
VGG-16 and MobileNetV2 convolutions lowered to GEMMs, block sizes 32/64, N:M
patterns with M = 4 and the M = 8 extensions); the values are random with the
stated distributions, they are not taken from any dataset or checkpoint.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

SEED_BASE = 2311142720

SAL_GIVEN = 0   # saliency tensor T handed in directly
SAL_GRAD = 1    # T = |W * G|  (paper Eq. 1 with a given gradient tensor)
SAL_MAG = 2     # T = |W|

ROW_UNIFORM = 0  # same number of kept blocks in every block-row (the paper's mode)
LAYER_TOPK = 1   # best blocks of the whole grid, rows may be uneven


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even) and return the raw 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class ConvShape:
    """Convolution geometry; activations are stored channel-major [C][batch][H][W]."""
    C: int
    H: int
    W: int
    batch: int
    kh: int
    kw: int
    stride: int
    pad: int

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.kh) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.kw) // self.stride + 1

    @property
    def K(self) -> int:
        return self.kh * self.kw * self.C

    @property
    def Ncol(self) -> int:
        return self.batch * self.Ho * self.Wo


@dataclass
class LayerSpec:
    name: str
    S: int
    K: int
    Ncol: int
    n: int
    m: int
    B: int
    density: float
    sal_kind: int
    w_sigma: float
    conv: Optional[ConvShape] = None
    select_mode: int = ROW_UNIFORM


@dataclass
class Workload:
    name: str
    seed: int
    layers: List[LayerSpec] = field(default_factory=list)


def he_sigma(K: int) -> float:
    return float(np.sqrt(2.0 / K))


def config(cid: int, batch: Optional[int] = None) -> Workload:
    """Workload cid in 1..5 (the five benchmark configurations)."""
    seed = SEED_BASE + cid
    if cid == 1:
        return Workload("c1", seed, [LayerSpec("c1", 256, 1152, 3136, 2, 4, 32, 0.5, SAL_GRAD, 0.02)])
    if cid == 2:
        b = 32 if batch is None else batch
        n_col = b * 14 * 14
        conv = ConvShape(256, 14, 14, b, 3, 3, 1, 1)
        return Workload("c2", seed, [
            LayerSpec("c2a", 256, 1024, n_col, 1, 4, 64, 0.3, SAL_MAG, he_sigma(1024)),
            LayerSpec("c2b", 256, 2304, n_col, 1, 4, 64, 0.3, SAL_MAG, he_sigma(2304), conv=conv),
            LayerSpec("c2c", 1024, 256, n_col, 1, 4, 64, 0.3, SAL_MAG, he_sigma(256)),
        ])
    if cid == 3:
        b = 64 if batch is None else batch
        return Workload("c3", seed, [LayerSpec("c3", 512, 4608, b * 28 * 28, 2, 8, 64, 0.25, SAL_MAG, he_sigma(4608))])
    if cid == 4:
        b = 128 if batch is None else batch
        return Workload("c4", seed, [
            LayerSpec("c4a", 160, 960, b * 7 * 7, 2, 4, 32, 0.6, SAL_MAG, he_sigma(960)),
            LayerSpec("c4b", 24, 144, b * 56 * 56, 2, 4, 32, 0.6, SAL_MAG, he_sigma(144)),
        ])
    if cid == 5:
        return resnet50(256 if batch is None else batch, seed)
    raise ValueError("config id must be 1..5")


NM_CHOICES: Tuple[Tuple[int, int], ...] = ((1, 4), (2, 4), (1, 8), (2, 8), (4, 8))


def resnet50_convs(batch: int) -> List[Tuple[str, int, ConvShape]]:
    """(name, out_channels, geometry) of the 53 convolutions of ResNet-50 at 224x224,
    stride on the 3x3 conv of each stage's first bottleneck."""
    out: List[Tuple[str, int, ConvShape]] = []
    out.append(("conv1", 64, ConvShape(3, 224, 224, batch, 7, 7, 2, 3)))
    cin, hw = 64, 56
    for si, (mid, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3))):
        cout = mid * 4
        for bi in range(blocks):
            stride = 2 if (bi == 0 and si > 0) else 1
            pre = "s%db%d" % (si + 1, bi)
            out.append((pre + ".a", mid, ConvShape(cin, hw, hw, batch, 1, 1, 1, 0)))
            out.append((pre + ".b", mid, ConvShape(mid, hw, hw, batch, 3, 3, stride, 1)))
            hw2 = hw // stride
            out.append((pre + ".c", cout, ConvShape(mid, hw2, hw2, batch, 1, 1, 1, 0)))
            if bi == 0:
                out.append((pre + ".ds", cout, ConvShape(cin, hw, hw, batch, 1, 1, stride, 0)))
            cin, hw = cout, hw2
    return out


def resnet50(batch: int, seed: int) -> Workload:
    """All 53 convs as GEMMs; the per-layer (n:m, density) draws are made first,
    before any tensor, from the workload's generator."""
    rng = np.random.Generator(np.random.PCG64(seed))
    convs = resnet50_convs(batch)
    layers = []
    for name, S, cv in convs:
        n, m = NM_CHOICES[int(rng.integers(0, len(NM_CHOICES)))]
        d = float(rng.uniform(0.2, 0.8))
        layers.append(LayerSpec(name, S, cv.K, cv.Ncol, n, m, 64, d, SAL_GRAD, he_sigma(cv.K), conv=cv))
    return Workload("c5", seed, layers)


def layer_rng(wl: Workload, layer_index: int) -> np.random.Generator:
    """Independent, reproducible stream per layer of a workload."""
    return np.random.Generator(np.random.PCG64([wl.seed, 1000 + layer_index]))


def draw_weight(rng: np.random.Generator, L: LayerSpec) -> np.ndarray:
    """W as raw bf16 bits, S x K row-major, N(0, w_sigma)."""
    w = rng.standard_normal((L.S, L.K), dtype=np.float32) * np.float32(L.w_sigma)
    return f32_to_bf16_bits(w)


def draw_grad(rng: np.random.Generator, L: LayerSpec, classes: int = 1) -> np.ndarray:
    """G fp32, S x K: sum over `classes` N(0,1) tensors, accumulated in class order in fp32."""
    g = np.zeros((L.S, L.K), dtype=np.float32)
    for _ in range(classes):
        g = (g + rng.standard_normal((L.S, L.K), dtype=np.float32)).astype(np.float32)
    return g


def draw_relu_normal(rng: np.random.Generator, shape) -> np.ndarray:
    """ReLU(N(0,1)) as raw bf16 bits."""
    x = rng.standard_normal(shape, dtype=np.float32)
    np.maximum(x, np.float32(0), out=x)
    return f32_to_bf16_bits(x)


def draw_layer(wl: Workload, layer_index: int, with_x: bool = True, x_cols: Optional[int] = None):
    """Returns dict(W, G (or None), X (K x Ncol bits or None), act (conv input or None)).

    Draw order is fixed: W, then G (if the layer uses a gradient), then the
    activation.  For a layer with a conv geometry larger than 1x1 the drawn
    tensor is the conv's input activation [C][batch][H][W]; otherwise it is X
    itself (K x Ncol).  `x_cols` limits the number of X columns drawn (only for
    non-conv layers; used for bounded samples of the very large workloads).
    """
    L = wl.layers[layer_index]
    rng = layer_rng(wl, layer_index)
    out = {"W": draw_weight(rng, L), "G": None, "X": None, "act": None}
    if L.sal_kind == SAL_GRAD:
        out["G"] = draw_grad(rng, L, classes=10 if wl.name == "c5" else 1)
    if with_x:
        cv = L.conv
        if cv is not None and (cv.kh > 1 or cv.kw > 1 or cv.stride > 1):
            out["act"] = draw_relu_normal(rng, (cv.C, cv.batch, cv.H, cv.W))
        else:
            ncol = L.Ncol if x_cols is None else min(x_cols, L.Ncol)
            out["X"] = draw_relu_normal(rng, (L.K, ncol))
    return out


def small_cases() -> List[LayerSpec]:
    """Small shapes that still span several tiles and ragged tails; the oracle
    finishes each in well under a second."""
    mk = LayerSpec
    return [
        mk("t_2:4_b32", 96, 160, 200, 2, 4, 32, 0.5, SAL_GRAD, 0.05),
        mk("t_1:4_b64", 128, 320, 328, 1, 4, 64, 0.4, SAL_MAG, 0.05),
        mk("t_2:8_b64", 192, 256, 520, 2, 8, 64, 0.5, SAL_MAG, 0.05),
        mk("t_4:8_b32", 64, 224, 136, 4, 8, 32, 0.7, SAL_GRAD, 0.05),
        mk("t_1:8_b64", 64, 192, 72, 1, 8, 64, 0.67, SAL_MAG, 0.05),
        mk("t_3:4_b32", 64, 96, 264, 3, 4, 32, 0.67, SAL_MAG, 0.05),
        mk("t_ragged_b32", 24, 144, 1000, 2, 4, 32, 0.6, SAL_MAG, 0.1),
        mk("t_ragged_b64", 70, 147, 392, 2, 4, 64, 0.67, SAL_GRAD, 0.1),
        mk("t_ragged_m8", 40, 150, 80, 2, 8, 32, 0.5, SAL_GRAD, 0.1),
        mk("t_odd_ncol", 64, 128, 1003, 2, 4, 32, 0.5, SAL_MAG, 0.05),
        mk("t_dense_nm", 64, 128, 96, 4, 4, 32, 0.5, SAL_MAG, 0.05),
        mk("t_dense_m8", 64, 128, 160, 8, 8, 64, 0.5, SAL_MAG, 0.05),
        mk("t_all_blocks", 64, 128, 64, 2, 4, 64, 1.0, SAL_MAG, 0.05),
        mk("t_uneven_rows", 256, 512, 264, 2, 4, 64, 0.3, SAL_GRAD, 0.05, None, LAYER_TOPK),
        mk("t_uneven_b32", 160, 320, 136, 1, 4, 32, 0.25, SAL_MAG, 0.05, None, LAYER_TOPK),
    ]


def draw_two_per_quad_weight(rng: np.random.Generator, S: int, K: int) -> np.ndarray:
    """bf16 bits of a weight whose four largest magnitudes in every group of eight columns are two per aligned
    group of four (random places, random signs): what a 4:8 pruning keeps of it passes the 2-of-4 test of the
    pack.  K must be a multiple of 4."""
    r = rng.random((S, K // 4, 4))
    big = (np.argsort(np.argsort(r, axis=2), axis=2) >= 2).reshape(S, K)
    mag = np.where(big, 2.0, 0.3) * rng.uniform(1.0, 1.4, size=(S, K))
    return f32_to_bf16_bits((mag * rng.choice([-1.0, 1.0], size=(S, K))).astype(np.float32))


def b16_cases() -> List[LayerSpec]:
    """16 x 16 blocks (the paper's smallest block size)."""
    mk = LayerSpec
    return [
        mk("b16_2:4", 48, 80, 200, 2, 4, 16, 0.5, SAL_GRAD, 0.05),
        mk("b16_1:4", 64, 48, 328, 1, 4, 16, 0.67, SAL_MAG, 0.05),
        mk("b16_2:8_ragged", 40, 90, 77, 2, 8, 16, 0.5, SAL_MAG, 0.05),
        mk("b16_4:8", 32, 64, 520, 4, 8, 16, 0.75, SAL_MAG, 0.05),
        mk("b16_3:4_uneven", 64, 128, 136, 3, 4, 16, 0.4, SAL_GRAD, 0.05, None, LAYER_TOPK),
    ]


def draw_small(L: LayerSpec, seed: int):
    rng = np.random.Generator(np.random.PCG64([SEED_BASE, seed]))
    W = draw_weight(rng, L)
    G = draw_grad(rng, L) if L.sal_kind == SAL_GRAD else None
    X = draw_relu_normal(rng, (L.K, L.Ncol))
    return W, G, X
