"""Seeded synthetic workloads: chain descriptions and random tensors.

This module is shared by the CPU oracle's tests and by the GPU path's tests and
bench. It holds *inputs only*: layer hyper-parameters (what a caller of the
library would write down) and seeded random tensors. None of the method's
arithmetic lives here: no shape inference, no halo propagation, no convolution.

Chains are stand-ins for the vision models the paper evaluates (Sec. VI lists
VGGNet and ResNet among its models); weights are random because trained
checkpoints are not available offline.

Conventions
-----------
* Logical tensor layout is NCHW for activations and OIHW for weights (the
  textbook convention). Consumers that want NHWC permute on their side.
* ``input_from`` / ``residual_from`` are 0-based layer indices; ``-1`` is the
  chain input; ``residual_from == -2`` means "no residual".
* bf16 tensors are returned as float32 arrays whose values are exactly
  representable in bfloat16 (rounded with torch's round-to-nearest-even cast),
  together with the raw uint16 bit patterns where a consumer wants them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

CONV, DWCONV, MAXPOOL, ELTWISE = "conv", "dwconv", "maxpool", "eltwise"
ACT_NONE, ACT_RELU, ACT_RELU6 = "none", "relu", "relu6"
NO_RESIDUAL = -2
CHAIN_INPUT = -1

BASE_SEED = 250705829


@dataclass
class Layer:
    op: str
    c_in: int
    c_out: int
    k: Tuple[int, int] = (1, 1)
    s: Tuple[int, int] = (1, 1)
    p: Tuple[int, int] = (0, 0)
    d: Tuple[int, int] = (1, 1)
    act: str = ACT_NONE
    input_from: int = CHAIN_INPUT
    residual_from: int = NO_RESIDUAL
    has_bias: bool = True

    @property
    def groups(self) -> int:
        return self.c_in if self.op == DWCONV else 1

    @property
    def has_weight(self) -> bool:
        return self.op in (CONV, DWCONV)


@dataclass
class Chain:
    name: str
    in_shape: Tuple[int, int, int, int]          # N, C, H, W
    dtype: str                                   # "f32" | "bf16"
    n_bands: int
    layers: List[Layer] = field(default_factory=list)
    seed: int = BASE_SEED
    in_range: Tuple[float, float] = (0.0, 1.0)

    def add(self, op, c_in, c_out, k=1, s=1, p=0, d=1, act=ACT_NONE,
            input_from: Optional[int] = None, residual_from: int = NO_RESIDUAL,
            has_bias: bool = True) -> int:
        """Append a layer; by default it consumes the previous layer's output."""
        if input_from is None:
            input_from = len(self.layers) - 1
        pair = lambda v: (v, v) if isinstance(v, int) else tuple(v)
        self.layers.append(Layer(op, c_in, c_out, pair(k), pair(s), pair(p), pair(d), act,
                                 input_from, residual_from,
                                 has_bias and op != MAXPOOL))
        return len(self.layers) - 1


# --------------------------------------------------------------------------- chains

def tiny_chain() -> Chain:
    """Two conv3x3 (16->16, s1 p1) + bias + ReLU on 1x16x32x32, fp32, 4 bands."""
    c = Chain("tiny", (1, 16, 32, 32), "f32", 4, seed=BASE_SEED + 0)
    c.add(CONV, 16, 16, 3, 1, 1, act=ACT_RELU)
    c.add(CONV, 16, 16, 3, 1, 1, act=ACT_RELU)
    return c


def resnet18_chain(h: int = 224, w: int = 224, n: int = 1, n_bands: int = 4,
                   dtype: str = "f32") -> Chain:
    """ResNet-18-style backbone without batch-norm, average pool or classifier.

    conv7x7 s2 p3 + ReLU, maxpool3x3 s2 p1, then four stages of two basic blocks
    (conv3x3-ReLU-conv3x3, + shortcut, ReLU). The first block of stages 2-4
    downsamples with stride 2 and uses a conv1x1 s2 shortcut. 21 layers.
    """
    c = Chain("resnet18", (n, 3, h, w), dtype, n_bands, seed=BASE_SEED + 1)
    c.add(CONV, 3, 64, 7, 2, 3, act=ACT_RELU)
    x = c.add(MAXPOOL, 64, 64, 3, 2, 1)
    ch = 64
    for stage, width in enumerate((64, 128, 256, 512)):
        for block in range(2):
            down = stage > 0 and block == 0
            a = c.add(CONV, ch, width, 3, 2 if down else 1, 1, act=ACT_RELU, input_from=x)
            if down:
                sc = c.add(CONV, ch, width, 1, 2, 0, act=ACT_NONE, input_from=x)
            else:
                sc = x
            x = c.add(CONV, width, width, 3, 1, 1, act=ACT_RELU, input_from=a, residual_from=sc)
            ch = width
    return c


def vgg16_chain(h: int = 224, w: int = 224, n: int = 1, n_bands: int = 8,
                dtype: str = "bf16") -> Chain:
    """VGG-16 convolutional stack: 13 conv3x3 p1 + ReLU, 5 maxpool2x2 s2."""
    c = Chain("vgg16", (n, 3, h, w), dtype, n_bands, seed=BASE_SEED + 2)
    ch = 3
    for width, reps in ((64, 2), (128, 2), (256, 3), (512, 3), (512, 3)):
        for _ in range(reps):
            c.add(CONV, ch, width, 3, 1, 1, act=ACT_RELU)
            ch = width
        c.add(MAXPOOL, ch, ch, 2, 2, 0)
    return c


def detector_chain(h: int = 720, w: int = 1280, n: int = 1, n_bands: int = 16,
                   dtype: str = "bf16", stride2_layers=(1, 3, 5, 7)) -> Chain:
    """Ten conv3x3 p1 + ReLU; ``stride2_layers`` are 1-based layer numbers."""
    c = Chain("detector720p", (n, 3, h, w), dtype, n_bands, seed=BASE_SEED + 3)
    ch = 3
    for i, width in enumerate((32, 32, 64, 64, 128, 128, 256, 256, 256, 256), start=1):
        c.add(CONV, ch, width, 3, 2 if i in stride2_layers else 1, 1, act=ACT_RELU)
        ch = width
    return c


def mbv2_chain(h: int = 640, w: int = 640, n: int = 8, n_bands: int = 8,
               dtype: str = "bf16", width: int = 32, expand: int = 6) -> Chain:
    """Six inverted-residual blocks of constant width.

    Each block: conv1x1 expand (x6) + ReLU6, depthwise 3x3 p1 + ReLU6 (stride 2
    in blocks 1 and 4, 1-based), conv1x1 project without activation, plus the
    block input as a residual where the shapes match (blocks 2, 3, 5, 6).
    """
    c = Chain("mbv2", (n, width, h, w), dtype, n_bands, seed=BASE_SEED + 4,
              in_range=(-1.0, 1.0))
    x = CHAIN_INPUT
    for block in range(1, 7):
        s = 2 if block in (1, 4) else 1
        c.add(CONV, width, width * expand, 1, 1, 0, act=ACT_RELU6, input_from=x)
        c.add(DWCONV, width * expand, width * expand, 3, s, 1, act=ACT_RELU6)
        x = c.add(CONV, width * expand, width, 1, 1, 0, act=ACT_NONE,
                  residual_from=x if s == 1 else NO_RESIDUAL)
    return c


CONFIGS = {
    "tiny": tiny_chain,
    "resnet18": resnet18_chain,
    "vgg16": vgg16_chain,
    "detector720p": detector_chain,
    "mbv2": mbv2_chain,
}


# --------------------------------------------------------------------------- tensors

def to_bf16_values(a: np.ndarray) -> np.ndarray:
    """Round finite float32 values to the nearest bfloat16 (ties to even), keep float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(a))


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Bit patterns (uint16) of float32 values that are already bf16-representable."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(u & 0xFFFF), "values are not bf16-representable"
    return (u >> 16).astype(np.uint16)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """float32 values of bf16 bit patterns."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


@dataclass
class Tensors:
    x: np.ndarray                         # N,C,H,W float32
    weights: List[Optional[np.ndarray]]   # per layer OIHW float32 (depthwise: C,1,kh,kw) or None
    biases: List[Optional[np.ndarray]]    # per layer float32 [c_out] or None


def make_tensors(chain: Chain, zero_bias: bool = True, seed: Optional[int] = None) -> Tensors:
    """Draw the chain input, then per layer the weight and then the bias.

    Input ~ U[in_range]; weights ~ N(0, sqrt(2/fan_in)) with
    fan_in = (c_in/groups)*kh*kw; biases are zero (the bench setting) or, for
    tests that exercise the bias path, U[-0.5, 0.5]. For bf16 chains the input
    and weights are rounded to bf16-representable values; biases stay fp32.
    """
    rng = np.random.Generator(np.random.PCG64(chain.seed if seed is None else seed))
    lo, hi = chain.in_range
    x = rng.random(chain.in_shape, dtype=np.float32) * np.float32(hi - lo) + np.float32(lo)
    ws, bs = [], []
    for L in chain.layers:
        if L.has_weight:
            cig = L.c_in // L.groups
            fan_in = cig * L.k[0] * L.k[1]
            w = rng.standard_normal((L.c_out, cig, L.k[0], L.k[1]), dtype=np.float32)
            w *= np.float32(np.sqrt(2.0 / fan_in))
        else:
            w = None
        if L.has_bias:
            b = (np.zeros(L.c_out, np.float32) if zero_bias
                 else rng.random(L.c_out, dtype=np.float32) - np.float32(0.5))
        else:
            b = None
        ws.append(w)
        bs.append(b)
    if chain.dtype == "bf16":
        x = to_bf16_values(x)
        ws = [None if w is None else to_bf16_values(w) for w in ws]
    return Tensors(x, ws, bs)


def small_int_tensors(chain: Chain, seed: int = 7) -> Tensors:
    """Small-integer tensors: every partial sum is exact in fp32 for short chains.

    x in {0..3}, w in {-2..2}, b in {-4..4}: a GPU result must then equal the
    oracle bit-for-bit regardless of summation order, which separates indexing
    mistakes from rounding differences.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.integers(0, 4, chain.in_shape).astype(np.float32)
    ws, bs = [], []
    for L in chain.layers:
        if L.has_weight:
            cig = L.c_in // L.groups
            ws.append(rng.integers(-2, 3, (L.c_out, cig, L.k[0], L.k[1])).astype(np.float32))
        else:
            ws.append(None)
        bs.append(rng.integers(-4, 5, L.c_out).astype(np.float32) if L.has_bias else None)
    return Tensors(x, ws, bs)


# ---- row-wise local operators (matrix chains): shapes only, like the chains above ----

@dataclass
class RowLayer:
    k: int                               # columns of the input matrix
    n: int                               # columns of the output matrix
    act: str = ACT_NONE
    input_from: int = CHAIN_INPUT
    residual_from: int = NO_RESIDUAL
    has_bias: bool = True


@dataclass
class RowChain:
    """y_l = act(x_l W_l^T + b_l + residual) on a matrix of m rows, W_l of n x k."""
    name: str
    m: int
    k: int
    dtype: str
    n_bands: int
    layers: List[RowLayer] = field(default_factory=list)
    seed: int = BASE_SEED + 100

    @property
    def in_shape(self) -> Tuple[int, int, int, int]:
        """The matrix seen as a tensor: one image of m x 1 pixels with k channels."""
        return (1, self.k, self.m, 1)

    def add(self, n: int, act: str = ACT_NONE, residual_from: int = NO_RESIDUAL,
            has_bias: bool = True, input_from: Optional[int] = None) -> "RowChain":
        src = (len(self.layers) - 1) if input_from is None else input_from
        k = self.k if src < 0 else self.layers[src].n
        self.layers.append(RowLayer(k, n, act, src, residual_from, has_bias))
        return self


def mlp_chain(m: int = 65536, k: int = 1024, hidden: int = 4096, dtype: str = "bf16",
              n_bands: int = 8) -> RowChain:
    """Two matrix products with a ReLU between and a residual around: the feed-forward block
    of a transformer-style model as a chain of row-wise local operators."""
    c = RowChain("mlp", m, k, dtype, n_bands)
    c.add(hidden, ACT_RELU)
    c.add(k, ACT_NONE, residual_from=CHAIN_INPUT)
    return c


def make_row_tensors(chain: RowChain, zero_bias: bool = True, seed: Optional[int] = None) -> Tensors:
    """Input matrix ~ U[-1, 1], then per layer W ~ N(0, sqrt(2/k)) (n x k) and the bias."""
    rng = np.random.Generator(np.random.PCG64(chain.seed if seed is None else seed))
    x = rng.random((chain.m, chain.k), dtype=np.float32) * np.float32(2) - np.float32(1)
    ws, bs = [], []
    for L in chain.layers:
        w = rng.standard_normal((L.n, L.k), dtype=np.float32) * np.float32(np.sqrt(2.0 / L.k))
        b = None
        if L.has_bias:
            b = (np.zeros(L.n, np.float32) if zero_bias
                 else rng.random(L.n, dtype=np.float32) - np.float32(0.5))
        ws.append(w)
        bs.append(b)
    if chain.dtype == "bf16":
        x = to_bf16_values(x)
        ws = [to_bf16_values(w) for w in ws]
    return Tensors(x, ws, bs)


# ---- two-party schedules (Sec. IV-C variables x_M(v), x_R(v)) ----
def random_schedule(heights: Sequence[int], seed: int, overlap: int = 2):
    """One pair of contiguous intervals per layer whose union is [0, h): party M takes
    [0, a), party R takes [b, h) with b <= a (the overlap is replication); either party may
    end up with nothing, and which party takes the top rows is drawn per layer."""
    rng = np.random.default_rng(seed)
    out = []
    for h in heights:
        a = int(rng.integers(0, h + 1))
        b = max(0, a - int(rng.integers(0, overlap + 1)))
        first, second = (0, a), (b, h)
        if a == 0:
            second = (0, h)
        if b >= h:
            second = (0, 0)
        if rng.integers(0, 2):
            out.append({"M": first, "R": second})
        else:
            out.append({"M": second, "R": first})
    return out
