"""Seeded synthetic workloads shared by the CPU oracle's tests and the GPU tests.

This module holds workload *descriptions* (the operator shapes of the TVM
paper's Table 2 and the five benchmark configurations built from them) and the
seeded random input generators.  It contains none of the method's arithmetic:
no convolution, no epilogue, no pooling.  Neither the oracle nor the GPU
library is imported here.

Value recipe (all workloads): x ~ U[-1, 1]; w ~ N(0, sigma) with the He-normal
sigma = sqrt(2 / fan_in), fan_in = IC*R*S (9 for depthwise); scale ~ U[0.5, 1.5];
shift ~ U[-0.1, 0.1]; residual ~ U[-1, 1].  Draw order x, w, scale, shift,
residual from ``numpy.random.default_rng(seed)`` in fp64, cast to fp32, and for
bf16 workloads rounded to the nearest bfloat16 (ties to even) so that both the
oracle and the GPU see bf16-representable values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

SEED_BASE = 180204799


@dataclass(frozen=True)
class ConvShape:
    """One conv2d (or depthwise conv2d) problem, NCHW / OIHW, symmetric zero padding."""
    name: str
    n: int
    ic: int
    h: int
    w: int
    oc: int
    r: int
    s: int
    stride: int
    pad: int
    depthwise: bool = False

    @property
    def oh(self) -> int:
        return (self.h + 2 * self.pad - self.r) // self.stride + 1

    @property
    def ow(self) -> int:
        return (self.w + 2 * self.pad - self.s) // self.stride + 1

    @property
    def fan_in(self) -> int:
        return (1 if self.depthwise else self.ic) * self.r * self.s

    @property
    def flops(self) -> int:
        """2 * MACs of the direct method, padded taps counted, epilogue not counted."""
        return 2 * self.n * self.oc * self.oh * self.ow * self.fan_in

    def x_shape(self):
        return (self.n, self.ic, self.h, self.w)

    def w_shape(self):
        return (self.oc, 1 if self.depthwise else self.ic, self.r, self.s)

    def y_shape(self):
        return (self.n, self.oc, self.oh, self.ow)

    def algorithmic_bytes(self, elem_bytes: int, residual: bool = False) -> int:
        """Compulsory traffic of the fused operator: x, w, y (and residual) moved once,
        plus the fp32 scale and shift vectors."""
        nx = int(np.prod(self.x_shape()))
        nw = int(np.prod(self.w_shape()))
        ny = int(np.prod(self.y_shape()))
        return (nx + nw + ny * (2 if residual else 1)) * elem_bytes + 2 * self.oc * 4

    def with_batch(self, n: int) -> "ConvShape":
        return ConvShape(self.name, n, self.ic, self.h, self.w, self.oc, self.r, self.s,
                         self.stride, self.pad, self.depthwise)


def _c(name, hw, ic, oc, k, s, n=1) -> ConvShape:
    return ConvShape(name, n, ic, hw, hw, oc, k, k, s, k // 2)


def _d(name, hw, c, s, n=1) -> ConvShape:
    return ConvShape(name, n, c, hw, hw, c, 3, 3, s, 1, depthwise=True)


def resnet18_convs(n: int = 1) -> List[ConvShape]:
    """C1..C12 of Table 2 (all conv2d operators of ResNet-18), pad = k // 2."""
    return [
        _c("C1", 224, 3, 64, 7, 2, n), _c("C2", 56, 64, 64, 3, 1, n), _c("C3", 56, 64, 64, 1, 1, n),
        _c("C4", 56, 64, 128, 3, 2, n), _c("C5", 56, 64, 128, 1, 2, n),
        _c("C6", 28, 128, 128, 3, 1, n), _c("C7", 28, 128, 256, 3, 2, n),
        _c("C8", 28, 128, 256, 1, 2, n), _c("C9", 14, 256, 256, 3, 1, n),
        _c("C10", 14, 256, 512, 3, 2, n), _c("C11", 14, 256, 512, 1, 2, n),
        _c("C12", 7, 512, 512, 3, 1, n),
    ]


def mobilenet_depthwise(n: int = 1) -> List[ConvShape]:
    """D1..D9 of Table 2 (all depthwise conv2d operators of MobileNet), 3x3, pad 1."""
    return [
        _d("D1", 112, 32, 1, n), _d("D2", 112, 64, 2, n), _d("D3", 56, 128, 1, n),
        _d("D4", 56, 128, 2, n), _d("D5", 28, 256, 1, n), _d("D6", 28, 256, 2, n),
        _d("D7", 14, 512, 1, n), _d("D8", 14, 512, 2, n), _d("D9", 7, 1024, 1, n),
    ]


def layer_seed(config: int, layer_index: int) -> int:
    return SEED_BASE + 1000 * config + layer_index


# ----------------------------------------------------------------------------------------
# bfloat16 helpers for preparing inputs (bit-level, host side)
# ----------------------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest, ties to even.
    Finite values only (the generators never produce NaN or infinity)."""
    bits = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> the float32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize_bf16(a: np.ndarray) -> np.ndarray:
    """float32 values rounded to bf16-representable float32 values."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a)).reshape(np.shape(a))


# ----------------------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------------------

def make_inputs(shape: ConvShape, seed: int, dtype: str = "f32", residual: bool = False,
                bias: bool = False) -> Dict[str, Optional[np.ndarray]]:
    """Draw x, w, scale, shift (and residual, bias) for one layer.

    Returns float32 arrays; with ``dtype == "bf16"`` x, w and residual hold
    bf16-representable values (scale/shift/bias stay full fp32, as in the ABI).
    """
    if dtype not in ("f32", "bf16"):
        raise ValueError(dtype)
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1.0, 1.0, size=shape.x_shape()).astype(np.float32)
    sigma = float(np.sqrt(2.0 / shape.fan_in))
    w = (rng.standard_normal(size=shape.w_shape()) * sigma).astype(np.float32)
    scale = rng.uniform(0.5, 1.5, size=(shape.oc,)).astype(np.float32)
    shift = rng.uniform(-0.1, 0.1, size=(shape.oc,)).astype(np.float32)
    res = rng.uniform(-1.0, 1.0, size=shape.y_shape()).astype(np.float32) if residual else None
    b = rng.uniform(-0.1, 0.1, size=(shape.oc,)).astype(np.float32) if bias else None
    if dtype == "bf16":
        x, w = quantize_bf16(x), quantize_bf16(w)
        if res is not None:
            res = quantize_bf16(res)
    return {"x": x, "w": w, "scale": scale, "shift": shift, "residual": res, "bias": b}


def make_weights(shape: ConvShape, seed: int, dtype: str = "f32") -> Dict[str, np.ndarray]:
    """Weights, scale and shift only (for layers of a chained network)."""
    rng = np.random.default_rng(seed)
    sigma = float(np.sqrt(2.0 / shape.fan_in))
    w = (rng.standard_normal(size=shape.w_shape()) * sigma).astype(np.float32)
    scale = rng.uniform(0.5, 1.5, size=(shape.oc,)).astype(np.float32)
    shift = rng.uniform(-0.1, 0.1, size=(shape.oc,)).astype(np.float32)
    if dtype == "bf16":
        w = quantize_bf16(w)
    return {"w": w, "scale": scale, "shift": shift}


# ----------------------------------------------------------------------------------------
# the five benchmark configurations
# ----------------------------------------------------------------------------------------

def config1_shape() -> ConvShape:
    """Single fused conv2d, fp32, batch 1: Table 2's C2."""
    return resnet18_convs(1)[1]


@dataclass(frozen=True)
class Step:
    """One launch of a network body: tensors are named by small integer ids."""
    op: str                      # "conv", "dwconv", "maxpool" or "conv_dual"
    name: str
    src: int
    dst: int
    shape: Optional[ConvShape] = None
    residual: Optional[int] = None
    relu: bool = True
    layer_index: int = 0         # index used for the layer's weight seed
    # "conv_dual": a 3x3 conv (shape, relu, layer_index -> dst) and a 1x1 conv of the same input
    # with the same stride (shape2, relu2, layer_index2 -> dst2) as one launch
    dst2: Optional[int] = None
    shape2: Optional[ConvShape] = None
    relu2: bool = False
    layer_index2: int = 0


def resnet18_body(n: int = 32, fuse_projection: bool = False) -> List[Step]:
    """ResNet-18 convolutional body as a flat launch list (tensor 0 = the images).

    fuse_projection: a down-sampling block's first conv and its projection shortcut, which read
    the same tensor, become ONE "conv_dual" step (18 launches instead of 21); tensor ids, layer
    indices and therefore every weight stay those of the unfused list.

    Stem conv (C1) + ReLU, 3x3 stride-2 pad-1 max-pool, then 8 basic blocks:
    conv-scale/shift-ReLU, conv-scale/shift + shortcut, ReLU.  Down-sampling
    blocks use a 1x1 stride-2 projection (scale/shift, no ReLU) as the shortcut.
    20 convolutions in total: C1, 4xC2, C4, C5, 3xC6, C7, C8, 3xC9, C10, C11, 3xC12.
    """
    C = {s.name: s for s in resnet18_convs(n)}
    steps: List[Step] = []
    counter = {"t": 1, "l": 0}

    def new_tensor() -> int:
        t = counter["t"]
        counter["t"] += 1
        return t

    def conv(name, shape, src, residual=None, relu=True) -> int:
        dst = new_tensor()
        steps.append(Step("conv", name, src, dst, shape, residual, relu, counter["l"]))
        counter["l"] += 1
        return dst

    t = conv("stem", C["C1"], 0)
    pooled = new_tensor()
    steps.append(Step("maxpool", "pool", t, pooled))
    t = pooled

    def basic_block(tag, t_in, first, second, proj=None) -> int:
        if proj is not None and fuse_projection:
            a, shortcut = new_tensor(), new_tensor()
            steps.append(Step("conv_dual", f"{tag}.conv1+proj", t_in, a, first, None, True, counter["l"],
                              shortcut, proj, False, counter["l"] + 1))
            counter["l"] += 2
            return conv(f"{tag}.conv2", second, a, residual=shortcut)
        a = conv(f"{tag}.conv1", first, t_in)
        shortcut = t_in if proj is None else conv(f"{tag}.proj", proj, t_in, relu=False)
        return conv(f"{tag}.conv2", second, a, residual=shortcut)

    t = basic_block("s1b1", t, C["C2"], C["C2"])
    t = basic_block("s1b2", t, C["C2"], C["C2"])
    t = basic_block("s2b1", t, C["C4"], C["C6"], C["C5"])
    t = basic_block("s2b2", t, C["C6"], C["C6"])
    t = basic_block("s3b1", t, C["C7"], C["C9"], C["C8"])
    t = basic_block("s3b2", t, C["C9"], C["C9"])
    t = basic_block("s4b1", t, C["C10"], C["C12"], C["C11"])
    t = basic_block("s4b2", t, C["C12"], C["C12"])
    return steps


def mobilenet_body(n: int = 32) -> List[Step]:
    """MobileNet (v1, width 1, 224 x 224) convolutional body as a flat launch list.

    Stem: 3x3 stride-2 conv 3 -> 32, then 13 blocks of a depthwise 3x3 conv (Table 2's
    D1..D9, D7 five times) followed by a 1x1 conv; every layer carries scale/shift + ReLU.
    27 launches; tensor 0 = the images, the last tensor is [n][1024][7][7].
    """
    D = {s.name: s for s in mobilenet_depthwise(n)}
    blocks = [("D1", 64), ("D2", 128), ("D3", 128), ("D4", 256), ("D5", 256), ("D6", 512),
              ("D7", 512), ("D7", 512), ("D7", 512), ("D7", 512), ("D7", 512), ("D8", 1024),
              ("D9", 1024)]
    steps: List[Step] = [Step("conv", "stem", 0, 1, ConvShape("M0", n, 3, 224, 224, 32, 3, 3, 2, 1),
                              None, True, 0)]
    t, layer = 1, 1
    for b, (dname, oc) in enumerate(blocks, start=1):
        d = D[dname]
        steps.append(Step("dwconv", f"b{b}.dw", t, t + 1, d, None, True, layer))
        pw = ConvShape(f"P{b}", n, d.ic, d.oh, d.ow, oc, 1, 1, 1, 0)
        steps.append(Step("conv", f"b{b}.pw", t + 1, t + 2, pw, None, True, layer + 1))
        t += 2
        layer += 2
    return steps


def tensor_lives(steps: List[Step], elem_bytes: int = 2):
    """(bytes, first_step, last_step) per tensor id of a launch list, for a static memory plan.

    A tensor must stay intact from the launch that writes it to the last launch that reads it
    (as src or residual); tensor 0, the images, is there from launch 0, and the last tensor
    stays until the end because the caller reads it.
    """
    shapes = {0: steps[0].shape.x_shape()}
    first, last = {0: 0}, {0: 0}
    for i, st in enumerate(steps):
        if st.op == "maxpool":
            n, c, h, w = shapes[st.src]
            shapes[st.dst] = (n, c, (h - 1) // 2 + 1, (w - 1) // 2 + 1)
        else:
            shapes[st.dst] = st.shape.y_shape()
        first[st.dst] = last[st.dst] = i
        if st.op == "conv_dual":
            shapes[st.dst2] = st.shape2.y_shape()
            first[st.dst2] = last[st.dst2] = i
        for t in (st.src, st.residual):
            if t is not None:
                last[t] = i
    last[steps[-1].dst] = len(steps) - 1
    return {t: (int(np.prod(shapes[t])) * elem_bytes, first[t], last[t]) for t in sorted(shapes)}


def body_images(n: int, seed: int) -> np.ndarray:
    """U[-1, 1] images [n][3][224][224], bf16-representable float32."""
    rng = np.random.default_rng(seed)
    return quantize_bf16(rng.uniform(-1.0, 1.0, size=(n, 3, 224, 224)).astype(np.float32))
