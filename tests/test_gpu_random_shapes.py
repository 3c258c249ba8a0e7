"""Seeded random problem shapes through the C ABI against the oracle, full outputs.

The shape lists of test_gpu_parity.py are written by hand around the cases each kernel is known
to have; this sweep draws shapes, tails and tile overrides at random (fixed seeds, so every run
sees the same cases) to reach the combinations nobody thought of.  It found the stem kernel's
unreadable last weight when OC x IC is odd.
"""
import random

import numpy as np
import pytest

import oracle
import tvg_inputs as ti
from _util import BLOCK_TIGHT, check, dev_inputs, fixed_tile, to_host

pytestmark = pytest.mark.gpu

TILES = ["", "", "64,256", "64,128", "128,64", "64,64", "128,128"]


def draw_dense(rng):
    kind = rng.choice(["3x3", "3x3", "3x3deep", "3x3deep_s2", "1x1", "7x7", "odd"])
    if kind == "3x3":
        ic, r, stride, pad = 16 * rng.randint(1, 6), 3, rng.choice([1, 2]), 1
    elif kind == "3x3deep":
        ic, r, stride, pad = 32 * rng.randint(4, 8), 3, 1, 1
    elif kind == "3x3deep_s2":
        ic, r, stride, pad = 32 * rng.randint(4, 8), 3, 2, 1
    elif kind == "1x1":
        ic, r, stride, pad = 8 * rng.randint(1, 40), 1, rng.choice([1, 2]), 0
    elif kind == "7x7":
        ic, r, stride, pad = rng.randint(1, 4), 7, 2, 3
    else:                                   # shapes no specialised kernel takes
        r = rng.choice([1, 2, 3, 5])
        ic, stride, pad = rng.randint(1, 20), rng.choice([1, 2, 3]), rng.randint(0, r - 1)   # pad < r
    n = rng.choice([1, 2, 3, 5, 8])
    lo = 4 if r == 7 else max(1, r - 2 * pad)
    h, w = rng.randint(lo, 30), rng.randint(lo, 30)
    if kind == "7x7":
        w = 8 * rng.randint(1, 5)
    elif rng.random() < 0.5:
        w += w & 1                          # favour even rows (wide loads)
    oc = rng.choice([1, 8, 33, 64, 70, 128, 130, 200])
    return ti.ConvShape("r", n, ic, h, w, oc, r, r, stride, pad)


def cases(seed, count):
    rng = random.Random(seed)
    out = []
    while len(out) < count:
        sh = draw_dense(rng)
        if sh.flops > 4e8:
            continue
        out.append((len(out), sh, rng.choice(TILES), rng.random() < 0.7, rng.random() < 0.5,
                    rng.random() < 0.5, rng.random() < 0.5))
    return out


@pytest.mark.parametrize("case", cases(20260, 300), ids=lambda c: f"{c[0]}")
def test_random_dense_bf16(tvg, case):
    import torch
    i, sh, tile, relu, hint, res, bias = case
    inp = ti.make_inputs(sh, 52000 + i, "bf16", residual=res, bias=bias)
    d = dev_inputs(inp, "bf16")
    with fixed_tile(tvg, sh, "bf16", tile):
        y = tvg.conv2d_fused(d["x"], d["w"], d["scale"], d["shift"], d["bias"], d["residual"],
                             stride=sh.stride, pad=sh.pad, relu=relu, stream_out=hint)
        torch.cuda.synchronize()
    want = oracle.conv2d_fused(inp["x"], inp["w"], inp["scale"], inp["shift"], inp["bias"],
                               inp["residual"], stride=(sh.stride,) * 2, pad=(sh.pad,) * 2, relu=relu)
    check(to_host(y), want, "bf16", sh)


@pytest.mark.parametrize("case", cases(20261, 100), ids=lambda c: f"{c[0]}")
def test_random_dense_fp32(tvg, case):
    i, sh, _, relu, hint, res, bias = case
    inp = ti.make_inputs(sh, 53000 + i, "f32", residual=res, bias=bias)
    d = dev_inputs(inp, "f32")
    y = tvg.conv2d_fused(d["x"], d["w"], d["scale"], d["shift"], d["bias"], d["residual"],
                         stride=sh.stride, pad=sh.pad, relu=relu, stream_out=hint)
    want = oracle.conv2d_fused(inp["x"], inp["w"], inp["scale"], inp["shift"], inp["bias"],
                               inp["residual"], stride=(sh.stride,) * 2, pad=(sh.pad,) * 2, relu=relu)
    check(to_host(y), want, "f32", sh)


def dw_cases(seed, count):
    rng = random.Random(seed)
    out = []
    for i in range(count):
        n, c = rng.choice([1, 2, 5]), rng.choice([1, 3, 8, 32, 100])
        h, w = rng.randint(1, 40), rng.randint(1, 40)
        if rng.random() < 0.5:
            w = 4 * rng.randint(1, 10)
        out.append((i, n, c, h, w, rng.choice([1, 2]), rng.choice(["f32", "f32", "bf16"]),
                    rng.random() < 0.7, rng.random() < 0.5, rng.random() < 0.5))
    return out


@pytest.mark.parametrize("case", dw_cases(20262, 120), ids=lambda c: f"{c[0]}")
def test_random_depthwise(tvg, case):
    i, n, c, h, w, stride, dtype, relu, hint, res = case
    sh = ti.ConvShape("rd", n, c, h, w, c, 3, 3, stride, 1, depthwise=True)
    inp = ti.make_inputs(sh, 54000 + i, dtype, residual=res, bias=True)
    d = dev_inputs(inp, dtype)
    y = tvg.dwconv2d_fused(d["x"], d["w"], d["scale"], d["shift"], d["bias"], d["residual"],
                           stride=stride, pad=1, relu=relu, stream_out=hint)
    want = oracle.dwconv2d_fused(inp["x"], inp["w"], inp["scale"], inp["shift"], inp["bias"],
                                 inp["residual"], stride=(stride,) * 2, pad=(1, 1), relu=relu)
    check(to_host(y), want, dtype, sh)


def dw_many_plane_cases(seed, count):
    """Launches with thousands of planes: what the row-per-lane kernel (output rows of 7, 14 and,
    in bf16, 28 pixels) and the taller row blocks of the fp32 register-blocked kernel take."""
    rng = random.Random(seed)
    out = []
    for i in range(count):
        stride = rng.choice([1, 2])
        if rng.random() < 0.6:
            w = rng.choice([7, 14, 28]) * stride              # the row kernel's widths
        else:
            w = 4 * rng.randint(2, 16)                        # rows of whole 16-byte vectors
        h = rng.randint(2, 30)
        oh = (h - 1) // stride + 1
        planes = max(1, rng.choice([17000, 20000, 140000]) // max(1, oh) + rng.randint(0, 7))
        planes = min(planes, 3_000_000 // (h * w))            # keep the oracle's work small
        c = rng.choice([c for c in (64, 96, 256, 500, 1000) if c <= planes] or [planes])
        n = -(-planes // c)
        out.append((i, n, c, h, w, stride, rng.choice(["f32", "bf16"]), rng.random() < 0.7,
                    rng.random() < 0.5, rng.random() < 0.5))
    return out


@pytest.mark.parametrize("case", dw_many_plane_cases(31337, 48), ids=lambda c: f"{c[0]}")
def test_random_depthwise_many_planes(tvg, case):
    i, n, c, h, w, stride, dtype, relu, hint, res = case
    sh = ti.ConvShape("rp", n, c, h, w, c, 3, 3, stride, 1, depthwise=True)
    inp = ti.make_inputs(sh, 58000 + i, dtype, residual=res, bias=True)
    d = dev_inputs(inp, dtype)
    y = tvg.dwconv2d_fused(d["x"], d["w"], d["scale"], d["shift"], d["bias"], d["residual"],
                           stride=stride, pad=1, relu=relu, stream_out=hint)
    want = oracle.dwconv2d_fused(inp["x"], inp["w"], inp["scale"], inp["shift"], inp["bias"],
                                 inp["residual"], stride=(stride,) * 2, pad=(1, 1), relu=relu)
    check(to_host(y), want, dtype, sh)


def block_cases(seed, count):
    rng = random.Random(seed)
    out = []
    for i in range(count):
        n, c = rng.choice([1, 2, 3, 6]), 32 * rng.randint(1, 5)
        h, w = rng.randint(1, 30), rng.randint(1, 30)
        if rng.random() < 0.3:
            h = w = rng.choice([7, 14, 28])
        out.append((i, n, c, h, w, rng.choice([1, 7, 32, 64, 100, 128, 200, 256, 300]),
                    rng.choice([1, 1, 1, 2]), rng.random() < 0.7, rng.random() < 0.7,
                    rng.random() < 0.4, rng.random() < 0.4, rng.random() < 0.5))
    return out


@pytest.mark.parametrize("case", block_cases(20263, 80), ids=lambda c: f"{c[0]}")
def test_random_blocks(tvg, case):
    """tvg_dwpw_fused on random bf16 shapes: the one-kernel form wherever it exists (no
    workspace), and the two-kernel form for every case."""
    i, n, c, h, w, k, stride, relu_dw, relu_pw, res, bias, hint = case
    d = ti.ConvShape("bd", n, c, h, w, c, 3, 3, stride, 1, depthwise=True)
    p = ti.ConvShape("bp", n, c, d.oh, d.ow, k, 1, 1, 1, 0)
    a = ti.make_inputs(d, 56000 + 2 * i, "bf16")
    b = ti.make_inputs(p, 56001 + 2 * i, "bf16", residual=res, bias=bias)
    da, db = dev_inputs(a, "bf16"), dev_inputs(b, "bf16")
    want = oracle.dwpw_fused(a["x"], a["w"], a["scale"], a["shift"], b["w"], b["scale"], b["shift"],
                             b["bias"], b["residual"], stride=stride, relu_dw=relu_dw,
                             relu_pw=relu_pw, store="bf16")
    desc = tvg.ConvDesc(n, c, h, w, c, 3, 3, stride, stride, 1, 1, tvg.TVG_BF16, 0)
    forms = [False] + ([True] if tvg.tvg_dwpw_one_kernel(desc, k) else [])
    if stride == 1 and h * w >= 32 and w <= 30:
        assert True in forms, "every such map fits the one-kernel form"
    for one in forms:
        y = tvg.dwpw_fused(da["x"], da["w"], da["scale"], da["shift"], db["w"], db["scale"],
                           db["shift"], db["bias"], db["residual"], stride=stride, relu_dw=relu_dw,
                           relu_pw=relu_pw, stream_out=hint, one_kernel=one)
        check(to_host(y), want, "bf16", (one, d, k), tight=BLOCK_TIGHT)
