"""GPU parity of the pre-transformed-weights path (Winograd F(2x2, 3x3); paper Section 6.1, the
"TVM PT" variant) against the same fp64 oracle as the direct kernels: the operator's definition
does not change, only the arithmetic that reaches it.

Tolerance.  The stated one is the bf16 gate, 2e-2.  The bound this arithmetic gives: both
transformed operands are rounded to fp16 (relative error at most 2^-11 each, about 2^-11/sqrt(3)
rms); a product therefore carries about 4e-4 rms relative error; the 16 position sums M_k have a
joint rms of sqrt(2) times the output's (the inverse transform cancels half of their energy), so
the error reaches the output at about 6e-4 of its rms, and at a few sigma, about 3e-3, at the
worst of 10^7 elements; the final rounding to bf16 adds at most 2^-8 = 3.9e-3.  Asserted: 1e-2."""
import numpy as np
import pytest

import oracle
import tvg_inputs as ti
from _util import TOL, dev_inputs, rel_err, to_host

pytestmark = pytest.mark.gpu

WINO_TIGHT = 1e-2


def run_prepacked(tvg, sh, inp, relu=True, stream_out=False):
    import torch
    d = dev_inputs(inp, "bf16")
    flags = (tvg.TVG_RELU if relu else 0) | (tvg.TVG_STREAM_OUT if stream_out else 0)
    desc = tvg.ConvDesc(sh.n, sh.ic, sh.h, sh.w, sh.oc, 3, 3, 1, 1, 1, 1, tvg.TVG_BF16, flags)
    pb, wb = tvg.tvg_conv2d_prepack_size(desc)
    assert pb == 16 * sh.ic * sh.oc * 2
    assert wb == 16 * sh.ic * sh.n * ((sh.h + 1) // 2) * ((sh.w + 1) // 2) * 2
    packed = torch.empty(pb, dtype=torch.uint8, device="cuda")
    ws = torch.empty(wb, dtype=torch.uint8, device="cuda")
    assert tvg.tvg_conv2d_prepack(desc, d["w"], packed, pb) == 0
    y = torch.full(sh.y_shape(), float("nan"), dtype=torch.bfloat16, device="cuda")
    st = tvg.tvg_conv2d_fused_prepacked(desc, d["x"], packed, d["scale"], d["shift"], d["bias"],
                                        d["residual"], y, ws, wb)
    assert st == 0, tvg.status_string(st)
    torch.cuda.synchronize()
    return y


def oracle_out(sh, inp, relu=True):
    return oracle.conv2d_fused(inp["x"], inp["w"], inp["scale"], inp["shift"], inp["bias"],
                               inp["residual"], stride=(1, 1), pad=(1, 1), relu=relu)


def check_wino(got, want, what):
    err = rel_err(got, want)
    assert err <= TOL["bf16"], (what, err)
    assert err <= WINO_TIGHT, (what, err, "tight bound")
    return err


WINO_LAYERS = [1, 5, 8, 11]            # C2, C6, C9, C12: the 3x3 stride-1 layers of Table 2


@pytest.mark.parametrize("batch", [1, 64])
@pytest.mark.parametrize("i", WINO_LAYERS)
def test_winograd_table2_layers_full(tvg, i, batch):
    """C2, C6, C9, C12 at batch 1 and at batch 64 (the benchmark's launch): every output."""
    sh = ti.resnet18_convs(batch)[i]
    inp = ti.make_inputs(sh, ti.layer_seed(7, i), "bf16")
    got = to_host(run_prepacked(tvg, sh, inp, stream_out=batch == 64))
    assert tuple(got.shape) == sh.y_shape()
    check_wino(got, oracle_out(sh, inp), (sh.name, batch))
    assert np.all(got >= 0)


# (n, ic, h, w, oc): odd and tiny maps (half-empty last tile row / column), maps of one tile,
# tile counts that leave the last workgroup ragged, all three store paths (W % 8 == 0, even, odd)
RAGGED = [(1, 64, 1, 1, 64), (2, 64, 2, 3, 64), (3, 64, 5, 7, 128), (2, 128, 9, 6, 64),
          (1, 64, 13, 13, 192), (5, 64, 8, 16, 64), (2, 192, 11, 24, 64), (1, 64, 3, 130, 64),
          (7, 64, 7, 7, 64), (3, 128, 14, 14, 128), (1, 64, 40, 40, 64)]


@pytest.mark.parametrize("variant", ["plain", "bias+residual", "no-relu+residual"])
@pytest.mark.parametrize("cfg", RAGGED, ids=lambda c: "x".join(map(str, c)))
def test_winograd_ragged_shapes_full_tail(tvg, cfg, variant):
    n, ic, h, w, oc = cfg
    sh = ti.ConvShape("w", n, ic, h, w, oc, 3, 3, 1, 1)
    seed = 4100 + sum(cfg) + len(variant)
    inp = ti.make_inputs(sh, seed, "bf16", residual="residual" in variant, bias="bias" in variant)
    relu = "no-relu" not in variant
    got = to_host(run_prepacked(tvg, sh, inp, relu=relu))
    check_wino(got, oracle_out(sh, inp, relu=relu), (cfg, variant))


def test_winograd_single_taps_place_every_weight(tvg):
    """A filter with one non-zero tap is a shift of the input: nine of them pin the transforms'
    index conventions (which input row/column meets which tap) independently of the tolerance -
    a shift by one pixel or a transposed filter changes the result by whole values."""
    sh = ti.ConvShape("w", 2, 64, 6, 10, 64, 3, 3, 1, 1)
    rng = np.random.default_rng(991)
    x = np.round(rng.uniform(-4, 4, size=sh.x_shape())).astype(np.float32)      # small integers
    for tap in range(9):
        w = np.zeros(sh.w_shape(), np.float32)
        for oc in range(64):
            w[oc, (oc * 7 + tap) % 64, tap // 3, tap % 3] = 1.0
        inp = {"x": x, "w": w, "scale": np.ones(64, np.float32), "shift": np.zeros(64, np.float32),
               "bias": None, "residual": None}
        got = to_host(run_prepacked(tvg, sh, inp, relu=False))
        want = oracle_out(sh, inp, relu=False)
        # integers times weights of 1, 1/2, 1/4: every intermediate is exact in fp16 and fp32
        assert np.array_equal(got, want), tap


def test_winograd_agrees_with_direct_kernel_and_is_deterministic(tvg):
    import torch
    sh = ti.ConvShape("w", 4, 128, 28, 28, 128, 3, 3, 1, 1)
    inp = ti.make_inputs(sh, 4242, "bf16", residual=True)
    a = run_prepacked(tvg, sh, inp)
    b = run_prepacked(tvg, sh, inp)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    d = dev_inputs(inp, "bf16")
    direct = tvg.conv2d_fused(d["x"], d["w"], d["scale"], d["shift"], d["bias"], d["residual"],
                              stride=1, pad=1, relu=True)
    torch.cuda.synchronize()
    assert rel_err(to_host(a), to_host(direct)) <= WINO_TIGHT


def test_winograd_rejects_what_it_does_not_cover(tvg):
    import torch
    bad = [dict(stride=2), dict(c=32), dict(k=96), dict(r=1, pad=0), dict(dtype=tvg.TVG_F32), dict(pad=0)]
    for kw in bad:
        f = dict(n=1, c=64, h=8, w=8, k=64, r=3, stride=1, pad=1, dtype=tvg.TVG_BF16)
        f.update(kw)
        desc = tvg.ConvDesc(f["n"], f["c"], f["h"], f["w"], f["k"], f["r"], f["r"], f["stride"],
                            f["stride"], f["pad"], f["pad"], f["dtype"], 0)
        with pytest.raises(tvg.TvgError) as e:
            tvg.tvg_conv2d_prepack_size(desc)
        assert e.value.status == 3, kw
    desc = tvg.ConvDesc(1, 64, 8, 8, 64, 3, 3, 1, 1, 1, 1, tvg.TVG_BF16, 0)
    pb, wb = tvg.tvg_conv2d_prepack_size(desc)
    buf = torch.zeros(max(pb, wb) + 512, dtype=torch.uint8, device="cuda")
    f32 = torch.zeros(64, device="cuda")
    y = torch.zeros((1, 64, 8, 8), dtype=torch.bfloat16, device="cuda")
    assert tvg.tvg_conv2d_prepack(desc, buf, buf, pb - 1) == 4                       # short packed buffer
    assert tvg.tvg_conv2d_fused_prepacked(desc, buf, buf, f32, f32, None, None, y, buf, wb - 1) == 4
    assert tvg.tvg_conv2d_fused_prepacked(desc, buf, buf, f32, f32, None, None, y, None, 0) == 4
    assert tvg.tvg_conv2d_fused_prepacked(desc, buf, buf, f32, f32, None, None, y, buf[16:], wb) == 4
    assert tvg.tvg_conv2d_fused_prepacked(desc, None, buf, f32, f32, None, None, y, buf, wb) == 1
