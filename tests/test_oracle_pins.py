"""Pins for the CPU oracle: everything here runs without a GPU.

The TVM paper prints no worked numeric example for its operators, so the oracle
is pinned by what the mathematics fixes: an independent brute force (explicit
zero-padded array + window views), library routines for the same definition
(numpy matmul, torch CPU float64 conv2d), exact closed forms (identity kernel,
shifted delta, tap counts of an all-ones problem) and invariants (linearity,
depthwise = block-diagonal dense, epilogue identities).
"""
import itertools
import os

import numpy as np
import pytest
from numpy.lib.stride_tricks import sliding_window_view

import oracle
import tvg_inputs as ti

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------------------------
# an independent brute force: pad explicitly, take strided windows, contract with einsum
# ------------------------------------------------------------------------------------

def brute_conv(x, w, stride, pad):
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    xp = np.pad(x, ((0, 0), (0, 0), (pad[0], pad[0]), (pad[1], pad[1])))
    R, S = w.shape[2:]
    win = sliding_window_view(xp, (R, S), axis=(2, 3))[:, :, ::stride[0], ::stride[1]]
    return np.einsum("nchwrs,kcrs->nkhw", win, w)          # [N][OC][OH][OW]


def brute_depthwise(x, w, stride, pad):
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)[:, 0]
    xp = np.pad(x, ((0, 0), (0, 0), (pad[0], pad[0]), (pad[1], pad[1])))
    R, S = w.shape[1:]
    win = sliding_window_view(xp, (R, S), axis=(2, 3))[:, :, ::stride[0], ::stride[1]]
    return np.einsum("nchwrs,crs->nchw", win, w)


def rand(rng, *shape):
    return rng.uniform(-1, 1, size=shape).astype(np.float32)


ONES = lambda n: np.ones(n, np.float32)
ZEROS = lambda n: np.zeros(n, np.float32)


TINY = [
    # N, IC, H, W, OC, R, S, sh, sw, ph, pw
    (1, 1, 5, 5, 1, 3, 3, 1, 1, 1, 1),
    (2, 3, 7, 6, 4, 3, 3, 1, 1, 1, 1),
    (2, 3, 7, 6, 4, 3, 3, 2, 2, 1, 1),
    (1, 4, 6, 7, 2, 1, 1, 1, 1, 0, 0),
    (2, 2, 7, 7, 3, 1, 1, 2, 2, 0, 0),
    (1, 3, 11, 9, 2, 7, 7, 2, 2, 3, 3),
    (1, 2, 8, 8, 3, 3, 3, 2, 2, 0, 0),
    (1, 2, 9, 5, 3, 3, 2, 2, 1, 1, 0),      # R != S, stride and pad differ per axis
    (2, 3, 6, 10, 2, 5, 3, 1, 3, 2, 1),
    (1, 4, 4, 4, 4, 3, 3, 1, 1, 3, 3),      # padding wider than the usual k//2
]


@pytest.mark.parametrize("cfg", TINY)
def test_dense_matches_brute_force(cfg):
    N, IC, H, W, OC, R, S, sh, sw, ph, pw = cfg
    rng = np.random.default_rng(hash(cfg) % (2 ** 32))
    x, w = rand(rng, N, IC, H, W), rand(rng, OC, IC, R, S)
    got = oracle.conv2d_fused(x, w, ONES(OC), ZEROS(OC), stride=(sh, sw), pad=(ph, pw))
    want = brute_conv(x, w, (sh, sw), (ph, pw))
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("cfg", TINY)
def test_dense_matches_torch_float64(cfg):
    torch = pytest.importorskip("torch")
    N, IC, H, W, OC, R, S, sh, sw, ph, pw = cfg
    rng = np.random.default_rng(7 + hash(cfg) % (2 ** 32))
    x, w = rand(rng, N, IC, H, W), rand(rng, OC, IC, R, S)
    got = oracle.conv2d_fused(x, w, ONES(OC), ZEROS(OC), stride=(sh, sw), pad=(ph, pw))
    want = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                      stride=(sh, sw), padding=(ph, pw)).numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("stride,pad,H,W,C", [(1, 1, 7, 7, 3), (2, 1, 8, 6, 4), (2, 1, 7, 9, 2),
                                               (1, 0, 5, 5, 2)])
def test_depthwise_matches_brute_force_and_torch(stride, pad, H, W, C):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(100 * stride + H)
    x, w = rand(rng, 2, C, H, W), rand(rng, C, 1, 3, 3)
    got = oracle.dwconv2d_fused(x, w, ONES(C), ZEROS(C), stride=(stride, stride), pad=(pad, pad))
    np.testing.assert_allclose(got, brute_depthwise(x, w, (stride, stride), (pad, pad)),
                               rtol=0, atol=1e-12)
    want = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                      stride=stride, padding=pad, groups=C).numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_pointwise_conv_is_a_matmul():
    rng = np.random.default_rng(1)
    N, IC, H, W, OC = 2, 5, 6, 7, 3
    x, w = rand(rng, N, IC, H, W), rand(rng, OC, IC, 1, 1)
    got = oracle.conv2d_fused(x, w, ONES(OC), ZEROS(OC))
    for n in range(N):
        want = w[:, :, 0, 0].astype(np.float64) @ x[n].reshape(IC, H * W).astype(np.float64)
        np.testing.assert_allclose(got[n].reshape(OC, H * W), want, rtol=0, atol=1e-13)


def test_identity_kernel_is_a_copy():
    rng = np.random.default_rng(2)
    C = 4
    x = rand(rng, 2, C, 6, 5)
    w = np.zeros((C, C, 3, 3), np.float32)
    w[np.arange(C), np.arange(C), 1, 1] = 1.0
    got = oracle.conv2d_fused(x, w, ONES(C), ZEROS(C), pad=(1, 1))
    assert np.array_equal(got, x.astype(np.float64))


@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("r,s", list(itertools.product(range(3), range(3))))
def test_single_tap_is_a_shift(stride, r, s):
    """A kernel with one unit tap at (r, s) reads x at (oh*stride - pad + r, ow*stride - pad + s):
    pins the padding side, the stride phase and the absence of a kernel flip."""
    rng = np.random.default_rng(3)
    H, W, pad = 8, 6, 1
    x = rand(rng, 1, 1, H, W)
    w = np.zeros((1, 1, 3, 3), np.float32)
    w[0, 0, r, s] = 1.0
    got = oracle.conv2d_fused(x, w, ONES(1), ZEROS(1), stride=(stride, stride), pad=(pad, pad))
    OH, OW = (H + 2 - 3) // stride + 1, (W + 2 - 3) // stride + 1
    want = np.zeros((1, 1, OH, OW))
    for oh in range(OH):
        for ow in range(OW):
            ih, iw = oh * stride - pad + r, ow * stride - pad + s
            if 0 <= ih < H and 0 <= iw < W:
                want[0, 0, oh, ow] = x[0, 0, ih, iw]
    assert np.array_equal(got, want)


def test_all_ones_counts_in_bounds_taps():
    IC = 5
    x = np.ones((1, IC, 6, 6), np.float32)
    w = np.ones((2, IC, 3, 3), np.float32)
    y = oracle.conv2d_fused(x, w, ONES(2), ZEROS(2), pad=(1, 1))[0, 0]
    assert y[0, 0] == y[0, 5] == y[5, 0] == y[5, 5] == 4 * IC       # corners
    assert np.all(y[0, 1:5] == 6 * IC) and np.all(y[1:5, 0] == 6 * IC)   # edges
    assert np.all(y[5, 1:5] == 6 * IC) and np.all(y[1:5, 5] == 6 * IC)
    assert np.all(y[1:5, 1:5] == 9 * IC)                            # interior
    # stride 2 on an even size: the top/left border is clipped, the bottom/right one is not
    y2 = oracle.conv2d_fused(x, w, ONES(2), ZEROS(2), stride=(2, 2), pad=(1, 1))[0, 1]
    assert y2.shape == (3, 3)
    assert y2[0, 0] == 4 * IC and y2[0, 2] == 6 * IC and y2[2, 0] == 6 * IC and y2[2, 2] == 9 * IC
    # 7x7, pad 3, stride 2 on a 10x10 all-ones image: rows in range for oh=0 are r=3..6 (4 taps)
    x3 = np.ones((1, 1, 10, 10), np.float32)
    w3 = np.ones((1, 1, 7, 7), np.float32)
    y3 = oracle.conv2d_fused(x3, w3, ONES(1), ZEROS(1), stride=(2, 2), pad=(3, 3))[0, 0]
    assert y3.shape == (5, 5)
    assert y3[0, 0] == 16 and y3[2, 2] == 49 and y3[0, 2] == 28 and y3[4, 4] == 25


def test_linearity_in_input_and_weights():
    rng = np.random.default_rng(4)
    x1, x2 = rand(rng, 1, 3, 7, 7), rand(rng, 1, 3, 7, 7)
    w1, w2 = rand(rng, 4, 3, 3, 3), rand(rng, 4, 3, 3, 3)
    # coefficients and sums chosen exactly representable so both sides see the same inputs
    a, b = 0.5, -2.0
    f = lambda x, w: oracle.conv2d_fused(x, w, ONES(4), ZEROS(4), stride=(2, 2), pad=(1, 1))
    # use values on a coarse grid so a*x1+b*x2 is exact in float32
    g1 = np.round(x1 * 64) / 64
    g2 = np.round(x2 * 64) / 64
    gs = (a * g1 + b * g2).astype(np.float32)
    np.testing.assert_allclose(f(gs, w1), a * f(g1, w1) + b * f(g2, w1), rtol=0, atol=1e-12)
    v1 = np.round(w1 * 64) / 64
    v2 = np.round(w2 * 64) / 64
    vs = (a * v1 + b * v2).astype(np.float32)
    np.testing.assert_allclose(f(g1, vs), a * f(g1, v1) + b * f(g1, v2), rtol=0, atol=1e-12)


@pytest.mark.parametrize("stride", [1, 2])
def test_depthwise_equals_block_diagonal_dense(stride):
    rng = np.random.default_rng(5)
    C = 5
    x, wd = rand(rng, 2, C, 9, 8), rand(rng, C, 1, 3, 3)
    dense = np.zeros((C, C, 3, 3), np.float32)
    dense[np.arange(C), np.arange(C)] = wd[:, 0]
    scale, shift = rand(rng, C) + 2, rand(rng, C)
    a = oracle.dwconv2d_fused(x, wd, scale, shift, stride=(stride, stride), pad=(1, 1), relu=True)
    b = oracle.conv2d_fused(x, dense, scale, shift, stride=(stride, stride), pad=(1, 1), relu=True)
    assert np.array_equal(a, b)


def test_epilogue_identities():
    rng = np.random.default_rng(6)
    N, IC, H, W, OC = 2, 3, 6, 6, 4
    x, w = rand(rng, N, IC, H, W), rand(rng, OC, IC, 3, 3)
    scale, shift, bias = rand(rng, OC) + 2, rand(rng, OC), rand(rng, OC)
    res = rand(rng, N, OC, H, W)
    kw = dict(stride=(1, 1), pad=(1, 1))
    raw = brute_conv(x, w, (1, 1), (1, 1))
    sc = scale.astype(np.float64)[None, :, None, None]
    sf = shift.astype(np.float64)[None, :, None, None]
    bs = bias.astype(np.float64)[None, :, None, None]
    # the full chain, written out: bias, then scale and shift, then residual, then ReLU
    want = np.maximum((raw + bs) * sc + sf + res.astype(np.float64), 0.0)
    got = oracle.conv2d_fused(x, w, scale, shift, bias, res, relu=True, **kw)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    # each stage alone
    np.testing.assert_allclose(oracle.conv2d_fused(x, w, scale, shift, **kw), raw * sc + sf,
                               rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.conv2d_fused(x, w, scale, shift, None, res, **kw),
                               raw * sc + sf + res, rtol=0, atol=1e-12)
    # residual is added after the scale (not scaled) and before the ReLU (can be clipped)
    assert (got == 0).any() and (got > 0).any()
    # zero weights: only the shift and the residual survive
    z = oracle.conv2d_fused(x, 0 * w, scale, shift, None, res, relu=True, **kw)
    np.testing.assert_allclose(z, np.maximum(sf + res, 0.0), rtol=0, atol=0)
    # zero scale wipes the convolution and the bias
    z = oracle.conv2d_fused(x, w, 0 * scale, shift, bias, None, relu=False, **kw)
    np.testing.assert_allclose(z, np.broadcast_to(sf, z.shape), rtol=0, atol=0)
    # the depthwise entry point applies the same tail
    wd = rand(rng, IC, 1, 3, 3)
    s3, f3, b3 = rand(rng, IC) + 2, rand(rng, IC), rand(rng, IC)
    r3 = rand(rng, N, IC, H, W)
    d = oracle.dwconv2d_fused(x, wd, s3, f3, b3, r3, relu=True, **kw)
    dw_raw = brute_depthwise(x, wd, (1, 1), (1, 1))
    e = lambda v: v.astype(np.float64)[None, :, None, None]
    np.testing.assert_allclose(d, np.maximum((dw_raw + e(b3)) * e(s3) + e(f3) + r3, 0.0),
                               rtol=0, atol=1e-12)


def test_sampled_entry_point_equals_full():
    rng = np.random.default_rng(8)
    N, IC, H, W, OC = 2, 3, 9, 7, 5
    x, w = rand(rng, N, IC, H, W), rand(rng, OC, IC, 3, 3)
    scale, shift = rand(rng, OC) + 2, rand(rng, OC)
    res = rand(rng, N, OC, 5, 4)
    full = oracle.conv2d_fused(x, w, scale, shift, None, res, stride=(2, 2), pad=(1, 1), relu=True)
    idx = rng.choice(full.size, size=50, replace=False)
    part = oracle.conv2d_fused_at(x, w, scale, shift, None, res, idx=idx, stride=(2, 2),
                                  pad=(1, 1), relu=True)
    assert np.array_equal(part, full.reshape(-1)[idx])


def test_thread_count_does_not_change_bits():
    rng = np.random.default_rng(9)
    x, w = rand(rng, 2, 8, 12, 12), rand(rng, 6, 8, 3, 3)
    n0 = oracle.num_threads()
    a = oracle.conv2d_fused(x, w, ONES(6), ZEROS(6), pad=(1, 1))
    oracle.set_num_threads(1)
    b = oracle.conv2d_fused(x, w, ONES(6), ZEROS(6), pad=(1, 1))
    oracle.set_num_threads(n0)
    assert np.array_equal(a, b)


def test_maxpool_against_brute_force_and_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(10)
    for H, W in [(8, 8), (7, 9), (6, 5)]:
        x = rand(rng, 2, 3, H, W)
        got = oracle.maxpool2d(x, k=3, stride=2, pad=1)
        xp = np.pad(x.astype(np.float64), ((0, 0), (0, 0), (1, 1), (1, 1)), constant_values=-np.inf)
        win = sliding_window_view(xp, (3, 3), axis=(2, 3))[:, :, ::2, ::2]
        assert np.array_equal(got, win.max(axis=(4, 5)))
        want = torch.nn.functional.max_pool2d(torch.from_numpy(x).double(), 3, 2, 1).numpy()
        assert np.array_equal(got, want)


def test_bf16_rounding():
    # hand-checked values: the bf16 grid near 1 has spacing 2^-7
    cases = {1.0: 1.0, 1.0 + 2 ** -8: 1.0, 1.0 + 3 * 2 ** -8: 1.0 + 2 ** -6,
             1.0 + 2 ** -8 + 2 ** -20: 1.0 + 2 ** -7, -(1.0 + 2 ** -8): -1.0,
             0.0: 0.0, 3.0: 3.0, 255.5: 256.0, 0.1: 0.10009765625, 1e-3: 0.00099945068359375}
    got = oracle.round_to_bf16(np.array(list(cases.keys()), dtype=np.float64))
    assert np.array_equal(got.astype(np.float64), np.array(list(cases.values())))
    # against the independent bit-level rounding of the input generator, on float32 inputs
    rng = np.random.default_rng(11)
    v = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000),
                        ti.bf16_bits_to_f32(rng.integers(0x3000, 0x4800, 2000).astype(np.uint16))
                        .astype(np.float64) * (1 + 2.0 ** -8)]).astype(np.float32)
    assert np.array_equal(oracle.round_to_bf16(v.astype(np.float64)), ti.quantize_bf16(v))
    # values already on the grid are unchanged
    q = ti.quantize_bf16(v)
    assert np.array_equal(oracle.round_to_bf16(q.astype(np.float64)), q)


def test_shape_tables_match_the_papers_table():
    rows = {}
    with open(os.path.join(GOLDEN, "table2_shapes.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, hw, ic, oc, k, s, out = line.split()
            rows[name] = tuple(int(v) for v in (hw, ic, oc, k, s, out))
    shapes = ti.resnet18_convs(1) + ti.mobilenet_depthwise(1)
    assert [s.name for s in shapes] == list(rows)
    for sh in shapes:
        hw, ic, oc, k, s, out = rows[sh.name]
        assert (sh.h, sh.w, sh.ic, sh.oc, sh.r, sh.s, sh.stride) == (hw, hw, ic, oc, k, k, s)
        assert sh.pad == k // 2
        assert sh.oh == sh.ow == out == -(-hw // s)         # "SAME": ceil(H / S)
        assert sh.depthwise == sh.name.startswith("D")
    # the oracle derives the same output extents
    for sh in shapes:
        assert oracle.out_extent(sh.h, sh.pad, sh.r, sh.stride) == sh.oh


def test_body_graph_has_the_expected_convs():
    steps = ti.resnet18_body(2)
    convs = [s for s in steps if s.op == "conv"]
    assert len(convs) == 20 and sum(s.op == "maxpool" for s in steps) == 1
    from collections import Counter
    cnt = Counter(s.shape.name for s in convs)
    assert cnt == {"C1": 1, "C2": 4, "C4": 1, "C5": 1, "C6": 3, "C7": 1, "C8": 1, "C9": 3,
                   "C10": 1, "C11": 1, "C12": 3}
    assert sum(s.shape.flops for s in convs) // 2 == 2 * 1813561344   # 1.814 GMAC per image


def test_body_chain_small_runs_and_rounds():
    """The chained oracle stores bf16: every tensor it returns lies on the bf16 grid."""
    from oracle.resnet_body import run_steps
    steps = ti.resnet18_body(1)[:4]          # stem, pool, first block conv1
    w = {s.layer_index: ti.make_weights(s.shape, ti.layer_seed(5, s.layer_index), "bf16")
         for s in steps if s.op == "conv"}
    img = ti.body_images(1, ti.layer_seed(5, 999))
    out = run_steps(steps, img, w)
    for t in out.values():
        assert np.array_equal(ti.quantize_bf16(t), t)
    assert out[steps[-1].dst].shape == (1, 64, 56, 56)


def test_mobilenet_body_graph_has_the_expected_layers():
    """13 depthwise + 13 pointwise + the stem; 567.7 M multiply-adds per image (the network's
    published 569 M includes the 1.0 M of its classifier, which is not part of the body)."""
    steps = ti.mobilenet_body(2)
    from collections import Counter
    assert Counter(s.op for s in steps) == {"conv": 14, "dwconv": 13}
    cnt = Counter(s.shape.name for s in steps if s.op == "dwconv")
    assert cnt == {"D1": 1, "D2": 1, "D3": 1, "D4": 1, "D5": 1, "D6": 1, "D7": 5, "D8": 1, "D9": 1}
    assert sum(s.shape.flops for s in steps) // 2 == 2 * 567716352
    prev = None
    for s in steps:                                 # a plain chain: each layer reads the last one
        if prev is not None:
            assert s.src == prev.dst and s.shape.x_shape() == prev.shape.y_shape()
        prev = s
    assert steps[-1].shape.y_shape() == (2, 1024, 7, 7)
    assert [s.layer_index for s in steps] == list(range(27))


@pytest.mark.parametrize("stride", [1, 2])
def test_chain_depthwise_then_pointwise_equals_the_factorised_dense_conv(stride):
    """A depthwise 3x3 followed by a 1x1 conv (no tail in between) is the dense 3x3 conv with
    weights pw[oc][c] * dw[c][r][s]: pins the chain's depthwise step and its wiring against
    the dense operator."""
    from oracle.resnet_body import run_steps
    rng = np.random.default_rng(77 + stride)
    n, c, h, w, oc = 2, 5, 9, 8, 7
    d = ti.ConvShape("d", n, c, h, w, c, 3, 3, stride, 1, depthwise=True)
    p = ti.ConvShape("p", n, c, d.oh, d.ow, oc, 1, 1, 1, 0)
    steps = [ti.Step("dwconv", "dw", 0, 1, d, None, False, 0), ti.Step("conv", "pw", 1, 2, p, None, True, 1)]
    wd, wp = rand(rng, c, 1, 3, 3), rand(rng, oc, c, 1, 1)
    scale, shift = rand(rng, oc) + 2.0, rand(rng, oc)
    weights = {0: {"w": wd, "scale": np.ones(c, np.float32), "shift": np.zeros(c, np.float32)},
               1: {"w": wp, "scale": scale, "shift": shift}}
    x = rand(rng, n, c, h, w)
    got = run_steps(steps, x, weights, store_bf16=False)[2]
    dense_w = (wp[:, :, 0, 0][:, :, None, None].astype(np.float64) * wd[:, 0][None].astype(np.float64))
    want = oracle.conv2d_fused(x, dense_w.astype(np.float32), scale, shift, None, None,
                               stride=(stride, stride), pad=(1, 1), relu=True)
    assert got.shape == want.shape == (n, oc, d.oh, d.ow)
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-6)     # fp32 storage of the two stages


@pytest.mark.parametrize("stride", [1, 2])
def test_dwpw_block_equals_the_factorised_dense_conv_and_a_matmul(stride):
    """The MobileNet block oracle against two independent forms.  (1) Without a depthwise
    tail it is the dense 3x3 conv with weights pw[k][c] * dw[c][r][s].  (2) With the tail,
    the second stage is a plain matrix product over channels of the brute-force depthwise
    result (scale/shift/ReLU applied, rounded to bf16 by the input module's bit routine)."""
    rng = np.random.default_rng(910 + stride)
    n, c, h, w, k = 2, 6, 7, 10, 5
    x, wd, wp = rand(rng, n, c, h, w), rand(rng, c, 1, 3, 3), rand(rng, k, c, 1, 1)
    sd, fd = rand(rng, c) + 2.0, rand(rng, c)
    sp, fp, bp = rand(rng, k) + 2.0, rand(rng, k), rand(rng, k)
    ones, zeros = np.ones(c, np.float32), np.zeros(c, np.float32)
    got = oracle.dwpw_fused(x, wd, ones, zeros, wp, sp, fp, stride=stride, relu_dw=False,
                            relu_pw=True, store="f32")
    dense_w = wp[:, :, 0, 0][:, :, None, None].astype(np.float64) * wd[:, 0][None].astype(np.float64)
    want = oracle.conv2d_fused(x, dense_w.astype(np.float32), sp, fp, None, None,
                               stride=(stride, stride), pad=(1, 1), relu=True)
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-6)

    t = brute_depthwise(x, wd, (stride, stride), (1, 1)) * sd.astype(np.float64)[None, :, None, None] \
        + fd.astype(np.float64)[None, :, None, None]
    t = ti.quantize_bf16(np.maximum(t, 0.0).astype(np.float32)).astype(np.float64)
    oh, ow = t.shape[2:]
    res = rand(rng, n, k, oh, ow)
    z = np.einsum("kc,nchw->nkhw", wp[:, :, 0, 0].astype(np.float64), t)
    z = (z + bp.astype(np.float64)[None, :, None, None]) * sp.astype(np.float64)[None, :, None, None] \
        + fp.astype(np.float64)[None, :, None, None] + res
    got = oracle.dwpw_fused(x, wd, sd, fd, wp, sp, fp, bp, res, stride=stride, relu_dw=True,
                            relu_pw=False, store="bf16")
    # the bf16 rounding of t can flip where the fp64 and float32 sums straddle a tie: none here
    np.testing.assert_allclose(got, z, rtol=0, atol=1e-9)


# ------------------------------------------------------------------------------------
# the chain runner (residual wiring, projection shortcut, max-pool, storage rounding) against
# the same networks composed by hand from torch's float64 CPU routines
# ------------------------------------------------------------------------------------

def bf16_nearest_even(y64):
    """fp64 -> nearest bfloat16 (8 significant bits, ties to even) through frexp / rint /
    ldexp: no bit tricks, independent of the oracle's and the input module's routines."""
    m, e = np.frexp(np.asarray(y64, dtype=np.float64))          # |m| in [0.5, 1)
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


def torch_layer(x64, p, stride, pad, residual=None, relu=True, groups=1):
    """One fused layer as the paper's Section 3 fusion defines it, from library calls:
    conv2d, per-channel scale and shift, shortcut add, ReLU, storage rounding."""
    import torch
    import torch.nn.functional as F
    y = F.conv2d(torch.from_numpy(x64), torch.from_numpy(p["w"].astype(np.float64)), None, stride,
                 pad, 1, groups).numpy()
    y = y * p["scale"].astype(np.float64)[None, :, None, None] \
        + p["shift"].astype(np.float64)[None, :, None, None]
    if residual is not None:
        y = y + residual
    if relu:
        y = np.maximum(y, 0.0)
    return bf16_nearest_even(y)


def torch_pool(x64):
    import torch
    import torch.nn.functional as F
    return F.max_pool2d(torch.from_numpy(x64), 3, 2, 1).numpy()


def differs(a, b):
    """Fraction of elements on which two stored tensors disagree."""
    return float(np.mean(np.asarray(a, np.float64) != np.asarray(b, np.float64)))


def test_chain_runner_small_network_against_hand_composition_and_wrong_wirings():
    """Stem conv, max-pool, an identity-shortcut block and a down-sampling block with a 1x1
    stride-2 projection: every stored tensor of run_steps equals the network written out by
    hand.  The same network with the shortcut taken from the wrong tensor, without the pool,
    with ReLU on the projection or without the storage rounding is far from it, so each of
    those mistakes in run_steps would fail here."""
    from oracle.resnet_body import run_steps
    n, c0, c1, c2, hw = 2, 3, 8, 12, 18
    S = ti.ConvShape
    shapes = {"stem": S("stem", n, c0, hw, hw, c1, 3, 3, 1, 1),
              "a1": S("a1", n, c1, 9, 9, c1, 3, 3, 1, 1), "a2": S("a2", n, c1, 9, 9, c1, 3, 3, 1, 1),
              "b1": S("b1", n, c1, 9, 9, c2, 3, 3, 2, 1), "bp": S("bp", n, c1, 9, 9, c2, 1, 1, 2, 0),
              "b2": S("b2", n, c2, 5, 5, c2, 3, 3, 1, 1)}
    steps = [ti.Step("conv", "stem", 0, 1, shapes["stem"], None, True, 0),
             ti.Step("maxpool", "pool", 1, 2),
             ti.Step("conv", "a1", 2, 3, shapes["a1"], None, True, 1),
             ti.Step("conv", "a2", 3, 4, shapes["a2"], 2, True, 2),
             ti.Step("conv", "b1", 4, 5, shapes["b1"], None, True, 3),
             ti.Step("conv", "bp", 4, 6, shapes["bp"], None, False, 4),
             ti.Step("conv", "b2", 5, 7, shapes["b2"], 6, True, 5)]
    names = ["stem", "a1", "a2", "b1", "bp", "b2"]
    W = {i: ti.make_weights(shapes[k], 4100 + i, "bf16") for i, k in enumerate(names)}
    rng = np.random.default_rng(4099)
    img = ti.quantize_bf16(rng.uniform(-1, 1, (n, c0, hw, hw)).astype(np.float32))
    got = run_steps(steps, img, W)

    x = img.astype(np.float64)
    t1 = torch_layer(x, W[0], 1, 1)
    t2 = torch_pool(t1)
    t3 = torch_layer(t2, W[1], 1, 1)
    t4 = torch_layer(t3, W[2], 1, 1, residual=t2)
    t5 = torch_layer(t4, W[3], 2, 1)
    t6 = torch_layer(t4, W[4], 2, 0, relu=False)
    t7 = torch_layer(t5, W[5], 1, 1, residual=t6)
    for k, want in {1: t1, 2: t2, 3: t3, 4: t4, 5: t5, 6: t6, 7: t7}.items():
        assert got[k].shape == want.shape
        assert np.array_equal(got[k].astype(np.float64), want), k
    assert (t6 < 0).any()                       # the projection really carries no ReLU
    assert t2.shape == (n, c1, 9, 9) and t7.shape == (n, c2, 5, 5)

    # planted mistakes, each composed by hand, must NOT reproduce the runner's tensors
    wrong_identity = torch_layer(t3, W[2], 1, 1, residual=t3)            # shortcut = conv2's own input
    assert differs(wrong_identity, got[4]) > 0.5
    no_shortcut = torch_layer(t3, W[2], 1, 1)
    assert differs(no_shortcut, got[4]) > 0.5
    wrong_proj = torch_layer(t5, W[5], 1, 1, residual=torch_layer(t4, W[4], 2, 0, relu=True))
    assert differs(wrong_proj, got[7]) > 0.1                             # ReLU on the projection
    pool_as_stride = t1[:, :, ::2, ::2]                                  # pool replaced by subsampling
    assert differs(torch_layer(pool_as_stride, W[1], 1, 1), got[3]) > 0.5
    unrounded = run_steps(steps, img, W, store_bf16=False)
    assert differs(unrounded[7], got[7]) > 0.5                           # storage rounding is applied


def torch_resnet18_body(img, W):
    """The ResNet-18 convolutional body (basic blocks, projection shortcuts on the three
    down-sampling blocks) written as nested code, not from the launch list; the weights of
    layer i in launch order are W[i]."""
    it = iter(range(20))
    x = torch_layer(img.astype(np.float64), W[next(it)], 2, 3)
    x = torch_pool(x)
    for stage, down in ((0, False), (1, True), (2, True), (3, True)):
        for block in range(2):
            first = block == 0 and down
            a = torch_layer(x, W[next(it)], 2 if first else 1, 1)
            shortcut = torch_layer(x, W[next(it)], 2, 0, relu=False) if first else x
            x = torch_layer(a, W[next(it)], 1, 1, residual=shortcut)
    return x


def test_chain_runner_resnet18_body_against_hand_composition():
    """The 21-launch list of the ResNet-18 body at batch 1 through run_steps against the network
    composed by hand from torch float64 calls.  Two fp64 sums in different orders can land on
    opposite sides of a bf16 tie about once in 10^13 values, so the stored tensors agree bit for
    bit here; the assertion leaves room for a handful of such flips."""
    from oracle.resnet_body import run_steps
    steps = ti.resnet18_body(1)
    W = {s.layer_index: ti.make_weights(s.shape, ti.layer_seed(5, s.layer_index), "bf16")
         for s in steps if s.op == "conv"}
    img = ti.body_images(1, ti.layer_seed(5, 998))
    got = run_steps(steps, img, W)[steps[-1].dst].astype(np.float64)
    want = torch_resnet18_body(img, W)
    assert got.shape == want.shape == (1, 512, 7, 7)
    assert differs(got, want) < 1e-3
    rho = float(np.sqrt(np.mean(want * want)))
    assert rho > 0.1 and np.max(np.abs(got - want)) <= 1e-2 * rho


def test_chain_runner_mobilenet_body_against_hand_composition():
    """The 27-launch MobileNet body at batch 1 against stem + 13 x (depthwise via groups = C, 1x1)
    written as a loop over the block table."""
    from oracle.resnet_body import run_steps
    steps = ti.mobilenet_body(1)
    W = {s.layer_index: ti.make_weights(s.shape, ti.layer_seed(6, s.layer_index), "bf16")
         for s in steps}
    img = ti.body_images(1, ti.layer_seed(6, 998))
    got = run_steps(steps, img, W)[steps[-1].dst].astype(np.float64)
    strides = [1, 2, 1, 2, 1, 2, 1, 1, 1, 1, 1, 2, 1]
    x = torch_layer(img.astype(np.float64), W[0], 2, 1)
    for b, s in enumerate(strides):
        x = torch_layer(x, W[1 + 2 * b], s, 1, groups=x.shape[1])
        x = torch_layer(x, W[2 + 2 * b], 1, 0)
    assert got.shape == x.shape == (1, 1024, 7, 7)
    assert differs(got, x) < 1e-3
    rho = float(np.sqrt(np.mean(x * x)))
    assert rho > 0.01 and np.max(np.abs(got - x)) <= 1e-2 * rho


def test_chain_runner_two_head_steps_equal_the_separate_steps():
    """The ResNet-18 launch list with the down-sampling blocks' first conv and projection recorded
    as one two-head step (18 launches) yields, tensor by tensor, what the 21-launch list yields:
    the two-head step is by definition the two operators evaluated separately."""
    from oracle.resnet_body import run_steps
    plain, fused = ti.resnet18_body(1), ti.resnet18_body(1, fuse_projection=True)
    assert len(plain) == 21 and len(fused) == 18
    assert sum(s.op == "conv_dual" for s in fused) == 3
    for s in fused:
        if s.op == "conv_dual":          # a 3x3 and a 1x1 of the same input, same stride and outputs
            assert (s.shape.r, s.shape2.r, s.shape2.pad) == (3, 1, 0) and s.shape.stride == s.shape2.stride == 2
            assert s.shape.x_shape() == s.shape2.x_shape() and s.shape.y_shape() == s.shape2.y_shape()
            assert s.relu and not s.relu2
    W = {s.layer_index: ti.make_weights(s.shape, ti.layer_seed(5, s.layer_index), "bf16")
         for s in plain if s.op == "conv"}
    img = ti.body_images(1, ti.layer_seed(5, 997))
    a, b = run_steps(plain, img, W), run_steps(fused, img, W)
    assert sorted(a) == sorted(b)
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    assert ti.tensor_lives(plain).keys() == ti.tensor_lives(fused).keys()
