"""tvg_conv2d_fused_static: the entry point for callers that cannot allocate (no workspace
argument; split-reduction partials live in an array inside the library).  Through the C ABI,
against the existing entry point (bit for bit: same kernels) and against the oracle, on two calls
in a row, the second on a smaller problem that finds the first one's partials in the array."""
import numpy as np
import pytest

import oracle
import tvg_inputs as ti
from _util import check, dev_inputs, to_host

pytestmark = pytest.mark.gpu


def both_entry_points(tvg, sh, inp, dtype):
    import torch
    d = dev_inputs(inp, dtype)
    code = tvg.TVG_BF16 if dtype == "bf16" else tvg.TVG_F32
    desc = tvg.ConvDesc(sh.n, sh.ic, sh.h, sh.w, sh.oc, sh.r, sh.s, sh.stride, sh.stride, sh.pad,
                        sh.pad, code, tvg.TVG_RELU)
    need = tvg.tvg_conv2d_workspace_size(desc)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    y_static = torch.full(sh.y_shape(), float("nan"), dtype=tdt, device="cuda:0")
    y_ws = torch.full(sh.y_shape(), float("nan"), dtype=tdt, device="cuda:0")
    ws = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    st = tvg.tvg_conv2d_fused_static(desc, d["x"], d["w"], d["scale"], d["shift"], d["bias"],
                                     d["residual"], y_static)
    assert st == 0, tvg.status_string(st)
    st = tvg.tvg_conv2d_fused(desc, d["x"], d["w"], d["scale"], d["shift"], d["bias"],
                              d["residual"], y_ws, ws, need)
    assert st == 0, tvg.status_string(st)
    torch.cuda.synchronize()
    return need, y_static, y_ws


def test_static_scratch_entry_point_two_calls_in_a_row(tvg):
    import torch
    assert tvg.tvg_static_scratch_bytes() == 16 << 20
    # Problems whose reduction the generic kernel splits across workgroups (fp32 shapes the
    # one-launch fp32 kernels do not take: a 5x5 filter, input channels no multiple of 8).
    # first call: a 5x5 stride-2 layer on a 224x224 map (6.4 MB of partials); then 512 x 100 channels on a 7x7 map
    # (1.4 MB), then a small ragged problem (42 KB) - each finds the previous call's partials in
    # the array; last a bf16 problem that needs none
    calls = [(ti.ConvShape("five", 1, 5, 224, 224, 64, 5, 5, 2, 2), 29, "f32"),
             (ti.ConvShape("mid", 1, 100, 7, 7, 512, 3, 3, 1, 1), 30, "f32"),
             (ti.ConvShape("small", 1, 36, 5, 6, 70, 3, 3, 1, 1), 31, "f32"),
             (ti.ConvShape("small16", 2, 64, 6, 5, 33, 3, 3, 2, 1), 32, "bf16")]
    needs = []
    for sh, seed, dtype in calls:
        inp = ti.make_inputs(sh, seed, dtype, residual=True, bias=True)
        need, y_static, y_ws = both_entry_points(tvg, sh, inp, dtype)
        needs.append(need)
        assert not torch.isnan(y_static.float()).any()
        assert torch.equal(y_static, y_ws), sh.name            # same kernels, same order: same bits
        want = oracle.conv2d_fused(inp["x"], inp["w"], inp["scale"], inp["shift"], inp["bias"],
                                   inp["residual"], stride=(sh.stride,) * 2, pad=(sh.pad,) * 2,
                                   relu=True)
        check(to_host(y_static), want, dtype, sh.name)
    assert needs[0] > needs[1] > needs[2] > 0                  # the scratch really was in use


def test_static_scratch_entry_point_without_a_split_and_beyond_the_limit(tvg):
    import torch
    # a problem that needs no scratch (bf16 3x3, batch 8): the two entry points agree
    sh = ti.ConvShape("c6", 8, 128, 28, 28, 128, 3, 3, 1, 1)
    inp = ti.make_inputs(sh, 77, "bf16")
    need, y_static, y_ws = both_entry_points(tvg, sh, inp, "bf16")
    assert need == 0 and torch.equal(y_static, y_ws)
    # a problem whose partials exceed the array: an error code, nothing launched
    big = tvg.ConvDesc(1, 516, 28, 28, 512, 3, 3, 1, 1, 1, 1, tvg.TVG_F32, 0)
    assert tvg.tvg_conv2d_workspace_size(big) > tvg.tvg_static_scratch_bytes()
    y = torch.full((1, 512, 28, 28), 7.0, device="cuda:0")
    x = torch.zeros((1, 516, 28, 28), device="cuda:0")
    w = torch.zeros((512, 516, 3, 3), device="cuda:0")
    s = torch.ones(512, device="cuda:0")
    assert tvg.tvg_conv2d_fused_static(big, x, w, s, s, None, None, y) == 4
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
