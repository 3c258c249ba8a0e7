"""Boundary tests that need no GPU: the C-ABI library loads, exports every symbol the
header declares, and rejects bad arguments on the host before any device call."""
import ctypes
import os
import re

import pytest

import paper_1802_04799_amd as tvg
from paper_1802_04799_amd import ConvDesc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000  # a non-null "device pointer" for calls that must fail before touching it


def desc(**kw):
    base = dict(n=1, c=8, h=10, w=10, k=8, r=3, s=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1,
                dtype=tvg.TVG_F32, flags=0)
    base.update(kw)
    return ConvDesc(**base)


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "tvg.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(tvg_[a-z0-9_]+)\s*\(", header))
    assert {"tvg_conv2d_fused", "tvg_dwconv2d_fused", "tvg_conv2d_workspace_size",
            "tvg_dwconv2d_workspace_size", "tvg_maxpool2d_3x3s2", "tvg_status_string",
            "tvg_version", "tvg_conv2d_set_tile", "tvg_conv2d_get_plan", "tvg_dwpw_fused",
            "tvg_dwpw_workspace_size", "tvg_dwpw_one_kernel"} <= names
    lib = tvg.load()
    for n in names:
        assert hasattr(lib, n), n
    assert tvg.tvg_version() >= 100
    assert tvg.status_string(0) == "ok"


def test_struct_layout_matches_header():
    assert ctypes.sizeof(ConvDesc) == 13 * 4


@pytest.mark.parametrize("kw,status", [
    (dict(n=0), 2), (dict(c=-1), 2), (dict(h=0), 2), (dict(k=0), 2), (dict(r=0), 2),
    (dict(stride_h=0), 2), (dict(stride_w=9), 2), (dict(pad_h=-1), 2), (dict(pad_h=3), 2),
    (dict(h=1, w=1, r=5, s=5, pad_h=1, pad_w=1), 2),          # empty output
    (dict(dtype=2), 3), (dict(flags=4), 3), (dict(flags=8 | 1), 3), (dict(r=17, s=17, pad_h=8, pad_w=8, h=40, w=40), 3),
    (dict(n=64, c=4096, h=256, w=256), 3),                    # 2^34 input elements
])
def test_conv_rejects_bad_descriptors_on_the_host(kw, status):
    d = desc(**kw)
    with pytest.raises(tvg.TvgError) as e:
        tvg.tvg_conv2d_workspace_size(d)
    assert e.value.status == status
    assert tvg.tvg_conv2d_fused(d, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, None, 0, 0) == status


def test_null_pointers_are_rejected():
    d = desc()
    lib = tvg.load()
    assert lib.tvg_conv2d_workspace_size(None, ctypes.byref(ctypes.c_size_t())) == 1
    assert lib.tvg_conv2d_workspace_size(ctypes.byref(d), None) == 1
    for missing in range(5):
        args = [FAKE] * 5
        args[missing] = None
        x, w, scale, shift, y = args
        assert tvg.tvg_conv2d_fused(d, x, w, scale, shift, None, None, y, None, 0, 0) == 1
        dd = desc(k=8, c=8)
        assert tvg.tvg_dwconv2d_fused(dd, x, w, scale, shift, None, None, y, None, 0, 0) == 1
    assert tvg.tvg_maxpool2d_3x3s2(1, 1, 4, 4, 0, None, FAKE, 0) == 1
    assert tvg.tvg_maxpool2d_3x3s2(1, 1, 0, 4, 0, FAKE, FAKE, 0) == 2
    assert tvg.tvg_maxpool2d_3x3s2(1, 1, 4, 4, 7, FAKE, FAKE, 0) == 3


@pytest.mark.parametrize("kw,status", [
    (dict(k=16), 2), (dict(r=5, s=5, pad_h=2, pad_w=2), 3), (dict(stride_h=3, stride_w=3), 3),
    (dict(stride_h=1, stride_w=2), 3), (dict(pad_h=0, pad_w=0), 3), (dict(pad_h=2, pad_w=2), 3),
    (dict(pad_h=1, pad_w=0), 3),
])
def test_depthwise_rejects_what_it_does_not_build(kw, status):
    d = desc(**kw)
    assert tvg.tvg_dwconv2d_fused(d, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, None, 0, 0) == status
    with pytest.raises(tvg.TvgError):
        tvg.tvg_dwconv2d_workspace_size(d)


@pytest.mark.parametrize("kw", [
    dict(r=2**31 - 1, pad_h=2**31 - 2), dict(s=2**31 - 1, pad_w=2**31 - 2, w=3),
    dict(h=2**31 - 1, w=2**31 - 1, pad_h=2, pad_w=2), dict(r=2**30, s=2**30, pad_h=2**30 - 1, pad_w=5),
    dict(n=2**31 - 1, c=2**31 - 1, k=2**31 - 1),
    dict(n=1, c=1, k=1, h=2**31 - 1, w=1, pad_h=2, pad_w=0, s=1),      # output rows: 2^31 + 1
])
def test_extreme_descriptors_are_rejected_without_arithmetic_on_them(kw):
    """Extents near INT_MAX: the filter-size limit is checked before any sum involving the
    padding, and element counts are formed in 64 bits, so every such descriptor is an error
    code (bad shape or unsupported), from the query and from the operator alike."""
    d = desc(**kw)
    with pytest.raises(tvg.TvgError) as e:
        tvg.tvg_conv2d_workspace_size(d)
    assert e.value.status in (2, 3)
    assert tvg.tvg_conv2d_fused(d, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, None, 0, 0) == e.value.status
    assert tvg.tvg_maxpool2d_3x3s2(2**31 - 1, 2**31 - 1, 2**31 - 1, 2**31 - 1, 0, FAKE, FAKE, 0) == 3


@pytest.mark.parametrize("w,stride,dtype,ok", [
    (2726, 1, 0, True), (2727, 1, 0, False), (1817, 2, 1, True), (1818, 2, 1, False),
    (5001, 1, 0, False), (3001, 1, 1, False), (3001, 2, 1, False)])
def test_depthwise_row_width_limit_is_the_same_for_query_and_operator(w, stride, dtype, ok):
    """The documented limit (3*stride + 3) * (w + 2) <= 16372: the size query and the operator
    give the same answer on both sides of it (the operator is called with no pointers, so a
    descriptor that passes fails on the NULL check instead of launching)."""
    d = desc(n=1, c=8, k=8, h=8, w=w, stride_h=stride, stride_w=stride, dtype=dtype)
    op = tvg.tvg_dwconv2d_fused(d, None, None, None, None, None, None, None, None, 0, 0)
    if ok:
        assert tvg.tvg_dwconv2d_workspace_size(d) == 0 and op == 1
    else:
        with pytest.raises(tvg.TvgError) as e:
            tvg.tvg_dwconv2d_workspace_size(d)
        assert e.value.status == 3 and op == 3


def test_plans_do_not_depend_on_the_environment(monkeypatch):
    """No environment variable reaches planning: the variables an earlier build read change
    nothing, and the query agrees with itself across calls (plans are remembered)."""
    c6 = desc(n=64, c=128, h=28, w=28, k=128, dtype=tvg.TVG_BF16)
    c12 = desc(n=1, c=512, h=7, w=7, k=512)
    before = (tvg.tvg_conv2d_get_plan(c6), tvg.tvg_conv2d_workspace_size(c12))
    monkeypatch.setenv("TVG_FORCE_TILE", "64,64")
    monkeypatch.setenv("TVG_DBUF", "0")
    assert tvg.tvg_conv2d_set_tile(c6, 64, 128) == 0        # empties the remembered plans
    assert tvg.tvg_conv2d_set_tile(c6, 0, 0) == 0
    assert (tvg.tvg_conv2d_get_plan(c6), tvg.tvg_conv2d_workspace_size(c12)) == before
    # more distinct problems than the plan memory holds: old entries are replaced, answers stay
    for n in range(1, 300):
        tvg.tvg_conv2d_get_plan(desc(n=n, c=16, h=9, w=9, k=16, dtype=tvg.TVG_BF16))
    assert (tvg.tvg_conv2d_get_plan(c6), tvg.tvg_conv2d_workspace_size(c12)) == before


def test_workspace_query_and_too_small_workspace():
    # a large-batch problem fills the chip without splitting the reduction
    big = desc(n=64, c=64, h=56, w=56, k=64, dtype=tvg.TVG_BF16)
    assert tvg.tvg_conv2d_workspace_size(big) == 0
    # 49 pixels at batch 1, and input channels that are no multiple of 8 (so that the generic
    # kernel runs the problem, not the one-launch fp32 kernel): the reduction is partitioned
    small = desc(n=1, c=508, h=7, w=7, k=512)
    need = tvg.tvg_conv2d_workspace_size(small)
    assert need > 0 and need % (512 * 49 * 4) == 0
    assert tvg.tvg_conv2d_fused(small, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, None, 0, 0) == 4
    assert tvg.tvg_conv2d_fused(small, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE,
                                need - 1, 0) == 4
    # the workspace must be 256-byte aligned
    assert tvg.tvg_conv2d_fused(small, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE + 64,
                                need, 0) == 4
    assert tvg.tvg_dwconv2d_workspace_size(desc(k=8, c=8)) == 0


def test_static_scratch_entry_point_validates_on_the_host():
    """tvg_conv2d_fused_static: descriptor, NULL and size errors come back before any device
    call (this machine has no GPU)."""
    assert tvg.tvg_static_scratch_bytes() == 16 << 20
    assert tvg.tvg_conv2d_fused_static(desc(n=0), FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 0) == 2
    assert tvg.tvg_conv2d_fused_static(desc(dtype=5), FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 0) == 3
    assert tvg.tvg_conv2d_fused_static(desc(), FAKE, None, FAKE, FAKE, None, None, FAKE, 0) == 1
    assert tvg.load().tvg_conv2d_fused_static(None, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, None) == 1
    big = desc(n=1, c=516, h=28, w=28, k=512)
    assert tvg.tvg_conv2d_workspace_size(big) > tvg.tvg_static_scratch_bytes()
    assert tvg.tvg_conv2d_fused_static(big, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 0) == 4


def test_prepacked_entry_points_validate_on_the_host():
    """tvg_conv2d_prepack_size / prepack / fused_prepacked: sizes are a pure function of the
    descriptor, everything else is rejected before any device call (this machine has no GPU)."""
    d = desc(n=2, c=128, h=9, w=7, k=64, dtype=tvg.TVG_BF16)
    pb, wb = tvg.tvg_conv2d_prepack_size(d)
    assert pb == 16 * 128 * 64 * 2                         # [16 positions][c][k] fp16
    assert wb == 16 * 128 * (2 * 5 * 4) * 2                # [16 positions][c][2x2 output tiles] fp16
    for kw in (dict(stride_h=2, stride_w=2), dict(c=32), dict(k=96), dict(dtype=tvg.TVG_F32),
               dict(r=1, s=1, pad_h=0, pad_w=0), dict(pad_h=0, pad_w=0), dict(n=8192, h=512, w=512)):
        f = dict(n=2, c=128, h=9, w=7, k=64, dtype=tvg.TVG_BF16)
        f.update(kw)
        with pytest.raises(tvg.TvgError) as e:
            tvg.tvg_conv2d_prepack_size(desc(**f))
        assert e.value.status == 3, kw
        assert tvg.tvg_conv2d_prepack(desc(**f), FAKE, FAKE, 1 << 30, 0) == 3
        assert tvg.tvg_conv2d_fused_prepacked(desc(**f), FAKE, FAKE, FAKE, FAKE, None, None, FAKE,
                                              FAKE * 16, 1 << 40, 0) == 3
    with pytest.raises(tvg.TvgError) as e:
        tvg.tvg_conv2d_prepack_size(desc(n=0, dtype=tvg.TVG_BF16))
    assert e.value.status == 2
    lib = tvg.load()
    assert lib.tvg_conv2d_prepack_size(ctypes.byref(d), None, None) == 1
    A = 0x10000                                             # 256-byte aligned fake pointer
    assert tvg.tvg_conv2d_prepack(d, None, A, pb, 0) == 1
    assert tvg.tvg_conv2d_prepack(d, A, A, pb - 1, 0) == 4
    assert tvg.tvg_conv2d_prepack(d, A, A + 8, pb, 0) == 4
    assert tvg.tvg_conv2d_prepack(d, A + 8, A, pb, 0) == 3          # w must be 16-byte aligned
    assert tvg.tvg_conv2d_fused_prepacked(d, A, A, A, A, None, None, None, A, wb, 0) == 1
    assert tvg.tvg_conv2d_fused_prepacked(d, A, A, A, A, None, None, A, None, 0, 0) == 4
    assert tvg.tvg_conv2d_fused_prepacked(d, A, A, A, A, None, None, A, A, wb - 1, 0) == 4
    assert tvg.tvg_conv2d_fused_prepacked(d, A, A, A, A, None, None, A, A + 128, wb, 0) == 4
    assert tvg.tvg_conv2d_fused_prepacked(d, A, A + 8, A, A, None, None, A, A, wb, 0) == 3


def test_tile_table_sets_overrides_and_forgets():
    """tvg_conv2d_set_tile / tvg_conv2d_get_plan are host-only: the planners' choice, a fixed
    tile, its removal, and what is rejected."""
    c6 = desc(n=64, c=128, h=28, w=28, k=128, dtype=tvg.TVG_BF16, flags=tvg.TVG_RELU)
    assert tvg.tvg_conv2d_get_plan(c6) == (2, 64, 256)               # pipelined 3x3, 64 x 256
    assert tvg.tvg_conv2d_set_tile(c6, 64, 128) == 0
    plain = desc(n=64, c=128, h=28, w=28, k=128, dtype=tvg.TVG_BF16, flags=0)
    assert tvg.tvg_conv2d_get_plan(plain)[1:] == (64, 128)           # flags are not part of the key
    other = desc(n=32, c=128, h=28, w=28, k=128, dtype=tvg.TVG_BF16)
    assert tvg.tvg_conv2d_get_plan(other)[1:] != (64, 128) or tvg.tvg_conv2d_get_plan(other)[0] != 2
    assert tvg.tvg_conv2d_set_tile(c6, 128, 64) == 0                 # replaces the entry
    assert tvg.tvg_conv2d_get_plan(c6)[1:] == (128, 64)
    assert tvg.tvg_conv2d_set_tile(c6, 0, 0) == 0
    assert tvg.tvg_conv2d_get_plan(c6) == (2, 64, 256)
    assert tvg.tvg_conv2d_set_tile(c6, 0, 0) == 0                    # forgetting twice is fine
    # 128 x 256 is the pipelined kernel's channel-split variant: it runs when named with its stages
    assert tvg.tvg_conv2d_set_knobs(c6, (128, 256, 2, 0, 0, 0)) == 0
    assert tvg.tvg_conv2d_get_plan(c6) == (2, 128, 256)
    assert tvg.tvg_conv2d_set_knobs(c6, None) == 0
    for mt, nt in [(64, 100), (256, 64), (256, 256), (-64, 64), (64, 0)]:
        assert tvg.tvg_conv2d_set_tile(c6, mt, nt) == 3
    assert tvg.tvg_conv2d_set_tile(desc(n=0), 64, 64) == 2
    lib = tvg.load()
    assert lib.tvg_conv2d_set_tile(None, 64, 64) == 1
    assert lib.tvg_conv2d_get_plan(ctypes.byref(c6), None, None, None) == 1
    # kernels by problem: stem, 1x1, generic (fp32)
    assert tvg.tvg_conv2d_get_plan(desc(n=64, c=3, h=224, w=224, k=64, r=7, s=7, stride_h=2,
                                        stride_w=2, pad_h=3, pad_w=3, dtype=tvg.TVG_BF16))[0] == 3
    assert tvg.tvg_conv2d_get_plan(desc(n=64, c=128, h=28, w=28, k=256, r=1, s=1, stride_h=2,
                                        stride_w=2, pad_h=0, pad_w=0, dtype=tvg.TVG_BF16)) == (4, 128, 64)
    assert tvg.tvg_conv2d_get_plan(desc(n=1, c=64, h=56, w=56, k=64)) == (5, 32, 32)     # fp32, launch-bound
    # ... with 16 x 16 tiles where 32 x 32 ones are at most 64 and the small ones need no second launch
    assert tvg.tvg_conv2d_get_plan(desc(n=1, c=128, h=28, w=28, k=256, stride_h=2, stride_w=2)) == (5, 16, 16)
    assert tvg.tvg_conv2d_get_plan(desc(n=1, c=256, h=14, w=14, k=256)) == (5, 16, 16)
    assert tvg.tvg_conv2d_get_plan(desc(n=1, c=512, h=7, w=7, k=512)) == (5, 32, 32)     # (split either way)
    assert tvg.tvg_conv2d_get_plan(desc(n=1, c=60, h=56, w=56, k=64))[0] == 0            # channels not 8n
    assert tvg.tvg_conv2d_get_plan(desc(n=64, c=64, h=56, w=56, k=64))[0] == 0           # fills the chip
    assert tvg.tvg_conv2d_get_plan(desc(n=1, c=64, h=56, w=56, k=64, r=5, s=5, pad_h=2, pad_w=2))[0] == 0


def test_block_entry_point_validates_on_the_host():
    """tvg_dwpw_fused / tvg_dwpw_workspace_size / tvg_dwpw_one_kernel: which problems have the
    one-kernel form, the workspace of the two-kernel form, and every error path before a
    device call."""
    small = desc(n=32, c=512, h=14, w=14, k=512, dtype=tvg.TVG_BF16, flags=tvg.TVG_RELU)
    assert tvg.tvg_dwpw_one_kernel(small, 512)
    assert tvg.tvg_dwpw_one_kernel(desc(n=32, c=1024, h=7, w=7, k=1024, dtype=tvg.TVG_BF16), 1024)
    assert tvg.tvg_dwpw_workspace_size(small, 512) == 32 * 512 * 14 * 14 * 2
    wide = desc(n=2, c=32, h=112, w=112, k=32, dtype=tvg.TVG_BF16)
    assert not tvg.tvg_dwpw_one_kernel(wide, 64)                        # rows too long
    assert tvg.tvg_dwpw_workspace_size(wide, 64) == 2 * 32 * 112 * 112 * 2
    s2 = desc(n=2, c=64, h=14, w=14, k=64, stride_h=2, stride_w=2, dtype=tvg.TVG_BF16)
    assert not tvg.tvg_dwpw_one_kernel(s2, 64)
    assert tvg.tvg_dwpw_workspace_size(s2, 64) == 2 * 64 * 7 * 7 * 2         # 12544 = 49 * 256
    f32 = desc(n=1, c=32, h=14, w=14, k=32)
    assert not tvg.tvg_dwpw_one_kernel(f32, 8)
    assert tvg.tvg_dwpw_workspace_size(f32, 8) >= 32 * 14 * 14 * 4
    odd = desc(n=1, c=24, h=14, w=14, k=24, dtype=tvg.TVG_BF16)        # channels not a multiple of 32
    assert not tvg.tvg_dwpw_one_kernel(odd, 8)
    A = 0x10000
    args = [A] * 7 + [None, None, A]        # x w_dw scale_dw shift_dw w_pw scale_pw shift_pw bias res y
    assert tvg.tvg_dwpw_fused(small, 0, 0, *args, stream=0) == 2
    assert tvg.tvg_dwpw_fused(small, 512, 4, *args, stream=0) == 3               # unknown flag
    assert tvg.tvg_dwpw_fused(desc(k=16), 8, 0, *args, stream=0) == 2            # not depthwise
    assert tvg.tvg_dwpw_fused(desc(k=8, c=8, pad_h=0, pad_w=0), 8, 0, *args, stream=0) == 3
    for missing in (0, 1, 2, 3, 4, 5, 6, 9):
        a2 = list(args)
        a2[missing] = None
        assert tvg.tvg_dwpw_fused(small, 512, 0, *a2, stream=0) == 1
    for k in (0, 4, 8, 9):                                             # x, w_pw, residual, y alignment
        a2 = list(args)
        a2[k] = A + 8
        assert tvg.tvg_dwpw_fused(small, 512, 0, *a2, stream=0) == 3
    assert tvg.tvg_dwpw_fused(wide, 64, 0, *args, stream=0) == 4       # no one-kernel form, no workspace
    need = tvg.tvg_dwpw_workspace_size(wide, 64)
    assert tvg.tvg_dwpw_fused(wide, 64, 0, *args, A, need - 1, 0) == 4
    assert tvg.tvg_dwpw_fused(wide, 64, 0, *args, A + 64, need, 0) == 4
    assert tvg.tvg_dwpw_fused(small, 512, 0, *args, A, 16, 0) == 4     # a workspace, but too small
    with pytest.raises(tvg.TvgError):
        tvg.tvg_dwpw_workspace_size(desc(k=16), 8)
    with pytest.raises(tvg.TvgError):
        tvg.tvg_dwpw_one_kernel(desc(k=16), 8)
    lib = tvg.load()
    assert lib.tvg_dwpw_workspace_size(ctypes.byref(small), 8, None) == 1
    assert lib.tvg_dwpw_one_kernel(ctypes.byref(small), 8, None) == 1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_1802_04799_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", str(tmp_path / "libtvg.so"))
    with pytest.raises(ImportError):
        b.load()


def test_knob_table_host_side():
    """tvg_conv2d_set_knobs / tvg_conv2d_get_knobs (host only): what the library's rule picks, what
    a caller can fix, how the size query follows the reduction split, what is rejected."""
    c6 = desc(n=64, c=128, h=28, w=28, k=128, dtype=tvg.TVG_BF16)
    assert tvg.tvg_conv2d_get_knobs(c6) == (64, 256, 2, 1, 2, 0)        # pipelined, padded pitch
    assert tvg.tvg_conv2d_set_knobs(c6, (64, 128, 1, 0, 0, 0)) == 0
    assert tvg.tvg_conv2d_get_plan(c6) == (1, 64, 128)                 # the single-stage kernel
    assert tvg.tvg_conv2d_get_knobs(c6) == (64, 128, 1, 0, 0, 0)
    assert tvg.tvg_conv2d_set_tile(c6, 64, 64) == 0                    # the tile alone: stages stay
    assert tvg.tvg_conv2d_get_knobs(c6)[:3] == (64, 64, 1)
    assert tvg.tvg_conv2d_set_knobs(c6, None) == 0
    assert tvg.tvg_conv2d_get_knobs(c6) == (64, 256, 2, 1, 2, 0)
    # C12 at batch 64: odd 7-pixel rows, 200 tiles: by rule whole-row loads, one wave group, padded pitch
    c12 = desc(n=64, c=512, h=7, w=7, k=512, dtype=tvg.TVG_BF16)
    assert tvg.tvg_conv2d_get_knobs(c12) == (64, 128, 2, 1, 2, 2)
    assert tvg.tvg_conv2d_set_knobs(c12, (0, 0, 2, 0, 0, 1)) == 0       # element loads: two wave groups
    assert tvg.tvg_conv2d_get_knobs(c12)[2:] == (2, 2, 2, 1)
    assert tvg.tvg_conv2d_set_knobs(c12, None) == 0
    # C9 at batch 64: a lone workgroup per CU keeps the padded pitch (86 KB of LDS), one group
    c9 = desc(n=64, c=256, h=14, w=14, k=256, dtype=tvg.TVG_BF16)
    assert tvg.tvg_conv2d_get_knobs(c9) == (64, 256, 2, 1, 2, 0)
    # the generic kernel: the size query follows the split
    f = desc(n=1, c=508, h=7, w=7, k=512)
    auto = tvg.tvg_conv2d_workspace_size(f)
    k0 = tvg.tvg_conv2d_get_knobs(f)
    assert k0[2:] == (2, 32, 0, 0) and auto == 32 * 512 * 49 * 4
    assert tvg.tvg_conv2d_set_knobs(f, (0, 0, 0, 4, 0, 0)) == 0
    assert tvg.tvg_conv2d_workspace_size(f) == 4 * 512 * 49 * 4 and tvg.tvg_conv2d_get_knobs(f)[3] == 4
    assert tvg.tvg_conv2d_set_knobs(f, (0, 0, 0, 1, 0, 0)) == 0
    assert tvg.tvg_conv2d_workspace_size(f) == 0
    assert tvg.tvg_conv2d_set_knobs(f, None) == 0
    assert tvg.tvg_conv2d_workspace_size(f) == auto
    # the one-launch fp32 kernel: its waves split the reduction; a caller who fixes the generic
    # kernel's knobs gets the generic kernel
    g = desc(n=1, c=512, h=7, w=7, k=512)
    # (8 waves per workgroup x 8 slices across workgroups, the slices' sums in the workspace)
    assert tvg.tvg_conv2d_get_plan(g)[0] == 5 and tvg.tvg_conv2d_get_knobs(g) == (0, 0, 1, 64, 0, 0)
    assert tvg.tvg_conv2d_workspace_size(g) == 8 * 512 * 49 * 4
    c2 = desc(n=1, c=64, h=56, w=56, k=64)           # one pass: one launch, no workspace
    assert tvg.tvg_conv2d_get_knobs(c2) == (0, 0, 1, 8, 0, 0) and tvg.tvg_conv2d_workspace_size(c2) == 0
    assert tvg.tvg_conv2d_set_knobs(g, (0, 0, 0, 4, 0, 0)) == 0
    assert tvg.tvg_conv2d_get_plan(g)[0] == 0 and tvg.tvg_conv2d_workspace_size(g) == 4 * 512 * 49 * 4
    assert tvg.tvg_conv2d_set_knobs(g, None) == 0
    for bad in [(64, 100, 0, 0, 0, 0), (0, 0, 3, 0, 0, 0), (0, 0, 0, 33, 0, 0), (0, 0, 0, -1, 0, 0),
                (0, 0, 0, 0, 3, 0), (0, 0, 0, 0, 0, 3)]:
        assert tvg.tvg_conv2d_set_knobs(c6, bad) == 3
    assert tvg.tvg_conv2d_set_knobs(desc(n=0), (0, 0, 1, 0, 0, 0)) == 2
    lib = tvg.load()
    assert lib.tvg_conv2d_set_knobs(None, None) == 1
    assert lib.tvg_conv2d_get_knobs(ctypes.byref(c6), None) == 1
