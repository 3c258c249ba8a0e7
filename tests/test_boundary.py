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
            "tvg_version"} <= names
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
    (dict(stride_h=1, stride_w=2), 3),
])
def test_depthwise_rejects_what_it_does_not_build(kw, status):
    d = desc(**kw)
    assert tvg.tvg_dwconv2d_fused(d, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, None, 0, 0) == status
    with pytest.raises(tvg.TvgError):
        tvg.tvg_dwconv2d_workspace_size(d)


def test_workspace_query_and_too_small_workspace():
    # a large-batch problem fills the chip without splitting the reduction
    big = desc(n=64, c=64, h=56, w=56, k=64, dtype=tvg.TVG_BF16)
    assert tvg.tvg_conv2d_workspace_size(big) == 0
    # the last ResNet-18 shape at batch 1 has 49 pixels: the reduction is partitioned
    small = desc(n=1, c=512, h=7, w=7, k=512)
    need = tvg.tvg_conv2d_workspace_size(small)
    assert need > 0 and need % (512 * 49 * 4) == 0
    assert tvg.tvg_conv2d_fused(small, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, None, 0, 0) == 4
    assert tvg.tvg_conv2d_fused(small, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE,
                                need - 1, 0) == 4
    # the workspace must be 256-byte aligned
    assert tvg.tvg_conv2d_fused(small, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE + 64,
                                need, 0) == 4
    assert tvg.tvg_dwconv2d_workspace_size(desc(k=8, c=8)) == 0


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_1802_04799_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", str(tmp_path / "libtvg.so"))
    with pytest.raises(ImportError):
        b.load()
