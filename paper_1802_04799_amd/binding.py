"""ctypes binding of libtvg.so.  Names and argument order follow include/tvg.h."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libtvg.so")

TVG_F32, TVG_BF16 = 0, 1
TVG_RELU = 1
TVG_STREAM_OUT = 2      # hint: nothing reads y soon, store it past the caches
TVG_CENTRE_TAP_ONLY = 4  # flags2 of tvg_conv2d_fused_dual: head 2's filters are zero off the centre tap
TVG_OK = 0


class TvgError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class ConvDesc(ctypes.Structure):
    """Mirror of tvg_conv_desc."""
    _fields_ = [("n", ctypes.c_int32), ("c", ctypes.c_int32), ("h", ctypes.c_int32),
                ("w", ctypes.c_int32), ("k", ctypes.c_int32), ("r", ctypes.c_int32),
                ("s", ctypes.c_int32), ("stride_h", ctypes.c_int32), ("stride_w", ctypes.c_int32),
                ("pad_h", ctypes.c_int32), ("pad_w", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("flags", ctypes.c_uint32)]

    @property
    def oh(self) -> int:
        return (self.h + 2 * self.pad_h - self.r) // self.stride_h + 1

    @property
    def ow(self) -> int:
        return (self.w + 2 * self.pad_w - self.s) // self.stride_w + 1


class ConvKnobs(ctypes.Structure):
    """Mirror of tvg_conv_knobs (0 = the library's rule)."""
    _fields_ = [(n, ctypes.c_int32) for n in ("mt", "nt", "stages", "split_k", "lds_pitch", "row_loads")]

    def as_tuple(self):
        return tuple(int(getattr(self, n)) for n, _ in self._fields_)


class TensorLife(ctypes.Structure):
    """Mirror of tvg_tensor_life."""
    _fields_ = [("bytes", ctypes.c_uint64), ("first_step", ctypes.c_int32),
                ("last_step", ctypes.c_int32)]


_lib: Optional[ctypes.CDLL] = None


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Load libtvg.so (built in-tree by ``paper_1802_04799_amd.build``).

    torch is imported first so that the library binds to the HIP runtime torch
    already loaded; device pointers and streams are only valid within one runtime.
    """
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_1802_04799_amd.build` "
                          "(there is no fallback implementation)")
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_LIB_PATH, mode=ctypes.RTLD_GLOBAL)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    dp = ctypes.POINTER(ConvDesc)
    lib.tvg_conv2d_workspace_size.restype = ctypes.c_int
    lib.tvg_conv2d_workspace_size.argtypes = [dp, ctypes.POINTER(sz)]
    lib.tvg_dwconv2d_workspace_size.restype = ctypes.c_int
    lib.tvg_dwconv2d_workspace_size.argtypes = [dp, ctypes.POINTER(sz)]
    for f in (lib.tvg_conv2d_fused, lib.tvg_dwconv2d_fused):
        f.restype = ctypes.c_int
        f.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.tvg_conv2d_fused_dual.restype = ctypes.c_int
    lib.tvg_conv2d_fused_dual.argtypes = [dp, ctypes.c_int32, ctypes.c_uint32] + [vp] * 9
    lib.tvg_conv2d_fused_static.restype = ctypes.c_int
    lib.tvg_conv2d_fused_static.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.tvg_conv2d_prepack_size.restype = ctypes.c_int
    lib.tvg_conv2d_prepack_size.argtypes = [dp, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.tvg_conv2d_prepack.restype = ctypes.c_int
    lib.tvg_conv2d_prepack.argtypes = [dp, vp, vp, sz, vp]
    lib.tvg_conv2d_fused_prepacked.restype = ctypes.c_int
    lib.tvg_conv2d_fused_prepacked.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.tvg_static_scratch_bytes.restype = sz
    lib.tvg_static_scratch_bytes.argtypes = []
    lib.tvg_probe_copy.restype = ctypes.c_int
    lib.tvg_probe_copy.argtypes = [vp, vp, sz, vp]
    lib.tvg_probe_mfma.restype = ctypes.c_int
    lib.tvg_probe_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp,
                                   ctypes.POINTER(ctypes.c_double), vp]
    lib.tvg_dwpw_workspace_size.restype = ctypes.c_int
    lib.tvg_dwpw_workspace_size.argtypes = [dp, ctypes.c_int32, ctypes.POINTER(sz)]
    lib.tvg_dwpw_one_kernel.restype = ctypes.c_int
    lib.tvg_dwpw_one_kernel.argtypes = [dp, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    lib.tvg_dwpw_fused.restype = ctypes.c_int
    lib.tvg_dwpw_fused.argtypes = [dp, ctypes.c_int32, ctypes.c_uint32] + [vp] * 10 + [vp, sz, vp]
    lib.tvg_plan_arena.restype = ctypes.c_int
    lib.tvg_plan_arena.argtypes = [ctypes.POINTER(TensorLife), ctypes.c_int32,
                                   ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint64)]
    lib.tvg_maxpool2d_3x3s2.restype = ctypes.c_int
    lib.tvg_maxpool2d_3x3s2.argtypes = [ctypes.c_int32] * 5 + [vp, vp, vp]
    lib.tvg_status_string.restype = ctypes.c_char_p
    lib.tvg_status_string.argtypes = [ctypes.c_int]
    lib.tvg_version.restype = ctypes.c_int
    lib.tvg_conv2d_set_tile.restype = ctypes.c_int
    lib.tvg_conv2d_set_tile.argtypes = [dp, ctypes.c_int32, ctypes.c_int32]
    lib.tvg_conv2d_set_knobs.restype = ctypes.c_int
    lib.tvg_conv2d_set_knobs.argtypes = [dp, ctypes.POINTER(ConvKnobs)]
    lib.tvg_conv2d_get_knobs.restype = ctypes.c_int
    lib.tvg_conv2d_get_knobs.argtypes = [dp, ctypes.POINTER(ConvKnobs)]
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.tvg_conv2d_get_plan.restype = ctypes.c_int
    lib.tvg_conv2d_get_plan.argtypes = [dp, i32p, i32p, i32p]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().tvg_status_string(int(status)).decode()


def tvg_version() -> int:
    return int(load().tvg_version())


KERNEL_NAMES = {0: "generic", 1: "3x3", 2: "3x3-pipelined", 3: "stem", 4: "1x1", 5: "fp32-small", 6: "1x1-deep"}


def tvg_conv2d_set_tile(desc: "ConvDesc", mt: int, nt: int) -> int:
    """Fix (or, with 0, 0, forget) the tile shape this exact problem is planned with."""
    return int(load().tvg_conv2d_set_tile(ctypes.byref(desc), int(mt), int(nt)))


def tvg_conv2d_set_knobs(desc: "ConvDesc", knobs=None) -> int:
    """Fix the schedule knobs of this exact problem: a ConvKnobs, a 6-tuple
    (mt, nt, stages, split_k, lds_pitch, row_loads), or None to forget the problem."""
    if knobs is None:
        return int(load().tvg_conv2d_set_knobs(ctypes.byref(desc), None))
    if not isinstance(knobs, ConvKnobs):
        knobs = ConvKnobs(*[int(v) for v in knobs])
    return int(load().tvg_conv2d_set_knobs(ctypes.byref(desc), ctypes.byref(knobs)))


def tvg_conv2d_get_knobs(desc: "ConvDesc"):
    """The knobs a call with this descriptor would really use now, as a 6-tuple."""
    k = ConvKnobs()
    st = load().tvg_conv2d_get_knobs(ctypes.byref(desc), ctypes.byref(k))
    if st != TVG_OK:
        raise TvgError(st, "tvg_conv2d_get_knobs")
    return k.as_tuple()


def tvg_conv2d_get_plan(desc: "ConvDesc"):
    """(kernel id, mt, nt) a call with this descriptor would use now."""
    k, mt, nt = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    st = load().tvg_conv2d_get_plan(ctypes.byref(desc), ctypes.byref(k), ctypes.byref(mt), ctypes.byref(nt))
    if st != TVG_OK:
        raise TvgError(st, "tvg_conv2d_get_plan")
    return k.value, mt.value, nt.value


# ---------------------------------------------------------------------------------------
# raw entry points: torch tensors (or None / int addresses) in, status code out
# ---------------------------------------------------------------------------------------

def _addr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def tvg_conv2d_workspace_size(desc: ConvDesc) -> int:
    out = ctypes.c_size_t(0)
    st = load().tvg_conv2d_workspace_size(ctypes.byref(desc), ctypes.byref(out))
    if st != TVG_OK:
        raise TvgError(st, "tvg_conv2d_workspace_size")
    return int(out.value)


def tvg_dwconv2d_workspace_size(desc: ConvDesc) -> int:
    out = ctypes.c_size_t(0)
    st = load().tvg_dwconv2d_workspace_size(ctypes.byref(desc), ctypes.byref(out))
    if st != TVG_OK:
        raise TvgError(st, "tvg_dwconv2d_workspace_size")
    return int(out.value)


def tvg_conv2d_fused(desc, x, w, scale, shift, bias, residual, y, workspace=None,
                     workspace_bytes=0, stream=None) -> int:
    return int(load().tvg_conv2d_fused(ctypes.byref(desc), _addr(x), _addr(w), _addr(scale),
                                       _addr(shift), _addr(bias), _addr(residual), _addr(y),
                                       _addr(workspace), workspace_bytes, _stream(stream)))


def tvg_conv2d_fused_dual(desc, k1, flags2, x, w, scale, shift, bias, residual1, y1, y2, stream=None) -> int:
    """Two fused 3x3 convolutions of the same input in one launch (see include/tvg.h)."""
    return int(load().tvg_conv2d_fused_dual(ctypes.byref(desc), int(k1), int(flags2), _addr(x), _addr(w),
                                            _addr(scale), _addr(shift), _addr(bias), _addr(residual1),
                                            _addr(y1), _addr(y2), _stream(stream)))


def tvg_conv2d_fused_static(desc, x, w, scale, shift, bias, residual, y, stream=None) -> int:
    """tvg_conv2d_fused with the library's own static scratch instead of a workspace."""
    return int(load().tvg_conv2d_fused_static(ctypes.byref(desc), _addr(x), _addr(w), _addr(scale),
                                              _addr(shift), _addr(bias), _addr(residual), _addr(y),
                                              _stream(stream)))


def tvg_conv2d_prepack_size(desc):
    """Returns (packed_bytes, workspace_bytes) of the pre-transformed-weights path; raises on error."""
    pb, wb = ctypes.c_size_t(0), ctypes.c_size_t(0)
    st = load().tvg_conv2d_prepack_size(ctypes.byref(desc), ctypes.byref(pb), ctypes.byref(wb))
    if st != TVG_OK:
        raise TvgError(st, "tvg_conv2d_prepack_size")
    return int(pb.value), int(wb.value)


def tvg_conv2d_prepack(desc, w, packed, packed_bytes, stream=None) -> int:
    return int(load().tvg_conv2d_prepack(ctypes.byref(desc), _addr(w), _addr(packed), int(packed_bytes),
                                         _stream(stream)))


def tvg_conv2d_fused_prepacked(desc, x, packed, scale, shift, bias, residual, y, workspace,
                               workspace_bytes, stream=None) -> int:
    return int(load().tvg_conv2d_fused_prepacked(ctypes.byref(desc), _addr(x), _addr(packed), _addr(scale),
                                                 _addr(shift), _addr(bias), _addr(residual), _addr(y),
                                                 _addr(workspace), int(workspace_bytes), _stream(stream)))


def tvg_static_scratch_bytes() -> int:
    return int(load().tvg_static_scratch_bytes())


def tvg_probe_copy(src, dst, nbytes, stream=None) -> int:
    return int(load().tvg_probe_copy(_addr(src), _addr(dst), int(nbytes), _stream(stream)))


def tvg_probe_mfma(dtype, iters, workgroups, out, stream=None):
    """Launches the matrix-instruction probe; returns (status, flops of the launch)."""
    fl = ctypes.c_double(0.0)
    st = load().tvg_probe_mfma(int(dtype), int(iters), int(workgroups), _addr(out), ctypes.byref(fl),
                               _stream(stream))
    return int(st), float(fl.value)


def tvg_dwconv2d_fused(desc, x, w, scale, shift, bias, residual, y, workspace=None,
                       workspace_bytes=0, stream=None) -> int:
    return int(load().tvg_dwconv2d_fused(ctypes.byref(desc), _addr(x), _addr(w), _addr(scale),
                                         _addr(shift), _addr(bias), _addr(residual), _addr(y),
                                         _addr(workspace), workspace_bytes, _stream(stream)))


def tvg_dwpw_workspace_size(dw_desc: ConvDesc, pw_k: int) -> int:
    out = ctypes.c_size_t(0)
    st = load().tvg_dwpw_workspace_size(ctypes.byref(dw_desc), int(pw_k), ctypes.byref(out))
    if st != TVG_OK:
        raise TvgError(st, "tvg_dwpw_workspace_size")
    return int(out.value)


def tvg_dwpw_one_kernel(dw_desc: ConvDesc, pw_k: int) -> bool:
    out = ctypes.c_int32(0)
    st = load().tvg_dwpw_one_kernel(ctypes.byref(dw_desc), int(pw_k), ctypes.byref(out))
    if st != TVG_OK:
        raise TvgError(st, "tvg_dwpw_one_kernel")
    return bool(out.value)


def tvg_dwpw_fused(dw_desc, pw_k, pw_flags, x, w_dw, scale_dw, shift_dw, w_pw, scale_pw, shift_pw,
                   bias_pw, residual, y, workspace=None, workspace_bytes=0, stream=None) -> int:
    return int(load().tvg_dwpw_fused(ctypes.byref(dw_desc), int(pw_k), int(pw_flags), _addr(x),
                                     _addr(w_dw), _addr(scale_dw), _addr(shift_dw), _addr(w_pw),
                                     _addr(scale_pw), _addr(shift_pw), _addr(bias_pw),
                                     _addr(residual), _addr(y), _addr(workspace), workspace_bytes,
                                     _stream(stream)))


def tvg_plan_arena(lives):
    """lives: sequence of (bytes, first_step, last_step).  Returns (offsets, arena_bytes)."""
    n = len(lives)
    arr = (TensorLife * max(n, 1))(*[TensorLife(int(b), int(f), int(l)) for b, f, l in lives])
    offs = (ctypes.c_uint64 * max(n, 1))()
    total = ctypes.c_uint64(0)
    st = load().tvg_plan_arena(arr, n, offs, ctypes.byref(total))
    if st != TVG_OK:
        raise TvgError(st, "tvg_plan_arena")
    return [int(o) for o in offs[:n]], int(total.value)


def tvg_maxpool2d_3x3s2(n, c, h, w, dtype, x, y, stream=None) -> int:
    return int(load().tvg_maxpool2d_3x3s2(n, c, h, w, dtype, _addr(x), _addr(y), _stream(stream)))


# ---------------------------------------------------------------------------------------
# conveniences: build the descriptor from tensors, allocate y and workspace with torch
# ---------------------------------------------------------------------------------------

def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return TVG_F32
    if t.dtype == torch.bfloat16:
        return TVG_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _check(x, w, scale, shift, bias, residual):
    for name, t in (("x", x), ("w", w), ("scale", scale), ("shift", shift), ("bias", bias),
                    ("residual", residual)):
        if t is None:
            continue
        if not t.is_cuda:
            raise ValueError(f"{name} must be a device tensor")
        if not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous")
    import torch
    for name, t in (("scale", scale), ("shift", shift), ("bias", bias)):
        if t is not None and t.dtype != torch.float32:
            raise TypeError(f"{name} must be float32")
    if w.dtype != x.dtype or (residual is not None and residual.dtype != x.dtype):
        raise TypeError("x, w and residual must share one dtype")


def make_desc(x, w, stride, pad, relu, depthwise=False, stream_out=False) -> ConvDesc:
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    flags = (TVG_RELU if relu else 0) | (TVG_STREAM_OUT if stream_out else 0)
    return ConvDesc(n, c, h, wd, k, r, s, sh, sw, ph, pw, _dtype_code(x), flags)


def conv2d_fused(x, w, scale, shift, bias=None, residual=None, *, stride=1, pad=0, relu=False,
                 out=None, workspace=None, stream=None, stream_out=False):
    """y = tail(conv2d(x, w)); allocates y (and the workspace when needed) with torch."""
    import torch
    _check(x, w, scale, shift, bias, residual)
    desc = make_desc(x, w, stride, pad, relu, stream_out=stream_out)
    if w.shape[1] != x.shape[1]:
        raise ValueError("weight input channels do not match x")
    need = tvg_conv2d_workspace_size(desc)
    if out is None:
        out = torch.empty((desc.n, desc.k, desc.oh, desc.ow), dtype=x.dtype, device=x.device)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = tvg_conv2d_fused(desc, x, w, scale, shift, bias, residual, out, workspace, ws_bytes, stream)
    if st != TVG_OK:
        raise TvgError(st, "tvg_conv2d_fused")
    return out


def dwconv2d_fused(x, w, scale, shift, bias=None, residual=None, *, stride=1, pad=1, relu=False,
                   out=None, stream=None, stream_out=False):
    import torch
    _check(x, w, scale, shift, bias, residual)
    desc = make_desc(x, w, stride, pad, relu, depthwise=True, stream_out=stream_out)
    if out is None:
        out = torch.empty((desc.n, desc.k, desc.oh, desc.ow), dtype=x.dtype, device=x.device)
    st = tvg_dwconv2d_fused(desc, x, w, scale, shift, bias, residual, out, None, 0, stream)
    if st != TVG_OK:
        raise TvgError(st, "tvg_dwconv2d_fused")
    return out


def dwpw_fused(x, w_dw, scale_dw, shift_dw, w_pw, scale_pw, shift_pw, bias_pw=None, residual=None, *,
               stride=1, relu_dw=True, relu_pw=True, out=None, workspace=None, stream=None,
               stream_out=False, one_kernel=False):
    """MobileNet block (depthwise 3x3 + tail, 1x1 conv + tail) through tvg_dwpw_fused;
    allocates y with torch, and the workspace of the two-kernel form unless ``one_kernel``
    asks for the form that needs none."""
    import torch
    _check(x, w_pw, scale_pw, shift_pw, bias_pw, residual)
    _check(x, w_dw, scale_dw, shift_dw, None, None)
    desc = make_desc(x, w_dw, stride, 1, relu_dw, depthwise=True)
    k = w_pw.shape[0]
    if w_pw.shape[1] != x.shape[1] or tuple(w_pw.shape[2:]) != (1, 1):
        raise ValueError("w_pw must be [k][c][1][1]")
    flags = (TVG_RELU if relu_pw else 0) | (TVG_STREAM_OUT if stream_out else 0)
    if out is None:
        out = torch.empty((desc.n, k, desc.oh, desc.ow), dtype=x.dtype, device=x.device)
    if one_kernel:
        workspace = None
    else:
        need = tvg_dwpw_workspace_size(desc, k)
        if workspace is None or workspace.numel() * workspace.element_size() < need:
            workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = tvg_dwpw_fused(desc, k, flags, x, w_dw, scale_dw, shift_dw, w_pw, scale_pw, shift_pw,
                        bias_pw, residual, out, workspace, ws_bytes, stream)
    if st != TVG_OK:
        raise TvgError(st, "tvg_dwpw_fused")
    return out


def maxpool2d_3x3s2(x, out=None, stream=None):
    import torch
    if not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous device tensor")
    n, c, h, w = x.shape
    if out is None:
        out = torch.empty((n, c, (h - 1) // 2 + 1, (w - 1) // 2 + 1), dtype=x.dtype, device=x.device)
    st = tvg_maxpool2d_3x3s2(n, c, h, w, _dtype_code(x), x, out, stream)
    if st != TVG_OK:
        raise TvgError(st, "tvg_maxpool2d_3x3s2")
    return out
