"""Shared helpers of the GPU parity tests (no arithmetic of the method itself)."""
import contextlib

import numpy as np

TOL = {"f32": 1e-4, "bf16": 2e-2}          # the stated tolerances (max relative error)
# What the arithmetic of ONE fused operator allows: bf16 outputs are the fp32 result rounded
# once to 8 significant bits (at most 2^-8 = 3.9e-3 relative) plus fp32 accumulation (about
# 1e-6 of rho); a dropped tap or channel of a K = 4608 reduction (1.5 % rms) lands far outside.
# fp32 outputs carry the accumulation error only.
TIGHT = {"f32": 5e-5, "bf16": 5e-3}
# The MobileNet block rounds twice (the depthwise result to the storage type, then y): where the
# fp32 and fp64 depthwise sums straddle a rounding boundary the intermediate differs by one ulp,
# which with a single channel reaches y undiminished: 2 * 2^-8 = 7.8e-3 at worst.
BLOCK_TIGHT = 1e-2


def rel_err(got, want):
    """max_i |g_i - r_i| / max(|r_i|, rho), rho = RMS of the oracle's tensor.

    A pure element-wise ratio is unbounded wherever the exact result is 0 (after
    ReLU) or a cancelling sum, so the denominator is floored at the tensor's RMS.
    An all-zero reference falls back to an absolute bound.
    """
    g = np.asarray(got, dtype=np.float64).reshape(-1)
    r = np.asarray(want, dtype=np.float64).reshape(-1)
    assert g.shape == r.shape
    assert np.all(np.isfinite(g)), "non-finite values in the GPU output"
    rho = float(np.sqrt(np.mean(r * r))) if r.size else 0.0
    if rho == 0.0:
        return float(np.max(np.abs(g - r), initial=0.0)) / 1e-6 * 1e-4
    return float(np.max(np.abs(g - r) / np.maximum(np.abs(r), rho), initial=0.0))


def check(got, want, dtype, what=None, tight=None):
    """The parity gate of a single fused operator: the stated tolerance, and next to it the
    tight bound the arithmetic gives (TIGHT, or `tight` for an operator with its own bound)."""
    err = rel_err(got, want)
    assert err <= TOL[dtype], (what, err)
    assert err <= (TIGHT[dtype] if tight is None else tight), (what, err, "tight bound")
    return err


@contextlib.contextmanager
def fixed_tile(tvg, sh, dtype, tile):
    """Plan the dense problem `sh` with the workgroup tile "mt,nt" (through tvg_conv2d_set_tile)
    for the duration of the block; "" leaves the library's own choice."""
    if not tile:
        yield
        return
    mt, nt = (int(v) for v in tile.split(","))
    desc = tvg.ConvDesc(sh.n, sh.ic, sh.h, sh.w, sh.oc, sh.r, sh.s, sh.stride, sh.stride, sh.pad,
                        sh.pad, tvg.TVG_BF16 if dtype == "bf16" else tvg.TVG_F32, 0)
    assert tvg.tvg_conv2d_set_tile(desc, mt, nt) == 0
    try:
        yield
    finally:
        assert tvg.tvg_conv2d_set_tile(desc, 0, 0) == 0


def to_dev(a, dtype):
    """numpy float32 (bf16-representable for dtype == 'bf16') -> device tensor, exact."""
    import torch
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.cuda()


def to_host(t):
    """device tensor -> float64 numpy (exact widening)."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def dev_inputs(inp, dtype):
    return {"x": to_dev(inp["x"], dtype), "w": to_dev(inp["w"], dtype),
            "scale": to_dev(inp["scale"], "f32"), "shift": to_dev(inp["shift"], "f32"),
            "bias": to_dev(inp.get("bias"), "f32"), "residual": to_dev(inp.get("residual"), dtype)}
