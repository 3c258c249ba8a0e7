"""Shared helpers of the GPU parity tests (no arithmetic of the method itself)."""
import numpy as np

TOL = {"f32": 1e-4, "bf16": 2e-2}


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
