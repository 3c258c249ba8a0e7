"""Measured choice of a kernel's tile shape for one problem (TVM paper, Section 5: schedules
are chosen per operator shape by running candidates on the device; here the space is the handful
of tile shapes the kernels are built with, so the search is exhaustive and needs no cost model).

    from paper_1802_04799_amd import tune
    report = tune.tune_conv2d(desc, x, w, scale, shift, y)      # times, then fixes the best tile
    tune.save(path)  /  tune.load(path)                          # keep the choices across runs

Timing uses HIP events around back-to-back launches on torch's current stream; the library's own
rule is always one of the candidates, so a tuned problem is never slower than an untuned one by
more than the noise of the measurement.
"""
import json
from typing import Dict, List, Optional, Tuple

from . import binding as _b

TILES: List[Tuple[int, int]] = [(64, 256), (128, 128), (64, 128), (128, 64), (64, 64)]
_chosen: Dict[str, Tuple[int, int]] = {}


def _key(desc) -> str:
    return ",".join(str(int(getattr(desc, f))) for f in
                    ("n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w", "pad_h", "pad_w", "dtype"))


def _time_us(call, iters: int, repeats: int) -> float:
    import torch
    best = float("inf")
    for _ in range(repeats):
        for _ in range(3):
            call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            call()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) * 1e3 / iters)
    return best


def tune_conv2d(desc, x, w, scale, shift, y, bias=None, residual=None, workspace=None,
                iters: int = 30, repeats: int = 3, min_gain: float = 0.03) -> dict:
    """Times the library's own plan and every tile shape on this problem, fixes the fastest with
    tvg_conv2d_set_tile when it beats the library's plan by more than `min_gain` (a fraction),
    and returns what it measured.  y (and the workspace, if the problem needs one) are scratch."""
    import torch
    _b.tvg_conv2d_set_tile(desc, 0, 0)
    need = _b.tvg_conv2d_workspace_size(desc)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)

    def call():
        st = _b.tvg_conv2d_fused(desc, x, w, scale, shift, bias, residual, y, workspace, need, None)
        if st != _b.TVG_OK:
            raise _b.TvgError(st, "tvg_conv2d_fused")

    kernel, mt0, nt0 = _b.tvg_conv2d_get_plan(desc)
    base = _time_us(call, iters, repeats)
    report = {"key": _key(desc), "kernel": _b.KERNEL_NAMES[kernel], "default": [mt0, nt0],
              "default_us": round(base, 2), "candidates": {}}
    best, best_us = None, base
    if kernel in (1, 2, 4):                      # the kernels that have a tile knob
        for mt, nt in TILES:
            if _b.tvg_conv2d_set_tile(desc, mt, nt) != _b.TVG_OK:
                continue
            k2, mt2, nt2 = _b.tvg_conv2d_get_plan(desc)
            if k2 == 0 or (mt2, nt2) != (mt, nt):        # this kernel cannot use the tile
                continue
            us = _time_us(call, iters, repeats)
            report["candidates"][f"{mt}x{nt}"] = round(us, 2)
            if us < best_us:
                best, best_us = (mt, nt), us
    _b.tvg_conv2d_set_tile(desc, 0, 0)
    if best is not None and best_us < base * (1.0 - min_gain):
        _b.tvg_conv2d_set_tile(desc, *best)
        _chosen[report["key"]] = best
        report["chosen"] = list(best)
    else:
        _chosen.pop(report["key"], None)
        report["chosen"] = None                  # the library's rule stands
    report["tuned_us"] = round(min(best_us, base), 2)
    return report


def save(path: str) -> None:
    with open(path, "w") as f:
        json.dump({k: list(v) for k, v in sorted(_chosen.items())}, f, indent=1)


def load(path: str) -> int:
    """Re-applies saved choices; returns how many were set."""
    with open(path) as f:
        table = json.load(f)
    n = 0
    for key, (mt, nt) in table.items():
        v = [int(t) for t in key.split(",")]
        desc = _b.ConvDesc(*v[:12], 0)
        if _b.tvg_conv2d_set_tile(desc, mt, nt) == _b.TVG_OK:
            _chosen[key] = (mt, nt)
            n += 1
    return n
