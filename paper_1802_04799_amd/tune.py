"""Measured search over a problem's schedule knobs (TVM paper, Section 5: Section 5.1's schedule
space is a template with knobs per operator, Section 5.3 explores it by running candidates on
the device, with simulated annealing walking the space).  Here the knobs are the compiled kernel
instances and launch parameters behind ``tvg_conv2d_set_knobs`` - workgroup tile (and with it the
wave tile), LDS stages, split of the reduction, LDS pitch, row-load strategy - and every
candidate is timed on the device; there is no cost model.

    from paper_1802_04799_amd import tune
    report = tune.tune_conv2d(desc, x, w, scale, shift, y)      # walks, then fixes the best point
    tune.save(path)  /  tune.load(path)                          # keep the choices across runs

The walk: start at the library's own plan; a move changes one knob to another of its values; a
faster point is always accepted, a slower one with probability exp(-(t_new - t_cur) / (T * t_cur))
with T falling geometrically; after ``restart_after`` moves without a new best the walk jumps to a
random point (random restart).  Points whose knobs the problem's kernel cannot use (the library
would fall back to another kernel) are skipped, and every measured point is remembered, so the
walk never times a point twice.  Small spaces are simply covered completely.

Timing uses HIP events around back-to-back launches on torch's current stream; the library's own
plan is always the first point, so a tuned problem is never slower than an untuned one by more than
the noise of the measurement.
"""
import itertools
import json
import math
import random
import zlib
from typing import Dict, List, Optional, Tuple

from . import binding as _b

TILES: List[Tuple[int, int]] = [(64, 256), (128, 128), (64, 128), (128, 64), (64, 64)]
# the pipelined 3x3 kernel also has 128 x 256 (its channel-split variant: two wave groups share a patch),
# the single-stage one 64 x 512 (stride 1, rows of 8n pixels)
TILES_3X3: List[Tuple[int, int]] = TILES + [(128, 256), (64, 512)]
KNOBS = ("mt", "nt", "stages", "split_k", "lds_pitch", "row_loads")
_chosen: Dict[str, Tuple[int, ...]] = {}


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


def space_for(desc, kernel: int) -> Dict[str, list]:
    """The values each knob can take for this problem's kernel family (0 = the library's rule is
    not a value of its own: every point of the space names all its knobs)."""
    if kernel in (1, 2):                         # bf16 3x3: both kernels, all their knobs
        s1 = desc.stride_w == 1
        odd_small = desc.w % 2 == 1 and desc.w <= 7 and s1
        return {"tile": TILES_3X3, "stages": [1, 2], "split_k": [1, 2] if s1 else [1],
                "lds_pitch": [1, 2] if s1 else [0], "row_loads": [1, 2] if odd_small else [0]}
    if kernel in (4, 6):                         # bf16 1x1: its tiles, or the deep-reduction kernel
        deep = desc.stride_w == 1 and desc.c % 128 == 0 and (desc.h * desc.w) % 4 == 0
        return {"tile": TILES[1:], "stages": [1, 2] if deep else [1], "split_k": [0], "lds_pitch": [0],
                "row_loads": [0]}
    if kernel == 0:                              # generic kernel: tile rows and the reduction split
        return {"tile": [(64, 0), (128, 0)], "stages": [0],
                "split_k": [1, 2, 3, 4, 6, 8, 12, 16, 24, 32], "lds_pitch": [0], "row_loads": [0]}
    return {"tile": [(0, 0)], "stages": [0], "split_k": [0], "lds_pitch": [0], "row_loads": [0]}


def _point(tile, stages, split_k, lds_pitch, row_loads) -> Tuple[int, ...]:
    return (tile[0], tile[1], stages, split_k, lds_pitch, row_loads)


def _normalise(p: Tuple[int, ...]) -> Tuple[int, ...]:
    """Knobs that only the pipelined kernel has are dropped from a single-stage point, so that
    equivalent points share one measurement."""
    mt, nt, stages, split_k, pitch, rows = p
    if stages == 1:
        return (mt, nt, 1, 0, 0, 0)
    return p


def tune_conv2d(desc, x, w, scale, shift, y, bias=None, residual=None, workspace=None,
                iters: int = 30, repeats: int = 3, min_gain: float = 0.03, max_trials: int = 40,
                seed: int = 0, t0: float = 0.05, cooling: float = 0.85, restart_after: int = 8) -> dict:
    """Walks the knob space of this problem by measurement, fixes the fastest point with
    tvg_conv2d_set_knobs when it beats the library's plan by more than `min_gain` (a fraction),
    and returns what it measured: the walk (trials, accepted moves, restarts), every point's
    time, the choice.  y (and a workspace, allocated here as needed) are scratch."""
    import torch
    rng = random.Random(seed ^ zlib.crc32(_key(desc).encode()))
    _b.tvg_conv2d_set_knobs(desc, None)
    kernel, mt0, nt0 = _b.tvg_conv2d_get_plan(desc)
    ws = {"t": workspace}

    def call():
        need = ws["need"]
        st = _b.tvg_conv2d_fused(desc, x, w, scale, shift, bias, residual, y, ws["t"], need, None)
        if st != _b.TVG_OK:
            raise _b.TvgError(st, "tvg_conv2d_fused")

    def measure() -> float:
        ws["need"] = need = _b.tvg_conv2d_workspace_size(desc)
        if need and (ws["t"] is None or ws["t"].numel() * ws["t"].element_size() < need):
            ws["t"] = torch.empty(need, dtype=torch.uint8, device=x.device)
        return _time_us(call, iters, repeats)

    default_knobs = _b.tvg_conv2d_get_knobs(desc)
    base = measure()
    report = {"key": _key(desc), "kernel": _b.KERNEL_NAMES[kernel], "default": [mt0, nt0],
              "default_knobs": list(default_knobs), "default_us": round(base, 2), "candidates": {}}
    space = space_for(desc, kernel)
    axes = ["tile", "stages", "split_k", "lds_pitch", "row_loads"]
    seen: Dict[Tuple[int, ...], Optional[float]] = {}

    def evaluate(p: Tuple[int, ...]) -> Optional[float]:
        p = _normalise(p)
        if p in seen:
            return seen[p]
        us = None
        if _b.tvg_conv2d_set_knobs(desc, p) == _b.TVG_OK:
            eff = _b.tvg_conv2d_get_knobs(desc)
            k2 = _b.tvg_conv2d_get_plan(desc)[0]
            # usable if the library really runs what the point names (no silent fall-back)
            same_family = (k2 in (1, 2)) if kernel in (1, 2) else (k2 in (4, 6)) if kernel in (4, 6) else k2 == kernel
            named = all(want == 0 or want == got for want, got in zip(p, eff))
            if same_family and named:
                us = measure()
                report["candidates"]["/".join(map(str, p))] = round(us, 2)
        seen[p] = us
        return us

    all_points = [_point(*c) for c in itertools.product(*[space[a] for a in axes])]
    walk = {"space_points": len({_normalise(p) for p in all_points}), "trials": 0, "accepted": 0,
            "restarts": 0, "exhaustive": False}
    best_p, best_us = None, base
    if len(all_points) <= 1:
        pass
    elif walk["space_points"] <= max_trials:      # small space: cover it
        walk["exhaustive"] = True
        for p in all_points:
            us = evaluate(p)
            if us is not None and us < best_us:
                best_p, best_us = _normalise(p), us
        walk["trials"] = sum(v is not None for v in seen.values())
    else:                                          # simulated annealing with random restarts
        d = tuple(default_knobs)
        cur = [(d[0], d[1]), d[2], d[3], d[4], d[5]]
        # snap the library's plan onto the space (a knob it does not use takes the first value)
        for i, a in enumerate(axes):
            if cur[i] not in space[a]:
                cur[i] = space[a][0]
        cur_us = evaluate(_point(*cur)) or base
        temp, stale = t0, 0
        while walk["trials"] < max_trials:
            if stale >= restart_after:
                cand = [rng.choice(space[a]) for a in axes]
                walk["restarts"] += 1
                stale = 0
            else:
                cand = list(cur)
                movable = [i for i, a in enumerate(axes) if len(space[a]) > 1]
                i = rng.choice(movable)
                cand[i] = rng.choice([v for v in space[axes[i]] if v != cur[i]])
            fresh = _normalise(_point(*cand)) not in seen
            us = evaluate(_point(*cand))
            if fresh:
                walk["trials"] += 1
            elif all(_normalise(p) in seen for p in all_points):
                break                               # everything has been measured
            if us is None:
                stale += 1
                continue
            if us < cur_us or rng.random() < math.exp(-(us - cur_us) / (temp * cur_us)):
                cur, cur_us = cand, us
                walk["accepted"] += 1
            if us < best_us:
                best_p, best_us, stale = _normalise(_point(*cand)), us, 0
            else:
                stale += 1
            temp *= cooling
    report["walk"] = walk
    _b.tvg_conv2d_set_knobs(desc, None)
    if best_p is not None and best_us < base * (1.0 - min_gain):
        _b.tvg_conv2d_set_knobs(desc, best_p)
        _chosen[report["key"]] = tuple(best_p)
        report["chosen"] = list(best_p[:2])
        report["chosen_knobs"] = list(best_p)
    else:
        _chosen.pop(report["key"], None)
        report["chosen"] = None                  # the library's rule stands
        report["chosen_knobs"] = None
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
    for key, knobs in table.items():
        v = [int(t) for t in key.split(",")]
        desc = _b.ConvDesc(*v[:12], 0)
        knobs = tuple(knobs) + (0,) * (6 - len(knobs))      # older files hold (mt, nt) only
        if _b.tvg_conv2d_set_knobs(desc, knobs) == _b.TVG_OK:
            _chosen[key] = knobs
            n += 1
    return n
