"""Oracle run of a chained network (the ResNet-18 and MobileNet convolutional bodies).

TEST INFRASTRUCTURE ONLY.  Each layer is evaluated by the fp64 oracle from the
previous layers' stored outputs.  Because the workload stores every activation
as bfloat16, each layer's fp64 result is rounded to the nearest bf16 (ties to
even) before the next layer reads it: the rounding is part of what the
workload computes, not an approximation of the oracle.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional

import numpy as np

from . import conv2d_fused, dwconv2d_fused, maxpool2d, round_to_bf16


def run_steps(steps, images: np.ndarray, weights: Dict[int, dict], store_bf16: bool = True,
              on_step: Optional[Callable] = None) -> Dict[int, np.ndarray]:
    """Run ``steps`` (objects with op/src/dst/shape/residual/relu/layer_index).

    ``weights[layer_index]`` holds ``w``, ``scale``, ``shift`` for each conv.
    Returns every tensor by id as float32 arrays of stored values.
    """
    tensors: Dict[int, np.ndarray] = {0: np.ascontiguousarray(images, dtype=np.float32)}
    for st in steps:
        src = tensors[st.src]
        if st.op == "conv":
            p = weights[st.layer_index]
            sh = st.shape
            res = None if st.residual is None else tensors[st.residual]
            y64 = conv2d_fused(src, p["w"], p["scale"], p["shift"], None, res,
                               stride=(sh.stride, sh.stride), pad=(sh.pad, sh.pad), relu=st.relu)
        elif st.op == "dwconv":
            p = weights[st.layer_index]
            sh = st.shape
            y64 = dwconv2d_fused(src, p["w"], p["scale"], p["shift"], None, None,
                                 stride=(sh.stride, sh.stride), pad=(sh.pad, sh.pad), relu=st.relu)
        elif st.op == "conv_dual":
            # two convolutions of the same input recorded as one launch: by definition the two
            # operators evaluated separately (the 1x1 one with no padding), each stored on its own
            p2, s2 = weights[st.layer_index2], st.shape2
            y2 = conv2d_fused(src, p2["w"], p2["scale"], p2["shift"], None, None,
                              stride=(s2.stride, s2.stride), pad=(s2.pad, s2.pad), relu=st.relu2)
            tensors[st.dst2] = round_to_bf16(y2) if store_bf16 else y2.astype(np.float32)
            if on_step is not None:
                on_step(st, y2)
            p, sh = weights[st.layer_index], st.shape
            y64 = conv2d_fused(src, p["w"], p["scale"], p["shift"], None, None,
                               stride=(sh.stride, sh.stride), pad=(sh.pad, sh.pad), relu=st.relu)
        elif st.op == "maxpool":
            y64 = maxpool2d(src, k=3, stride=2, pad=1)
        else:
            raise ValueError(st.op)
        tensors[st.dst] = round_to_bf16(y64) if store_bf16 else y64.astype(np.float32)
        if on_step is not None:
            on_step(st, y64)
    return tensors
