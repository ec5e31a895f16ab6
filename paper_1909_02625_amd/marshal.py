"""Argument marshalling between numpy workloads and the library: numpy NCHW fp32/fp64 <-> torch device
tensors in NHWC, and construction of library blocks from one workload config.  Used by the benchmark,
the command-line tools and the tests.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from workloads import flatten_params
from workloads.configs import block_output_shape

from . import binding as D


def torch_dtype(dtype):
    return torch.bfloat16 if dtype == D.DSP_BF16 else torch.float32


def to_dev(a, dtype, feature_map=True):
    """numpy NCHW (or N x C) -> contiguous NHWC device tensor in the block storage type."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if t.dim() == 4:
        t = t.permute(0, 2, 3, 1).contiguous()
    td = torch_dtype(dtype) if (feature_map and t.dim() == 4) else torch.float32
    return t.to(device="cuda", dtype=td).contiguous()


def from_dev(t, shape):
    """device NHWC tensor (flat or shaped) -> numpy fp64 in NCHW ``shape`` (or N x C)."""
    h = t.detach().to(torch.float32).cpu().numpy().astype(np.float64)
    if len(shape) == 4:
        n, c, hh, ww = shape
        return h.reshape(n, hh, ww, c).transpose(0, 3, 1, 2).copy()
    return h.reshape(shape)


def round_like(a, dtype):
    """What the storage type keeps of fp32 values (bf16 round-to-nearest-even), as fp32 numpy."""
    if dtype == D.DSP_BF16:
        return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch.bfloat16).to(torch.float32).numpy()
    return np.asarray(a, np.float32)


def block_shapes(cfg):
    """Input shape of every block and the final output shape."""
    shapes = [tuple(cfg["input"])]
    for layers in cfg["blocks"]:
        shapes.append(tuple(block_output_shape(layers, shapes[-1])))
    return shapes


def build_gpu_blocks(cfg, params, dtype, p=None, m=None, standalone=False, spare=0):
    """One library block per config block; rings sized for DSP(p; m) (p_prev = 0 when stand-alone) plus
    ``spare`` entries of slack in every queue between two blocks."""
    p = list(cfg["p"] if p is None else p)
    m = list(cfg["m"] if m is None else m)
    K = len(cfg["blocks"])
    shapes = block_shapes(cfg)
    blocks = []
    for k, layers in enumerate(cfg["blocks"]):
        first = k == 0 and cfg.get("data_input", True)
        desc, keep = D.make_block_desc(layers, shapes[k], dtype, k, K, m[k],
                                       p_prev=0 if (standalone or k == 0) else p[k - 1] + spare,
                                       needs_input_grad=not first)
        blocks.append(D.dsp_block_init(desc, flatten_params(layers, params[k])))
        del keep
    return blocks


def destroy_blocks(blocks):
    for b in blocks:
        D.dsp_block_destroy(b)
