"""Helpers of the GPU parity tests: the package's marshalling functions plus the error norm the tests use."""
from __future__ import annotations

import numpy as np

from paper_1909_02625_amd.marshal import (block_shapes, build_gpu_blocks, destroy_blocks, from_dev, round_like,  # noqa: F401
                                          to_dev, torch_dtype)


def rel_err(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    nb = np.linalg.norm(b.ravel())
    return float(np.linalg.norm((a - b).ravel()) / (nb if nb > 0 else 1.0))


def dgrad_filter_copy(w, stride, pad, groups=1):
    """The filter copy dsp_conv_backward_data reads, from w[cout][cin / groups][r][s]: the flipped filter
    wf[cin][R-1-r][S-1-s][cout / groups] (row g cin/groups + ci holds the output channels of group g); for stride 2
    stored class by class of the input-pixel parity (hi % 2, wi % 2), class (ph, pw) keeping the taps r' = r0,
    r0 + 2, ... and s' = s0, s0 + 2, ... with r0 = (R-1-pad - ph) mod 2."""
    co = w.shape[0] // groups
    wf = np.concatenate([np.ascontiguousarray(w[g * co:(g + 1) * co, :, ::-1, ::-1].transpose(1, 2, 3, 0))
                         for g in range(groups)], axis=0)
    if stride == 1:
        return wf.ravel()
    R, S = w.shape[2], w.shape[3]
    parts = []
    for ph in range(2):
        for pw in range(2):
            r0, s0 = (R - 1 - pad - ph) % 2, (S - 1 - pad - pw) % 2
            parts.append(np.ascontiguousarray(wf[:, r0::2, s0::2, :]).ravel())
    return np.concatenate(parts)


def _raw_to_nchw(raw, shape, bf16):
    """Bytes of an NHWC device tensor (storage type) -> numpy fp32 in NCHW."""
    if bf16:
        vals = (raw.view(np.uint16).astype(np.uint32) << 16).view(np.float32)
    else:
        vals = raw.view(np.float32)
    n, c, h, w = shape
    return vals.reshape(n, h, w, c).transpose(0, 3, 1, 2)


def gpu_decisions(D, O, block, layers, in_shape, dtype, h_in, layer_params, eps=1e-5, band=1e-4):
    """The branch decisions the library's backward sweep of ``block`` was taken on, in the oracle's terms:
    {layer: boolean mask (output > 0)} for every batch norm with ReLU, {layer: source pixel h * W + w} for every
    max pool; plus {layer: stored output as fp32 NCHW} for the ReLU layers (for layer-wise forward checks).

    Every decision is validated against the layer's definition applied (by the oracle, in fp64) to the library's OWN
    stored inputs of that layer: a pooling choice must be the first maximum of the stored window bit for bit, and a
    rectifier mask may differ from sign(z) only where |z| is below ``band`` times the magnitude of the terms z is
    summed from (the library forms z in fp32; rounding the result to the storage type keeps its sign).  Returns
    (decisions, activations, number of such near-ties, largest relative margin among them)."""
    from workloads import infer_shapes
    shapes = infer_shapes(layers, in_shape)
    bf16 = dtype == D.DSP_BF16
    cache = {}

    def stored(i):  # the library's stored tensor i (block input for -1), fp32 NCHW
        if i == -1:
            return np.asarray(h_in, np.float32)
        if i not in cache:
            raw = D.dsp_block_get_activation(block, i, int(np.prod(shapes[i])) * (2 if bf16 else 4))
            cache[i] = _raw_to_nchw(raw, shapes[i], bf16)
        return cache[i]

    dec, acts, near_ties, worst = {}, {}, 0, 0.0
    for i, (L, s) in enumerate(zip(layers, shapes)):
        if L["op"] == "bn" and L["relu"]:
            acts[i] = stored(i)
            dec[i] = acts[i] > 0
            x = stored(L["in"]).astype(np.float64)
            gamma, beta = layer_params[i]["gamma"], layer_params[i]["beta"]
            z, mean, invstd = O.bn_forward(x, gamma, beta, eps)
            cs = (1, -1, 1, 1)
            mag = np.abs(gamma * invstd).reshape(cs) * (np.abs(x) + np.abs(mean).reshape(cs)) + np.abs(beta).reshape(cs)
            if L["res"] is not None:
                r = stored(L["res"]).astype(np.float64)
                z, mag = z + r, mag + np.abs(r)
            flips = dec[i] != (z > 0)
            if flips.any():
                near_ties += int(flips.sum())
                m = float((np.abs(z[flips]) / (mag[flips] + 1e-300)).max())
                worst = max(worst, m)
                assert m < band, ("layer %d: a rectifier mask contradicts the layer's own stored input" % i, int(flips.sum()), m)
        elif L["op"] == "maxpool":
            n, c, ho, wo = s
            a = D.dsp_block_get_pool_argmax(block, i, n * c * ho * wo).reshape(n, ho, wo, c).transpose(0, 3, 1, 2).astype(np.int64)
            w_in = (in_shape if L["in"] == -1 else shapes[L["in"]])[3]
            k, st, pd = L["k"], L["stride"], L["pad"]
            hh = np.arange(ho).reshape(1, 1, ho, 1) * st + a // k - pd
            ww = np.arange(wo).reshape(1, 1, 1, wo) * st + a % k - pd
            dec[i] = hh * w_in + ww
            _, arg = O.maxpool_forward(stored(L["in"]).astype(np.float64), k, st, pd)
            assert np.array_equal(dec[i], arg), "layer %d: a pooling choice is not the first maximum of the stored window" % i
    return dec, acts, near_ties, worst
