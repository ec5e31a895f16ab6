"""Seeded generators for parameters, mini-batches, labels and incoming error gradients.

Everything is drawn once on the host in fp32 with ``numpy.random.default_rng`` and handed
unchanged to whichever implementation is under test.
"""
from __future__ import annotations

import numpy as np

from .configs import param_shapes


def make_params(layers, rng):
    """Per layer a dict of fp32 arrays: Kaiming-normal weights, gamma=1, beta=0, bias 0."""
    out = []
    for L, shapes in zip(layers, param_shapes(layers)):
        d = {}
        for name, shp in shapes:
            if name == "w":
                fan_in = int(np.prod(shp[1:]))
                d[name] = (rng.standard_normal(shp) * np.sqrt(2.0 / fan_in)).astype(np.float32)
            elif name == "gamma":
                d[name] = np.ones(shp, np.float32)
            else:
                d[name] = np.zeros(shp, np.float32)
        out.append(d)
    return out


def perturb_affine(params, rng, scale=0.25):
    """Moves gamma/beta/bias off their trivial initial values (used by gradient tests)."""
    for d in params:
        for name in d:
            if name != "w":
                d[name] = (d[name] + scale * rng.standard_normal(d[name].shape)).astype(np.float32)
    return params


def perturb_one_ulp(params_per_block, seed):
    """Every parameter of every block moved by one fp32 ulp up or down (random signs): the smallest change of
    the inputs an fp32 program can see.  Used to measure how far two runs of one recursion drift apart."""
    rng = np.random.default_rng(seed)
    out = []
    for block in params_per_block:
        nb = []
        for d in block:
            nd = {}
            for k, v in d.items():
                v = np.asarray(v, np.float32)
                up = rng.random(v.shape) < 0.5
                nd[k] = np.where(up, np.nextafter(v, np.float32(np.inf)), np.nextafter(v, np.float32(-np.inf))).astype(np.float32)
            nb.append(nd)
        out.append(nb)
    return out


def make_batch(rng, shape, classes):
    """One mini-batch: data ~ N(0,1) in NCHW fp32, labels uniform in [0, classes)."""
    x = rng.standard_normal(shape).astype(np.float32)
    y = None if classes is None else rng.integers(0, classes, size=shape[0]).astype(np.int32)
    return x, y


def make_error_gradient(rng, shape, std):
    """An incoming error gradient G_{h_{k+1}} ~ N(0, std^2), NCHW fp32."""
    return (rng.standard_normal(shape) * std).astype(np.float32)


def flatten_params(layers, params):
    """Concatenates parameters in layer order (conv: w[co][ci][r][s]; bn: gamma, beta; linear: W, c)."""
    parts = []
    for shapes, d in zip(param_shapes(layers), params):
        for name, _ in shapes:
            parts.append(np.asarray(d[name]).ravel())
    if not parts:
        return np.zeros(0, np.float32)
    return np.concatenate(parts)


def unflatten_params(layers, flat):
    """Inverse of :func:`flatten_params`."""
    out, pos = [], 0
    flat = np.asarray(flat)
    for shapes in param_shapes(layers):
        d = {}
        for name, shp in shapes:
            n = int(np.prod(shp))
            d[name] = flat[pos:pos + n].reshape(shp).copy()
            pos += n
        out.append(d)
    assert pos == flat.size
    return out
