"""Helpers of the GPU parity tests: the package's marshalling functions plus the error norm the tests use."""
from __future__ import annotations

import numpy as np

from paper_1909_02625_amd.marshal import (block_shapes, build_gpu_blocks, destroy_blocks, from_dev, round_like,  # noqa: F401
                                          to_dev, torch_dtype)


def rel_err(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    nb = np.linalg.norm(b.ravel())
    return float(np.linalg.norm((a - b).ravel()) / (nb if nb > 0 else 1.0))
