"""Element-wise parity of the three convolution kernels with the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_1909_02625_amd as D
from oracle import dsp_oracle as O
from tests.gpu_harness import dgrad_filter_copy, from_dev, rel_err, round_like, to_dev

pytestmark = pytest.mark.gpu

# (N, H, W, Cin, Cout, R, S, stride, pad): several tiles, ragged tails, every tile family
SHAPES = [
    (3, 9, 9, 16, 16, 3, 3, 1, 1),      # small-channel tile, M = 243 (ragged)
    (2, 8, 8, 3, 16, 3, 3, 1, 1),       # first conv: Cin = 3 -> element-wise gather path
    (2, 12, 12, 16, 32, 3, 3, 2, 1),    # stride 2, 32-channel tile
    (2, 12, 12, 16, 32, 1, 1, 2, 0),    # projection shortcut
    (5, 7, 7, 64, 64, 3, 3, 1, 1),      # 64-wide tile
    (4, 14, 14, 32, 128, 1, 1, 1, 0),   # 1x1
    (2, 10, 10, 128, 256, 3, 3, 1, 1),  # wide
    (2, 20, 20, 3, 64, 7, 7, 2, 3),     # stem 7x7/2
    (2, 20, 20, 8, 64, 7, 7, 2, 3),     # the same with padded channels: 49 taps on the vector path (two mask words)
    (2, 6, 6, 8, 8, 3, 3, 1, 1),        # channel count below the tile width
    (1, 5, 5, 24, 40, 3, 3, 1, 1),      # channel counts that are no power of two
    (4, 13, 13, 16, 16, 3, 3, 2, 1),    # 16 -> 16 channels, stride 2, several slices with a ragged tail
    (2, 11, 11, 16, 16, 1, 1, 1, 0),    # 16 -> 16 channels, 1x1
    (3, 10, 10, 32, 32, 3, 3, 1, 1),    # 32 -> 32 channels: register-resident filters, two channel groups
    (2, 9, 9, 32, 16, 3, 3, 1, 1),      # 32 -> 16
    (33, 32, 32, 16, 16, 3, 3, 1, 1),   # enough pixel groups that each wave walks several of them
    (3, 11, 9, 16, 24, 3, 3, 2, 1),     # stride 2 on odd map sides: the four parity classes have different sizes
    (2, 12, 12, 32, 64, 1, 1, 2, 0),    # 1x1 stride 2: three of the four classes receive no gradient at all
    (2, 9, 9, 8, 16, 2, 2, 2, 0),       # 2x2 stride 2 without padding: one tap per class
    (2, 14, 14, 8, 8, 5, 5, 2, 2),      # 5x5 stride 2: classes of 3x3, 3x2, 2x3 and 2x2 taps
    # 64 -> 64 channels, 3x3: in bf16 the filters-in-registers kernel (persistent workgroups walking 256-pixel tiles,
    # input rows staged once in LDS); every element compared, M = 65856 with a ragged last tile of 64 pixels
    (21, 56, 56, 64, 64, 3, 3, 1, 1),
    (30, 52, 51, 64, 64, 3, 3, 1, 1),   # the shortest rows that kernel takes (a tile touches 8 input rows), H != W, odd W, M = 79560
    (20, 60, 62, 64, 64, 3, 3, 1, 1),   # the longest (patch rows of 64 pixels are full)
    (65, 32, 32, 64, 64, 3, 3, 1, 1),   # rows too short for it: the register-staged 256x64 tile at a large M
]


def _tol(dtype):
    return 2e-2 if dtype == D.DSP_BF16 else 1e-4


@pytest.mark.parametrize("dtype", [D.DSP_FP32, D.DSP_BF16], ids=["fp32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv_forward_dgrad_wgrad(shape, dtype):
    N, H, W, Ci, Co, R, S, st, pd = shape
    rng = np.random.default_rng(hash(shape) % 2**32)
    x = round_like(rng.standard_normal((N, Ci, H, W)), dtype)
    w = round_like(rng.standard_normal((Co, Ci, R, S)) * np.sqrt(2.0 / (Ci * R * S)), dtype)
    y_ref = O.conv2d_forward(x, w, st, pd)
    dy = round_like(rng.standard_normal(y_ref.shape), dtype)
    dx_ref = O.conv2d_backward_data(dy, w, x.shape, st, pd)
    dw_ref = O.conv2d_backward_weight(x, dy, w.shape, st, pd)

    td = torch.bfloat16 if dtype == D.DSP_BF16 else torch.float32
    d_x, d_dy = to_dev(x, dtype), to_dev(dy, dtype)
    d_w = torch.from_numpy(w.transpose(0, 2, 3, 1).copy()).to("cuda", td)                      # [co][r][s][ci]
    d_wt = torch.from_numpy(dgrad_filter_copy(w, st, pd)).to("cuda", td)   # [ci][R-1-r][S-1-s][co] (stride 2: by parity class)
    d_y = torch.full((N * y_ref.shape[2] * y_ref.shape[3] * Co,), float("nan"), device="cuda", dtype=td)
    D.dsp_conv_forward(dtype, d_x, d_w, d_y, N, H, W, Ci, Co, R, S, st, pd)
    torch.cuda.synchronize()
    assert rel_err(from_dev(d_y, y_ref.shape), y_ref) < _tol(dtype)
    assert np.abs(from_dev(d_y, y_ref.shape) - y_ref).max() < _tol(dtype) * 10 * max(1.0, np.abs(y_ref).max())

    d_dx = torch.full((N * H * W * Ci,), float("nan"), device="cuda", dtype=td)
    D.dsp_conv_backward_data(dtype, d_dy, d_wt, d_dx, N, H, W, Ci, Co, R, S, st, pd, accumulate=False)
    torch.cuda.synchronize()
    got = from_dev(d_dx, x.shape)
    assert rel_err(got, dx_ref) < _tol(dtype)
    # accumulate: dx += ...
    D.dsp_conv_backward_data(dtype, d_dy, d_wt, d_dx, N, H, W, Ci, Co, R, S, st, pd, accumulate=True)
    torch.cuda.synchronize()
    assert rel_err(from_dev(d_dx, x.shape), 2 * dx_ref) < _tol(dtype)

    ws_bytes = D.dsp_conv_workspace_bytes(N, H, W, Ci, Co, R, S, st, pd)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    d_dw = torch.full((Co * R * S * Ci,), float("nan"), device="cuda", dtype=torch.float32)
    D.dsp_conv_backward_weight(dtype, d_x, d_dy, d_dw, N, H, W, Ci, Co, R, S, st, pd, ws, ws_bytes)
    torch.cuda.synchronize()
    dw = d_dw.cpu().numpy().astype(np.float64).reshape(Co, R, S, Ci).transpose(0, 3, 1, 2)
    assert rel_err(dw, dw_ref) < _tol(dtype)
    # run-to-run identical (fixed-order split reduction)
    d_dw2 = torch.empty_like(d_dw)
    D.dsp_conv_backward_weight(dtype, d_x, d_dy, d_dw2, N, H, W, Ci, Co, R, S, st, pd, ws, ws_bytes)
    torch.cuda.synchronize()
    assert torch.equal(d_dw, d_dw2)


# (N, H, W, Cin, Cout, R, S, stride, pad, groups)
GROUPED = [
    (3, 9, 9, 32, 48, 3, 3, 1, 1, 4),       # 8 -> 12 channels per group: bf16 rows of the output are no whole 16-byte runs
    (2, 12, 12, 64, 64, 3, 3, 2, 1, 8),     # stride 2 (parity classes per group)
    (2, 8, 8, 128, 128, 3, 3, 1, 1, 2),     # 64 -> 64 per group
    (2, 6, 6, 12, 6, 1, 1, 1, 0, 3),        # 4 -> 2 per group: element-wise paths
    (2, 7, 7, 16, 16, 3, 3, 1, 1, 16),      # depthwise
    (2, 10, 10, 512, 512, 3, 3, 1, 1, 8),   # ResNeXt-29 (8 x 64d) stage 1
    (1, 9, 9, 256, 256, 3, 3, 2, 1, 8),     # 32 -> 32 per group, stride 2, odd sides
    (5, 6, 6, 24, 64, 1, 1, 1, 0, 2),       # 12 -> 32 per group
]


@pytest.mark.parametrize("dtype", [D.DSP_FP32, D.DSP_BF16], ids=["fp32", "bf16"])
@pytest.mark.parametrize("shape", GROUPED, ids=lambda s: "x".join(map(str, s)))
def test_grouped_conv_forward_dgrad_wgrad(shape, dtype):
    """The three kernels on grouped convolutions against the oracle's (one ordinary convolution per group); tensors start
    as NaN so that a channel a group forgot to write shows."""
    N, H, W, Ci, Co, R, S, st, pd, G = shape
    rng = np.random.default_rng(hash(shape) % 2**32)
    x = round_like(rng.standard_normal((N, Ci, H, W)), dtype)
    w = round_like(rng.standard_normal((Co, Ci // G, R, S)) * np.sqrt(2.0 * G / (Ci * R * S)), dtype)
    y_ref = O.conv2d_forward(x, w, st, pd, G)
    dy = round_like(rng.standard_normal(y_ref.shape), dtype)
    dx_ref = O.conv2d_backward_data(dy, w, x.shape, st, pd, G)
    dw_ref = O.conv2d_backward_weight(x, dy, w.shape, st, pd, G)

    td = torch.bfloat16 if dtype == D.DSP_BF16 else torch.float32
    d_x, d_dy = to_dev(x, dtype), to_dev(dy, dtype)
    d_w = torch.from_numpy(w.transpose(0, 2, 3, 1).copy()).to("cuda", td)         # [co][r][s][ci within the group]
    d_wt = torch.from_numpy(dgrad_filter_copy(w, st, pd, G)).to("cuda", td)
    d_y = torch.full((N * y_ref.shape[2] * y_ref.shape[3] * Co,), float("nan"), device="cuda", dtype=td)
    D.dsp_grouped_conv_forward(dtype, d_x, d_w, d_y, N, H, W, Ci, Co, R, S, st, pd, G)
    torch.cuda.synchronize()
    assert rel_err(from_dev(d_y, y_ref.shape), y_ref) < _tol(dtype)

    d_dx = torch.full((N * H * W * Ci,), float("nan"), device="cuda", dtype=td)
    D.dsp_grouped_conv_backward_data(dtype, d_dy, d_wt, d_dx, N, H, W, Ci, Co, R, S, st, pd, G, accumulate=False)
    torch.cuda.synchronize()
    assert rel_err(from_dev(d_dx, x.shape), dx_ref) < _tol(dtype)
    D.dsp_grouped_conv_backward_data(dtype, d_dy, d_wt, d_dx, N, H, W, Ci, Co, R, S, st, pd, G, accumulate=True)
    torch.cuda.synchronize()
    assert rel_err(from_dev(d_dx, x.shape), 2 * dx_ref) < _tol(dtype)

    ws_bytes = D.dsp_grouped_conv_workspace_bytes(N, H, W, Ci, Co, R, S, st, pd, G)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    d_dw = torch.full((Co * R * S * (Ci // G),), float("nan"), device="cuda", dtype=torch.float32)
    D.dsp_grouped_conv_backward_weight(dtype, d_x, d_dy, d_dw, N, H, W, Ci, Co, R, S, st, pd, G, ws, ws_bytes)
    torch.cuda.synchronize()
    dw = d_dw.cpu().numpy().astype(np.float64).reshape(Co, R, S, Ci // G).transpose(0, 3, 1, 2)
    assert rel_err(dw, dw_ref) < _tol(dtype)
    with pytest.raises(D.DSPError):
        D.dsp_grouped_conv_forward(dtype, d_x, d_w, d_y, N, H, W, Ci, Co, R, S, st, pd, 5 if G != 5 else 7)  # 5 divides no case


def test_conv_rejects_bad_arguments():
    x = torch.zeros(16, device="cuda")
    with pytest.raises(D.DSPError):
        D.dsp_conv_forward(D.DSP_FP32, x, x, x, 1, 2, 2, 4, 4, 3, 3, 0, 1)  # stride 0
    with pytest.raises(D.DSPError):
        D.dsp_conv_backward_data(D.DSP_FP32, x, x, x, 1, 8, 8, 4, 4, 3, 3, 3, 1)  # stride 3 unsupported
    with pytest.raises(D.DSPError):
        D.dsp_conv_backward_weight(D.DSP_FP32, x, x, x, 64, 32, 32, 16, 16, 3, 3, 1, 1, None, 0)  # no workspace


# ---- the layer shapes of the benchmark configurations at their full sizes ------------------------------
# The large tiles (128x128, 128x64, the 128x128 backward-weight tile, the dilated vector kernel) and
# the launch shapes bench.py times only occur at these sizes, where the full fp64 convolution would take
# minutes: a sample of output elements is checked, each computed by the oracle from the definition, plus
# the corners of every tensor (first / last image, channel and pixel: tile and slice tails).
FULL = [
    (D.DSP_FP32, 128, 32, 32, 16, 16, 3, 3, 1, 1),     # ResNet-20/56 stage 1 (register-resident filters, streaming wgrad)
    (D.DSP_FP32, 128, 16, 16, 32, 32, 3, 3, 1, 1),     # stage 2
    (D.DSP_FP32, 128, 8, 8, 64, 64, 3, 3, 1, 1),       # stage 3
    (D.DSP_FP32, 128, 32, 32, 16, 32, 3, 3, 2, 1),     # stage transition, stride 2 (dilated backward-data)
    (D.DSP_BF16, 64, 14, 14, 256, 256, 3, 3, 1, 1),    # ResNet-50 conv4_x 3x3
    (D.DSP_BF16, 64, 14, 14, 256, 1024, 1, 1, 1, 0),   # its 1x1 expansion
    (D.DSP_BF16, 64, 14, 14, 1024, 256, 1, 1, 1, 0),   # and reduction
    (D.DSP_BF16, 256, 28, 28, 128, 128, 3, 3, 1, 1),   # ResNet-18 stage 2 (128x128 tiles)
    (D.DSP_BF16, 256, 56, 56, 64, 128, 3, 3, 2, 1),    # ResNet-18 stage transition
    (D.DSP_BF16, 256, 7, 7, 512, 512, 3, 3, 1, 1),     # ResNet-18 stage 4 (7x7 maps: pixel runs cross image rows; direct-to-LDS 256x128 tiles)
    (D.DSP_BF16, 256, 14, 14, 256, 256, 3, 3, 1, 1),   # ResNet-18 stage 3 (direct-to-LDS 256x256 tiles)
    (D.DSP_BF16, 250, 14, 14, 256, 256, 3, 3, 1, 1),   # the same with a ragged last row tile (M = 49000)
    (D.DSP_BF16, 125, 14, 14, 256, 384, 3, 3, 1, 1),   # direct-to-LDS 256x128 tiles, three column tiles, ragged rows
    (D.DSP_BF16, 256, 56, 56, 64, 64, 3, 3, 1, 1),     # ResNet-18 stage 1 (filters in registers, 3136 tiles on 256 workgroups)
    (D.DSP_BF16, 128, 32, 32, 512, 512, 3, 3, 1, 1, 8),   # ResNeXt-29 (8 x 64d) stage 1: 8 groups of 64 -> 64
    (D.DSP_BF16, 128, 32, 32, 1024, 1024, 3, 3, 2, 1, 8), # stage 2 entry: 128 -> 128 per group, stride 2
    (D.DSP_FP32, 64, 8, 8, 2048, 2048, 3, 3, 1, 1, 8),    # stage 3: 256 -> 256 per group
]


def _sample(rng, shape, n):
    corners = [tuple(0 for _ in shape), tuple(d - 1 for d in shape)]
    rand = [tuple(int(rng.integers(0, d)) for d in shape) for _ in range(n)]
    return corners + rand


@pytest.mark.parametrize("cfg", FULL, ids=lambda c: ("bf16_" if c[0] == D.DSP_BF16 else "fp32_") + "x".join(map(str, c[1:])))
def test_conv_full_size_sampled(cfg):
    dtype, N, H, W, Ci, Co, R, S, st, pd = cfg[:10]
    G = cfg[10] if len(cfg) > 10 else 1
    rng = np.random.default_rng(1000 + Ci * 7 + Co * 3 + H)
    Ho, Wo = (H + 2 * pd - R) // st + 1, (W + 2 * pd - S) // st + 1
    x = round_like(rng.standard_normal((N, Ci, H, W), dtype=np.float32), dtype)
    w = round_like((rng.standard_normal((Co, Ci // G, R, S)) * np.sqrt(2.0 * G / (Ci * R * S))).astype(np.float32), dtype)
    dy = round_like(rng.standard_normal((N, Co, Ho, Wo), dtype=np.float32), dtype)
    td = torch.bfloat16 if dtype == D.DSP_BF16 else torch.float32
    d_x, d_dy = to_dev(x, dtype), to_dev(dy, dtype)
    d_w = torch.from_numpy(np.ascontiguousarray(w.transpose(0, 2, 3, 1))).to("cuda", td)
    d_wt = torch.from_numpy(dgrad_filter_copy(w, st, pd, G)).to("cuda", td)
    # relative to the typical magnitude of the tensor: stored bf16 has 8 mantissa bits, fp32 sums ~1e-6
    tol = 1e-2 if dtype == D.DSP_BF16 else 1e-4

    d_y = torch.full((N * Ho * Wo * Co,), float("nan"), device="cuda", dtype=td)
    D.dsp_grouped_conv_forward(dtype, d_x, d_w, d_y, N, H, W, Ci, Co, R, S, st, pd, G)
    torch.cuda.synchronize()
    assert not torch.isnan(d_y.float()).any()
    y = d_y.view(N, Ho, Wo, Co)
    idx = _sample(rng, (N, Co, Ho, Wo), 48)
    ref = O.conv2d_forward_at(x, w, st, pd, idx, G)
    got = np.array([float(y[n, ho, wo, k]) for (n, k, ho, wo) in idx])
    scale = max(np.sqrt(np.mean(ref ** 2)), 1e-6)
    assert np.abs(got - ref).max() < tol * 4 * scale, (np.abs(got - ref).max(), scale)

    d_dx = torch.full((N * H * W * Ci,), float("nan"), device="cuda", dtype=td)
    D.dsp_grouped_conv_backward_data(dtype, d_dy, d_wt, d_dx, N, H, W, Ci, Co, R, S, st, pd, G, accumulate=False)
    torch.cuda.synchronize()
    assert not torch.isnan(d_dx.float()).any()
    dx = d_dx.view(N, H, W, Ci)
    idx = _sample(rng, (N, Ci, H, W), 48)
    ref = O.conv2d_backward_data_at(dy, w, x.shape, st, pd, idx, G)
    got = np.array([float(dx[n, hi, wi, c]) for (n, c, hi, wi) in idx])
    scale = max(np.sqrt(np.mean(ref ** 2)), 1e-6)
    assert np.abs(got - ref).max() < tol * 4 * scale, (np.abs(got - ref).max(), scale)

    ws_bytes = D.dsp_grouped_conv_workspace_bytes(N, H, W, Ci, Co, R, S, st, pd, G)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    d_dw = torch.full((Co * R * S * (Ci // G),), float("nan"), device="cuda", dtype=torch.float32)
    D.dsp_grouped_conv_backward_weight(dtype, d_x, d_dy, d_dw, N, H, W, Ci, Co, R, S, st, pd, G, ws, ws_bytes)
    torch.cuda.synchronize()
    assert not torch.isnan(d_dw).any()
    dw = d_dw.view(Co, R, S, Ci // G)
    idx = _sample(rng, (Co, Ci // G, R, S), 24)
    ref = O.conv2d_backward_weight_at(x, dy, st, pd, idx, G)
    got = np.array([float(dw[k, r, s, c]) for (k, c, r, s) in idx])
    scale = max(np.sqrt(np.mean(ref ** 2)), 1e-6)
    # fp32 accumulation over N*Ho*Wo products of unit-variance terms
    assert np.abs(got - ref).max() < 1e-3 * scale, (np.abs(got - ref).max(), scale)
