"""Every non-convolution kernel of a block, alone, against the oracle's layer on IDENTICAL stored inputs.

Each test hands the kernel and the oracle the same tensors (rounded once to the storage type), so a ReLU
mask or a pooling choice is the same integer decision on both sides and the comparison is strict:
1e-4 in fp32, 2e-2 in bf16 (relative L2), element for element; integer results (pooling choices, pooled
values, copies) bit for bit.  Shapes span several workgroups, ragged tails, channel counts off the 16-byte
run, more channel vectors than one workgroup row holds, and an ImageNet-sized map (M = 401408 rows)."""
import numpy as np
import pytest
import torch

import paper_1909_02625_amd as D
from oracle import dsp_oracle as O
from tests.gpu_harness import from_dev, rel_err, round_like, to_dev, torch_dtype

pytestmark = pytest.mark.gpu

DTYPES = [D.DSP_FP32, D.DSP_BF16]
IDS = ["fp32", "bf16"]
TOL = {D.DSP_FP32: 1e-4, D.DSP_BF16: 2e-2}
EPS = 1e-5

# (N, C, H, W)
BN_SHAPES = [
    (3, 24, 7, 5),       # ragged rows, several channel vectors
    (2, 6, 5, 5),        # channel count off the 16-byte run: element-wise path
    (4, 16, 32, 32),     # CIFAR stage 1 rows
    (2, 2048, 3, 3),     # more channel vectors than one workgroup row holds (fp32: 512)
    (5, 64, 1, 1),       # 5 values per channel
    (128, 64, 56, 56),   # ImageNet-sized map: M = 401408 rows, 512 partial sums per channel
]


def _dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda()


@pytest.mark.parametrize("dtype", DTYPES, ids=IDS)
@pytest.mark.parametrize("shape", BN_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("relu,res", [(True, False), (True, True), (False, False)], ids=["relu", "res_relu", "plain"])
def test_batch_norm_forward_and_backward(shape, dtype, relu, res):
    N, C, H, W = shape
    if res and N * C * H * W > 10_000_000 and dtype == D.DSP_FP32:
        pytest.skip("the residual variant at full size is covered in bf16")
    tol = TOL[dtype]
    rng = np.random.default_rng(C * 1000 + H)
    M = N * H * W
    x = round_like(rng.standard_normal(shape) * 1.5 + 0.3, dtype)
    r = round_like(rng.standard_normal(shape), dtype) if res else None
    gamma = (1.0 + 0.25 * rng.standard_normal(C)).astype(np.float32)
    beta = (0.25 * rng.standard_normal(C)).astype(np.float32)

    # ---- forward
    z, mean, invstd = O.bn_forward(x, gamma, beta, EPS)
    if res:
        z = z + r
    y_ref = np.maximum(z, 0.0) if relu else z
    ws_bytes = D.dsp_bn_workspace_bytes(C)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    td = torch_dtype(dtype)
    d_x = to_dev(x, dtype)
    d_r = to_dev(r, dtype) if res else None
    d_y = torch.full((M * C,), float("nan"), device="cuda", dtype=td)
    d_mean, d_invstd = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    d_gamma, d_beta = _dev_f32(gamma), _dev_f32(beta)
    D.dsp_bn_forward(dtype, d_x, d_r, d_y, d_gamma, d_beta, EPS, M, C, relu, d_mean, d_invstd, ws, ws_bytes)
    torch.cuda.synchronize()
    y = from_dev(d_y, shape)
    assert rel_err(y, y_ref) < (tol if dtype == D.DSP_FP32 else 4e-3)   # bf16: one rounding of the result
    np.testing.assert_allclose(d_mean.cpu().numpy(), mean, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(d_invstd.cpu().numpy(), invstd, rtol=1e-5)
    if relu:  # the sign pattern is an integer result: it may differ only where the pre-activation is rounding noise
        flips = (y > 0) != (y_ref > 0)
        assert np.all(np.abs(z[flips]) < 1e-5 * (1 if dtype == D.DSP_FP32 else 1e3))

    # ---- backward on the same stored x, y, statistics
    y_st = round_like(y_ref, dtype)
    mean32, invstd32 = mean.astype(np.float32), invstd.astype(np.float32)
    dy = round_like(rng.standard_normal(shape) * 0.1, dtype)
    g = dy * (y_st > 0) if relu else dy
    dx_ref, dg_ref, db_ref = O.bn_backward(g, x, gamma, mean32, invstd32)
    d_dy, d_yst = to_dev(dy, dtype), to_dev(y_st, dtype)
    d_dx = torch.full((M * C,), float("nan"), device="cuda", dtype=td)
    d_dres = torch.full((M * C,), float("nan"), device="cuda", dtype=td) if res else None
    d_dg, d_db = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    D.dsp_bn_backward(dtype, d_dy, d_x, d_yst, d_dx, d_dres, False, False, d_gamma, _dev_f32(mean32), _dev_f32(invstd32), d_dg,
                      d_db, M, C, relu, ws, ws_bytes)
    torch.cuda.synchronize()
    assert rel_err(from_dev(d_dx, shape), dx_ref) < tol
    scale = max(1e-6, float(np.abs(dg_ref).max()))
    assert np.abs(d_dg.cpu().numpy() - dg_ref).max() < 1e-4 * scale
    assert np.abs(d_db.cpu().numpy() - db_ref).max() < 1e-4 * max(1e-6, float(np.abs(db_ref).max()))
    if res:
        got = from_dev(d_dres, shape)
        np.testing.assert_array_equal(got, g)   # a masked copy of dy: exact in either storage type

    # ---- accumulate variants: dx += ..., dres += ... on top of stored gradients
    if M * C < 5_000_000:
        dx0 = round_like(rng.standard_normal(shape) * 0.1, dtype)
        dr0 = round_like(rng.standard_normal(shape) * 0.1, dtype)
        d_dx2, d_dr2 = to_dev(dx0, dtype), (to_dev(dr0, dtype) if res else None)
        D.dsp_bn_backward(dtype, d_dy, d_x, d_yst, d_dx2, d_dr2, True, True, d_gamma, _dev_f32(mean32), _dev_f32(invstd32),
                          d_dg, d_db, M, C, relu, ws, ws_bytes)
        torch.cuda.synchronize()
        assert rel_err(from_dev(d_dx2, shape), dx0 + dx_ref) < tol
        if res:
            assert rel_err(from_dev(d_dr2, shape), dr0 + g) < (1e-6 if dtype == D.DSP_FP32 else 4e-3)


@pytest.mark.parametrize("dtype", DTYPES, ids=IDS)
@pytest.mark.parametrize("shape", [(3, 24, 7, 5), (4, 16, 32, 32), (2, 2048, 3, 3), (32, 64, 56, 56)], ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("res", [True, False], ids=["res", "nores"])
def test_batch_norm_relu_decided_from_sign_bytes(shape, dtype, res):
    """The forward apply kernel's sign bytes (bit k of byte v = element k of channel vector v of the stored output is
    positive) against the stored output itself, and the backward pass that reads them against the one that reads y:
    the same bits in dx, dres, dgamma, dbeta, overwriting and accumulating."""
    N, C, H, W = shape
    rng = np.random.default_rng(C * 7 + H)
    M = N * H * W
    td = torch_dtype(dtype)
    vw = 8 if dtype == D.DSP_BF16 else 4
    x = round_like(rng.standard_normal(shape) * 1.5 + 0.3, dtype)
    r = round_like(rng.standard_normal(shape), dtype) if res else None
    gamma = (1.0 + 0.25 * rng.standard_normal(C)).astype(np.float32)
    beta = (0.25 * rng.standard_normal(C)).astype(np.float32)
    ws_bytes = D.dsp_bn_workspace_bytes(C)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    d_x, d_r = to_dev(x, dtype), (to_dev(r, dtype) if res else None)
    d_gamma, d_beta = _dev_f32(gamma), _dev_f32(beta)
    d_mean, d_invstd = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    d_y = torch.full((M * C,), float("nan"), device="cuda", dtype=td)
    nb = D.dsp_bn_relu_bits_bytes(dtype, M, C)
    assert nb == M * C // vw
    d_bits = torch.full((nb,), 0xAA, device="cuda", dtype=torch.uint8)
    D.dsp_bn_forward_bits(dtype, d_x, d_r, d_y, d_gamma, d_beta, EPS, M, C, d_mean, d_invstd, d_bits, ws, ws_bytes)
    d_y2 = torch.full((M * C,), float("nan"), device="cuda", dtype=td)
    D.dsp_bn_forward(dtype, d_x, d_r, d_y2, d_gamma, d_beta, EPS, M, C, True, d_mean, d_invstd, ws, ws_bytes)
    torch.cuda.synchronize()
    assert torch.equal(d_y.view(torch.int16 if dtype == D.DSP_BF16 else torch.int32), d_y2.view(torch.int16 if dtype == D.DSP_BF16 else torch.int32))
    pos = (d_y.float() > 0).view(-1, vw).to(torch.int32)
    want = (pos << torch.arange(vw, device="cuda", dtype=torch.int32)).sum(dim=1).to(torch.uint8)
    assert torch.equal(d_bits, want)
    dy = to_dev(round_like(rng.standard_normal(shape) * 0.1, dtype), dtype)
    dx0 = to_dev(round_like(rng.standard_normal(shape) * 0.1, dtype), dtype)
    for acc in (False, True):
        outs = []
        for bits in (False, True):
            d_dx = dx0.clone() if acc else torch.full((M * C,), float("nan"), device="cuda", dtype=td)
            d_dr = (dx0.clone() if acc else torch.full((M * C,), float("nan"), device="cuda", dtype=td)) if res else None
            d_dg, d_db = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
            if bits:
                D.dsp_bn_backward_bits(dtype, dy, d_x, d_bits, d_dx, d_dr, acc, acc, d_gamma, d_mean, d_invstd, d_dg, d_db, M, C, ws, ws_bytes)
            else:
                D.dsp_bn_backward(dtype, dy, d_x, d_y, d_dx, d_dr, acc, acc, d_gamma, d_mean, d_invstd, d_dg, d_db, M, C, True, ws, ws_bytes)
            torch.cuda.synchronize()
            outs.append([d_dx.clone(), d_dg.clone(), d_db.clone()] + ([d_dr.clone()] if res else []))
        for u, v in zip(*outs):
            assert torch.equal(u.view(torch.uint8), v.view(torch.uint8))


def test_batch_norm_sign_bytes_need_whole_channel_vectors():
    x = torch.zeros(4096, device="cuda")
    ws = torch.empty(D.dsp_bn_workspace_bytes(6), dtype=torch.uint8, device="cuda")
    assert D.dsp_bn_relu_bits_bytes(D.DSP_FP32, 16, 6) == 0
    with pytest.raises(D.DSPError):
        D.dsp_bn_forward_bits(D.DSP_FP32, x, None, x, x, x, EPS, 16, 6, x, x, x.view(torch.uint8), ws, ws.numel())


FUSED_SHAPES = [  # (N, C, H, W, k, stride, pad)
    (2, 16, 9, 9, 3, 2, 1),       # odd map: windows cut by every border
    (3, 24, 6, 10, 3, 2, 1),      # the stem's window on a small even map, three channel vectors
    (3, 24, 8, 10, 2, 2, 0),      # 2 x 2 windows, no padding, three channel vectors
    (2, 64, 7, 5, 3, 1, 1),       # overlapping stride-1 windows
    (2, 8, 6, 6, 4, 2, 1),        # the largest window the tap code holds
    (16, 64, 112, 112, 3, 2, 1),  # ResNet-18 stem at 1/16 of its batch: several grid-stride trips per workgroup
]


@pytest.mark.parametrize("shape", FUSED_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_bn_relu_maxpool_in_one_pass_and_relu_decided_from_x(shape):
    """The two forms a block uses for a batch norm + ReLU without residual: the pool that forms the normalised tensor on
    the fly, and the backward pass that takes the ReLU decision from x.  Both must leave the very bits of the separate
    kernels (which the tests above check against the oracle), so the comparison is bit for bit; on top, the pooled
    tensor is checked against the oracle's layers on the same stored input."""
    N, C, H, W, k, st, pd = shape
    dtype = D.DSP_BF16
    rng = np.random.default_rng(11 * C + H + k)
    M = N * H * W
    x = round_like(rng.standard_normal((N, C, H, W)) * 1.5 + 0.3, dtype)
    gamma = (1.0 + 0.25 * rng.standard_normal(C)).astype(np.float32)
    gamma[::5] *= -1.0            # decreasing channels as well
    beta = (0.25 * rng.standard_normal(C)).astype(np.float32)
    beta[1::7] = -3.0             # channels the ReLU zeroes almost everywhere: windows full of ties
    ws_bytes = D.dsp_bn_workspace_bytes(C)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    d_x, d_gamma, d_beta = to_dev(x, dtype), _dev_f32(gamma), _dev_f32(beta)
    d_y = torch.full((M * C,), float("nan"), device="cuda", dtype=torch.bfloat16)
    d_mean, d_invstd = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    D.dsp_bn_forward(dtype, d_x, None, d_y, d_gamma, d_beta, EPS, M, C, True, d_mean, d_invstd, ws, ws_bytes)
    Ho, Wo = (H + 2 * pd - k) // st + 1, (W + 2 * pd - k) // st + 1
    n_out = N * Ho * Wo * C
    d_p = torch.full((n_out,), float("nan"), device="cuda", dtype=torch.bfloat16)
    d_a = torch.full((n_out,), 255, device="cuda", dtype=torch.uint8)
    D.dsp_maxpool_forward(dtype, d_y, d_p, d_a, N, H, W, C, k, st, pd)

    d_p2 = torch.full((n_out,), float("nan"), device="cuda", dtype=torch.bfloat16)
    d_a2 = torch.full((n_out,), 255, device="cuda", dtype=torch.uint8)
    d_mean2, d_invstd2 = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    d_coef = torch.empty(2 * C, device="cuda")
    D.dsp_bn_relu_maxpool_forward(dtype, d_x, d_gamma, d_beta, EPS, N, H, W, C, k, st, pd, d_p2, d_a2, d_mean2, d_invstd2, d_coef,
                                  ws, ws_bytes)
    torch.cuda.synchronize()
    assert torch.equal(d_mean, d_mean2) and torch.equal(d_invstd, d_invstd2)
    assert torch.equal(d_p.view(torch.int16), d_p2.view(torch.int16))
    assert torch.equal(d_a, d_a2)
    # against the layers' definitions on the stored input (values: one rounding of the normalised tensor)
    z, _, _ = O.bn_forward(x, gamma, beta, EPS)
    p_ref, _ = O.maxpool_forward(np.maximum(z, 0.0), k, st, pd)
    assert rel_err(from_dev(d_p2, p_ref.shape), p_ref) < 4e-3

    dy = round_like(rng.standard_normal((N, C, H, W)) * 0.1, dtype)
    d_dy = to_dev(dy, dtype)
    outs = []
    for from_x in (False, True):
        d_dx = torch.full((M * C,), float("nan"), device="cuda", dtype=torch.bfloat16)
        d_dg, d_db = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
        if from_x:
            D.dsp_bn_relu_backward_from_x(dtype, d_dy, d_x, d_coef, d_dx, False, d_gamma, d_mean, d_invstd, d_dg, d_db, M, C, ws, ws_bytes)
        else:
            D.dsp_bn_backward(dtype, d_dy, d_x, d_y, d_dx, None, False, False, d_gamma, d_mean, d_invstd, d_dg, d_db, M, C, True,
                              ws, ws_bytes)
        torch.cuda.synchronize()
        outs.append((d_dx.view(torch.int16).clone(), d_dg.clone(), d_db.clone()))
    for u, v in zip(*outs):
        assert torch.equal(u, v)

    # the pool's backward folded into the batch norm's: every masked gradient is the one dsp_maxpool_backward +
    # dsp_bn_backward work on; the channel sums are taken in another order (doubles, then one rounding to float)
    if (k, st, pd) == (3, 2, 1) and H % 2 == 0 and W % 2 == 0:
        dp = round_like(rng.standard_normal((N, C, Ho, Wo)) * 0.1, dtype)
        d_dp = to_dev(dp, dtype)
        d_dy2 = torch.full((M * C,), float("nan"), device="cuda", dtype=torch.bfloat16)
        D.dsp_maxpool_backward(dtype, d_dp, d_a, d_dy2, False, N, H, W, C, k, st, pd)
        dx0 = to_dev(round_like(rng.standard_normal((N, C, H, W)) * 0.1, dtype), dtype)
        for acc in (False, True):
            res = []
            for fused in (False, True):
                d_dx = dx0.clone() if acc else torch.full((M * C,), float("nan"), device="cuda", dtype=torch.bfloat16)
                d_dg, d_db = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
                if fused:
                    D.dsp_bn_relu_maxpool_backward(dtype, d_dp, d_a, d_x, d_coef, d_dx, acc, d_gamma, d_mean, d_invstd, d_dg, d_db,
                                                   N, H, W, C, k, st, pd, ws, ws_bytes)
                else:
                    D.dsp_bn_backward(dtype, d_dy2, d_x, d_y, d_dx, None, False, acc, d_gamma, d_mean, d_invstd, d_dg, d_db, M, C, True,
                                      ws, ws_bytes)
                torch.cuda.synchronize()
                res.append((d_dx.float().cpu().numpy(), d_dg.cpu().numpy(), d_db.cpu().numpy()))
            (dx_a, dg_a, db_a), (dx_b, dg_b, db_b) = res
            np.testing.assert_allclose(dg_b, dg_a, rtol=1e-6, atol=1e-6 * float(np.abs(dg_a).max()))
            np.testing.assert_allclose(db_b, db_a, rtol=1e-6, atol=1e-6 * float(np.abs(db_a).max()))
            # dx: the same bf16 values except where a coefficient moved by an ulp of float and tipped a rounding
            differ = dx_a != dx_b
            assert differ.mean() < 1e-3 and np.all(np.abs(dx_a - dx_b)[differ] <= 2.0 ** -7 * np.abs(dx_a)[differ] + 1e-30)
    else:
        with pytest.raises(D.DSPError):
            D.dsp_bn_relu_maxpool_backward(dtype, d_p, d_a, d_x, d_coef, d_y, False, d_gamma, d_mean, d_invstd, d_mean2, d_invstd2,
                                           N, H, W, C, k, st, pd, ws, ws_bytes)


def test_bn_relu_maxpool_rejects_what_it_does_not_cover():
    x = torch.zeros(4096, device="cuda")
    ws = torch.empty(D.dsp_bn_workspace_bytes(8), dtype=torch.uint8, device="cuda")
    for args in [(D.DSP_FP32, 8, 3), (D.DSP_BF16, 6, 3), (D.DSP_BF16, 8, 5)]:   # fp32, channels off the 16-byte run, window 5
        dt, C, k = args
        with pytest.raises(D.DSPError):
            D.dsp_bn_relu_maxpool_forward(dt, x, x, x, EPS, 1, 8, 8, C, k, 2, 1, x, x.view(torch.uint8), x, x, x, ws, ws.numel())


POOL_SHAPES = [  # (N, C, H, W, k, stride, pad)
    (2, 16, 9, 9, 3, 2, 1),
    (3, 6, 8, 8, 2, 2, 0),       # channel count off the 16-byte run
    (2, 64, 7, 5, 3, 1, 1),      # overlapping windows
    (16, 64, 112, 112, 3, 2, 1), # ResNet-18 stem at 1/16 of its batch
]


@pytest.mark.parametrize("dtype", DTYPES, ids=IDS)
@pytest.mark.parametrize("shape", POOL_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_max_pool_forward_and_backward(shape, dtype):
    N, C, H, W, k, st, pd = shape
    rng = np.random.default_rng(7 + C + H)
    x = round_like(rng.standard_normal((N, C, H, W)), dtype)   # bf16: ties inside a window do occur
    y_ref, arg_ref = O.maxpool_forward(x, k, st, pd)
    Ho, Wo = y_ref.shape[2:]
    td = torch_dtype(dtype)
    d_x = to_dev(x, dtype)
    d_y = torch.full((N * Ho * Wo * C,), float("nan"), device="cuda", dtype=td)
    d_arg = torch.full((N * Ho * Wo * C,), 255, device="cuda", dtype=torch.uint8)
    D.dsp_maxpool_forward(dtype, d_x, d_y, d_arg, N, H, W, C, k, st, pd)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(from_dev(d_y, y_ref.shape), y_ref)      # a selection of stored values: exact
    a = d_arg.cpu().numpy().reshape(N, Ho, Wo, C).transpose(0, 3, 1, 2).astype(np.int64)
    ho = np.arange(Ho).reshape(1, 1, Ho, 1)
    wo = np.arange(Wo).reshape(1, 1, 1, Wo)
    flat = (ho * st + a // k - pd) * W + (wo * st + a % k - pd)           # window position -> source pixel
    np.testing.assert_array_equal(flat, arg_ref)                           # first maximum in row-major order on both sides
    dy = round_like(rng.standard_normal(y_ref.shape), dtype)
    dx_ref = O.maxpool_backward(dy, arg_ref, x.shape)
    d_dy = to_dev(dy, dtype)
    d_dx = torch.full((N * H * W * C,), float("nan"), device="cuda", dtype=td)
    D.dsp_maxpool_backward(dtype, d_dy, d_arg, d_dx, False, N, H, W, C, k, st, pd)
    torch.cuda.synchronize()
    assert rel_err(from_dev(d_dx, x.shape), dx_ref) < (1e-6 if dtype == D.DSP_FP32 else 4e-3)
    dx0 = round_like(rng.standard_normal(x.shape), dtype)
    d_dx2 = to_dev(dx0, dtype)
    D.dsp_maxpool_backward(dtype, d_dy, d_arg, d_dx2, True, N, H, W, C, k, st, pd)
    torch.cuda.synchronize()
    assert rel_err(from_dev(d_dx2, x.shape), dx0 + dx_ref) < (1e-6 if dtype == D.DSP_FP32 else 4e-3)


@pytest.mark.parametrize("dtype", DTYPES, ids=IDS)
@pytest.mark.parametrize("shape", [(3, 20, 7, 5), (2, 7, 3, 3), (64, 256, 32, 32)], ids=lambda s: "x".join(map(str, s)))
def test_sum_of_two_maps_forward_and_backward(shape, dtype):
    rng = np.random.default_rng(sum(shape))
    a, b = round_like(rng.standard_normal(shape), dtype), round_like(rng.standard_normal(shape), dtype)
    n = int(np.prod(shape))
    td = torch_dtype(dtype)
    d_y = torch.full((n,), float("nan"), device="cuda", dtype=td)
    D.dsp_add_forward(dtype, to_dev(a, dtype), to_dev(b, dtype), d_y, n)
    torch.cuda.synchronize()
    # the oracle's layer: the exact sum, stored once.  fp32: one IEEE addition, bit for bit.  bf16: the kernel adds in
    # fp32 and rounds to bf16; that equals the nearest bf16 of the exact sum except for double-rounding ties
    want = (a + b).astype(np.float64) if dtype == D.DSP_FP32 else O.round_bf16(a.astype(np.float64) + b)
    got = from_dev(d_y, shape)
    assert np.mean(got != want) < 1e-5 and rel_err(got, want) < 1e-6
    dy = round_like(rng.standard_normal(shape), dtype)
    d0 = round_like(rng.standard_normal(shape), dtype)
    d_da = torch.full((n,), float("nan"), device="cuda", dtype=td)
    d_db = to_dev(d0, dtype)
    D.dsp_add_backward(dtype, to_dev(dy, dtype), d_da, False, d_db, True, n)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(from_dev(d_da, shape), dy)
    wantb = (d0 + dy).astype(np.float64) if dtype == D.DSP_FP32 else O.round_bf16(d0.astype(np.float64) + dy)
    gotb = from_dev(d_db, shape)
    assert np.mean(gotb != wantb) < 1e-5 and rel_err(gotb, wantb) < 1e-6


@pytest.mark.parametrize("dtype", DTYPES, ids=IDS)
@pytest.mark.parametrize("N,C,H,W,classes", [(5, 24, 3, 3, 10), (8, 64, 8, 8, 100), (256, 512, 7, 7, 1000), (3, 300, 1, 1, 7)])
def test_head_pool_linear_softmax(N, C, H, W, classes, dtype):
    """Global average pool -> linear -> softmax cross-entropy and back, each kernel on the oracle's inputs."""
    rng = np.random.default_rng(N + C + classes)
    x = round_like(rng.standard_normal((N, C, H, W)), dtype)
    wgt = (rng.standard_normal((classes, C)) * np.sqrt(2.0 / C)).astype(np.float32)
    bias = (0.1 * rng.standard_normal(classes)).astype(np.float32)
    labels = rng.integers(0, classes, N).astype(np.int32)
    HW = H * W
    # pool
    p_ref = x.astype(np.float64).mean(axis=(2, 3))
    d_p = torch.empty(N * C, device="cuda")
    D.dsp_gap_forward(dtype, to_dev(x, dtype), d_p, N, HW, C)
    torch.cuda.synchronize()
    assert rel_err(d_p.cpu().numpy().reshape(N, C), p_ref) < 1e-5
    # linear on the oracle's pooled values (as float)
    p32 = p_ref.astype(np.float32)
    z_ref = p32.astype(np.float64) @ wgt.astype(np.float64).T + bias
    d_z = torch.empty(N * classes, device="cuda")
    D.dsp_linear_forward(_dev_f32(p32), _dev_f32(wgt), _dev_f32(bias), d_z, N, C, classes)
    torch.cuda.synchronize()
    assert rel_err(d_z.cpu().numpy().reshape(N, classes), z_ref) < 1e-5
    # loss on the oracle's logits
    z32 = z_ref.astype(np.float32)
    loss_ref, dz_ref = O.SoftmaxCE().value_and_grad(z32, labels)
    d_loss, d_dz, d_rows = torch.zeros(1, device="cuda"), torch.empty(N * classes, device="cuda"), torch.empty(N, device="cuda")
    D.dsp_softmax_ce(_dev_f32(z32), torch.from_numpy(labels).cuda(), d_loss, d_dz, d_rows, N, classes)
    torch.cuda.synchronize()
    assert abs(d_loss.item() - loss_ref) < 1e-5 * abs(loss_ref)
    assert rel_err(d_dz.cpu().numpy().reshape(N, classes), dz_ref) < 1e-5
    # linear backward on the oracle's dz
    dz32 = dz_ref.astype(np.float32)
    d_dp, d_dw, d_dbias = torch.empty(N * C, device="cuda"), torch.empty(classes * C, device="cuda"), torch.empty(classes, device="cuda")
    D.dsp_linear_backward(_dev_f32(p32), _dev_f32(wgt), _dev_f32(dz32), d_dp, d_dw, d_dbias, N, C, classes)
    torch.cuda.synchronize()
    dz64 = dz32.astype(np.float64)
    assert rel_err(d_dp.cpu().numpy().reshape(N, C), dz64 @ wgt) < 1e-5
    assert rel_err(d_dw.cpu().numpy().reshape(classes, C), dz64.T @ p32) < 1e-5
    assert rel_err(d_dbias.cpu().numpy(), dz64.sum(axis=0)) < 1e-5
    # pool backward on the oracle's dp
    dp32 = (dz64 @ wgt).astype(np.float32)
    dx_ref = np.broadcast_to(dp32.astype(np.float64)[:, :, None, None] / HW, x.shape)
    d_dx = torch.full((N * HW * C,), float("nan"), device="cuda", dtype=torch_dtype(dtype))
    D.dsp_gap_backward(dtype, _dev_f32(dp32), d_dx, False, N, HW, C)
    torch.cuda.synchronize()
    assert rel_err(from_dev(d_dx, x.shape), dx_ref) < (1e-6 if dtype == D.DSP_FP32 else 4e-3)


def test_single_layer_entry_points_check_their_arguments():
    x = torch.zeros(64, device="cuda")
    ws = torch.empty(D.dsp_bn_workspace_bytes(4), dtype=torch.uint8, device="cuda")
    with pytest.raises(D.DSPError):
        D.dsp_bn_forward(D.DSP_FP32, x, None, x, x, x, 1e-5, 4, 4, True, x, x, ws, 16)          # workspace too small
    with pytest.raises(D.DSPError):
        D.dsp_bn_backward(D.DSP_FP32, x, x, None, x, None, False, False, x, x, x, x, x, 4, 4, True, ws, ws.numel())  # ReLU mask without y
    with pytest.raises(D.DSPError):
        D.dsp_maxpool_forward(D.DSP_FP32, x, x, x, 1, 2, 2, 4, 3, 2, 3)                          # pad >= window
    with pytest.raises(D.DSPError):
        D.dsp_add_forward(7, x, x, x, 16)                                                        # unknown storage type
    with pytest.raises(D.DSPError):
        D.dsp_softmax_ce(x, None, x, x, x, 4, 4)                                                 # no labels
