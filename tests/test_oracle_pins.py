"""Pins the CPU oracle to things other than itself: the hand-derived rational worked example,
the paper's DSP(p; m) tuples and queue identity, closed forms, adjoint identities, finite
differences, and torch's autograd + SGD for the zero-staleness case."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import dsp_oracle as O
from tests.toy_blocks import BatchIdLoss, CountingBlock, HalfSquare, ScalarBlock
from workloads import get_config, make_batch, make_params
from workloads.gen import perturb_affine

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "dsp_worked_example.txt")


# ----------------------------------------------------------------------------- worked example
def _parse_golden():
    cases, cur = {}, None
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("case "):
            _, name, p, m, beta = line.split()
            cur = {"p": [int(v) for v in p[2:].split(",")], "m": [int(v) for v in m[2:].split(",")],
                   "beta": Fraction(beta[5:])}
            cases[name] = cur
        else:
            key, vals = line.split(":")
            cur[key] = [Fraction(v) for v in vals.split()]
    return cases


@pytest.mark.parametrize("name", ["dsp_beta0", "dsp_beta_half", "bp_beta0"])
def test_worked_example_exact(name):
    c = _parse_golden()[name]
    b0, b1 = ScalarBlock(1, 2), ScalarBlock(Fraction(1, 2), 1)
    orc = O.DSPOracle([b0, b1], HalfSquare(), c["p"], c["m"], Fraction(1, 2), c["beta"])
    losses, x1, x0, g_h1, g_x0, h1 = [], [b1.x[0]], [b0.x[0]], [], [], {}
    for n in range(5):
        rec = orc.tick(Fraction(1), Fraction(1 if n % 2 == 0 else 0))
        if rec["loss"] is not None:
            losses.append(rec["loss"])
        if rec["bwd"][1] is not None:
            x1.append(b1.x[0])
            g_h1.append(rec["g_in"][1])
        if rec["bwd"][0] is not None:
            x0.append(b0.x[0])
            g_x0.append(rec["g_x"][0][0])
        h1[rec["fwd"][0]] = rec["out"][0]
    n = len(c["losses"])
    assert losses[:n] == c["losses"]
    assert x0[:len(c["x0_first"])] == c["x0_first"]
    if "x1" in c:
        assert x1[:len(c["x1"])] == c["x1"]
    if "g_h1" in c:
        assert g_h1[:len(c["g_h1"])] == c["g_h1"]
        assert g_x0[:len(c["g_x0_first"])] == c["g_x0_first"]
        assert h1[3] == c["h1_batch3"][0]


# ----------------------------------------------------------------------------- schedules / queues
PAPER_TUPLES = [  # the six DSP(p; m) rows of the paper's accuracy table, with q from Appendix A
    ((1, 1, 0), (4, 2, 0), (0, 1, 1)), ((2, 2, 0), (6, 3, 0), (0, 1, 1)), ((3, 3, 0), (10, 5, 0), (0, 2, 2)),
    ((1, 1, 1, 0), (6, 4, 2, 0), (0, 1, 1, 1)), ((2, 2, 2, 0), (9, 6, 3, 0), (0, 1, 1, 1)),
    ((3, 3, 3, 0), (15, 10, 5, 0), (0, 2, 2, 2)),
]


@pytest.mark.parametrize("p,m,q", PAPER_TUPLES)
def test_paper_tuples_validate(p, m, q):
    assert O.queue_lengths(p, m) == list(q)


@pytest.mark.parametrize("p,m", [((1, 0), (1, 0)), ((2, 0), (2, 0)), ((1, 1, 0), (2, 2, 0)), ((0, 1, 0), (4, 2, 0)),
                                 ((1, 1), (2, 0)), ((1, 0), (0, 0)), ((1, 1, 0), (4, 4, 0)), ((0, 0, 0), (1, 1, 0)),
                                 ((0, 0, 0), (2, 0, 0))])
def test_invalid_schedules_rejected(p, m):
    with pytest.raises(ValueError):
        O.queue_lengths(p, m)


def _run_counting(p, m, ticks):
    K = len(p)
    blocks = [CountingBlock() for _ in range(K)]
    orc = O.DSPOracle(blocks, BatchIdLoss(), p, m, 1, 0)
    for n in range(ticks):
        orc.tick(n, n)
    return blocks, orc


FORWARD_LOCKED = [((0, 0), (1, 0), (0, 1)), ((0, 0, 0), (2, 1, 0), (0, 1, 1)), ((0, 0, 0, 0), (3, 2, 1, 0), (0, 1, 1, 1)),
                  ((0, 0), (2, 0), (0, 2)), ((0, 0, 0), (5, 2, 1), (0, 3, 1))]


@pytest.mark.parametrize("p,m,q", FORWARD_LOCKED)
def test_forward_locked_schedules(p, m, q):
    """Every p_k = 0 (Section 6's features-replay comparison when m_k = K-1-k): each tick one mini-batch runs
    forward through ALL blocks, block k's backward pass handles the mini-batch of m_k ticks ago with parameters
    that have seen exactly m_k more updates, and the error gradient spends q_k = m_{k-1} - m_k ticks in Q_k."""
    assert O.queue_lengths(p, m) == list(q)
    K = len(p)
    blocks, orc = _run_counting(p, m, 40)
    for rec in orc.log:
        tau = rec["tau"]
        assert rec["fwd"] == [tau] * K and rec["loss_batch"] == tau
        assert rec["bwd"] == [tau - m[k] if tau >= m[k] else None for k in range(K)]
    for k in range(K):
        for n, vb in blocks[k].bwd_version.items():
            assert vb - blocks[k].fwd_version[n] == (m[k] if n >= m[k] else n)


@pytest.mark.parametrize("p,m,_q", PAPER_TUPLES + [((1, 0), (2, 0), None), ((1, 1, 0), (7, 3, 1), None)] + FORWARD_LOCKED)
def test_fifo_timeline_and_staleness(p, m, _q):
    """Real queues reproduce: forward batch tau - sum_{j<k} p_j, backward batch a - m_k, and the
    layer-wise staleness (Section 3.1; proof of Theorem 1: exactly Delta t_k = m_k updates lie
    between the forward and the backward use of block k's parameters for one batch)."""
    K, T = len(p), 64
    blocks, orc = _run_counting(p, m, T)
    for rec in orc.log:
        for k in range(K):
            a = rec["tau"] - sum(p[:k])
            assert rec["fwd"][k] == (a if a >= 0 else None)
            b = a - m[k]
            assert rec["bwd"][k] == (b if b >= 0 else None)
            assert rec["version"][k] == max(0, b)
    for k in range(K):
        for n, vb in blocks[k].bwd_version.items():
            assert vb == n                                    # backward of batch n sees n earlier updates
            assert blocks[k].fwd_version[n] == max(0, n - m[k])
            if n >= m[k]:
                assert vb - blocks[k].fwd_version[n] == m[k]  # layer-wise staleness


def test_figure2_timeline():
    """DSP(1,1,0;4,2,0): staleness {4,2,0} = index difference between forward and backward batch."""
    _, orc = _run_counting((1, 1, 0), (4, 2, 0), 8)
    rec = orc.log[6]
    assert rec["fwd"] == [6, 5, 4] and rec["bwd"] == [2, 3, 4]
    assert [f - b for f, b in zip(rec["fwd"], rec["bwd"])] == [4, 2, 0]
    assert orc.log[3]["bwd"] == [None, 0, 1] and orc.log[2]["loss_batch"] == 0


def test_mismatched_queue_is_caught():
    """If Q_k had the wrong length the stored input would meet another batch's gradient."""
    blocks = [CountingBlock() for _ in range(3)]
    orc = O.DSPOracle(blocks, BatchIdLoss(), (1, 1, 0), (4, 2, 0), 1, 0)
    orc.Q[1] = O._Fifo(1 + 2)  # should be 1 + 1
    with pytest.raises(AssertionError):
        for n in range(16):
            orc.tick(n, n)


# ----------------------------------------------------------------------------- Lemma 1 / Section 5.4
def _scalar_pipeline(p, m, lr, beta=0):
    blocks = [ScalarBlock(Fraction(3, 4), 1), ScalarBlock(Fraction(5, 4), 2), ScalarBlock(Fraction(2, 3), 1)]
    return O.DSPOracle(blocks, HalfSquare(), p, m, lr, beta)


def test_gradient_difference_closed_form_on_scalar_blocks():
    """f_k = x_k^{n_k} h, L = (h_K - l)^2 / 2.  With x_i^f / x_i^b the parameters block i held at the forward /
    backward of batch b: BP_k = n_k x_k^{f,n_k-1} h_k (h_K - l) prod_{i>k} (x_i^f)^{n_i} and DSP_k has x^b in
    place of x^f for the blocks i >= k (its own recompute included); h_k, h_K come from forward parameters."""
    p, m = (1, 1, 0), (4, 2, 0)
    orc = _scalar_pipeline(p, m, Fraction(1, 50), Fraction(1, 2))
    gd = O.GradientDifference(orc)
    P = [0, 1, 2]
    powers = [1, 2, 1]
    hist = []  # hist[tau][k] = parameter of block k at the start of tick tau
    data = []
    seen = 0
    for tau in range(9):  # exact rationals: the digit count multiplies every tick, keep it short
        hist.append([blk.x[0] for blk in orc.blocks])
        h0, l = Fraction(tau % 5 + 1, 3), Fraction(7 - tau % 4, 5)
        data.append((h0, l))
        _, out = gd.tick(h0, l)
        if out is None:
            continue
        b, diff, ref = out
        assert b == tau - m[0]
        xf = [hist[b + P[k]][k] for k in range(3)]
        xb = [hist[b + P[k] + m[k]][k] for k in range(3)]
        h = [data[b][0]]
        for k in range(3):
            h.append(xf[k] ** powers[k] * h[k])
        err = h[3] - data[b][1]
        for k in range(3):
            def grad(x):
                g = powers[k] * x[k] ** (powers[k] - 1) * h[k] * err
                for i in range(k + 1, 3):
                    g *= x[i] ** powers[i]
                return g
            bp, dsp = grad(xf), grad(xf[:k] + xb[k:])
            assert ref[k] == bp * bp
            assert diff[k] == (dsp - bp) ** 2
        assert diff[2] == 0  # the last block is not stale here
        assert (diff[0] != 0) == (b >= 1)  # batch 0 comes back before any block has made an update
        seen += 1
    assert seen == 5


def test_gradient_difference_vanishes_without_staleness_or_steps():
    """All-zero schedule: the DSP gradient is the BP gradient.  Zero step size: parameters never move."""
    for p, m, lr in (((0, 0, 0), (0, 0, 0), Fraction(1, 10)), ((1, 1, 0), (4, 2, 0), Fraction(0))):
        gd = O.GradientDifference(_scalar_pipeline(p, m, lr, Fraction(1, 2)))
        n = 0
        ticks = 5 if lr else 8  # exact rationals grow with every update
        for tau in range(ticks):
            _, out = gd.tick(Fraction(tau + 1, 3), Fraction(2))
            if out is not None:
                assert all(d == 0 for d in out[1]) and all(r != 0 for r in out[2])
                n += 1
        assert n == ticks - m[0]


def test_gradient_difference_on_cnn_blocks_matches_torch_autograd_bp():
    """The BP side on real layers: torch autograd through the whole network at the snapshot parameters."""
    cfg = get_config("tiny2")
    rng = np.random.default_rng(3)
    params = [perturb_affine(make_params(layers, rng), rng) for layers in cfg["blocks"]]
    orc = O.build_cnn_oracle(cfg, params)
    gd = O.GradientDifference(orc)
    batches, hist, fwd_tick, seen, stale_seen = [], [], {}, 0, False
    for tau in range(6):
        x, y = make_batch(rng, cfg["input"], cfg["classes"])
        batches.append((x, y))
        hist.append([[v.copy() for v in blk.param_list()] for blk in orc.blocks])
        rec, out = gd.tick(x, y)
        for k in range(cfg["K"]):
            if rec["fwd"][k] is not None:
                fwd_tick[(k, rec["fwd"][k])] = tau
        if out is None:
            continue
        b, diff, ref = out
        # the parameters each block held in the tick it forwarded batch b, taken from this test's own history
        frozen = [hist[fwd_tick[(k, b)]][k] for k in range(cfg["K"])]
        tot = _torch_bp_sumsq(cfg, params, frozen, *batches[b])
        for k in range(cfg["K"]):
            assert abs(tot[k] - ref[k]) <= 1e-9 * max(1.0, ref[k])
        assert diff[-1] <= 1e-20 * max(1.0, ref[-1])  # the last block of this schedule is not stale
        stale_seen = stale_seen or diff[0] > 1e-12 * ref[0]
        seen += 1
    assert seen >= 3 and stale_seen


# ----------------------------------------------------------------------------- update rule
def test_sum_constant_gradient_closed_form():
    """Heavy ball with a constant gradient g: x^n - x^{n+1} = alpha g (1 - beta^{n+1}) / (1 - beta)."""
    a, b, g = Fraction(1, 10), Fraction(9, 10), Fraction(3)
    opt, x = O.SUM([Fraction(0)], a, b), [Fraction(0)]
    for n in range(8):
        xn = opt.step(x, [g])
        assert x[0] - xn[0] == a * g * (1 - b ** (n + 1)) / (1 - b)
        x = xn


def test_sum_beta0_is_sgd_and_weight_decay():
    opt = O.SUM([Fraction(2)], Fraction(1, 4), 0)
    assert opt.step([Fraction(2)], [Fraction(3)]) == [Fraction(2) - Fraction(3, 4)]
    opt = O.SUM([Fraction(2), Fraction(2)], Fraction(1, 4), 0, wd=Fraction(1, 2), decay_mask=[True, False])
    assert opt.step([Fraction(2), Fraction(2)], [Fraction(3), Fraction(3)]) == [Fraction(1), Fraction(5, 4)]


@pytest.mark.parametrize("s", [0, 1])
def test_sum_appendix_recursion(s):
    """v^n = x^n - x^{n-1} + s alpha G^{n-1} obeys v^{n+1} = beta v^n + ((1-beta) s - 1) alpha G^n
    and z^n = x^n + beta/(1-beta) v^n moves by -alpha/(1-beta) G^n (appendix on momentum SGD)."""
    a, b = Fraction(1, 3), Fraction(3, 5)
    G = [Fraction(v) for v in (2, -1, 5, 3, -7, 4)]
    opt, xs = O.SUM([Fraction(1)], a, b, s=s), [Fraction(1)]
    for g in G:
        xs.append(opt.step([xs[-1]], [g])[0])
    v = [Fraction(0)] + [xs[n] - xs[n - 1] + s * a * G[n - 1] for n in range(1, len(xs))]
    for n in range(len(G)):
        assert v[n + 1] == b * v[n] + ((1 - b) * s - 1) * a * G[n]
        z0, z1 = xs[n] + b / (1 - b) * v[n], xs[n + 1] + b / (1 - b) * v[n + 1]
        assert z1 == z0 - a / (1 - b) * G[n]


def test_sum_matches_torch_sgd_momentum():
    rng = np.random.default_rng(0)
    x0 = rng.standard_normal(7)
    t = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    topt = torch.optim.SGD([t], lr=0.05, momentum=0.9)
    opt, x = O.SUM([x0.copy()], 0.05, 0.9), [x0.copy()]
    for _ in range(6):
        g = rng.standard_normal(7)
        t.grad = torch.tensor(g)
        topt.step()
        x = opt.step(x, [g])
        np.testing.assert_allclose(x[0], t.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_sum_s1_matches_torch_nesterov():
    """Eq. (3) with s = 1 is Nesterov's method; torch's SGD(nesterov=True) is the same iteration."""
    rng = np.random.default_rng(1)
    x0 = rng.standard_normal(7)
    t = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    topt = torch.optim.SGD([t], lr=0.05, momentum=0.9, nesterov=True)
    opt, x = O.SUM([x0.copy()], 0.05, 0.9, s=1), [x0.copy()]
    for _ in range(6):
        g = rng.standard_normal(7)
        t.grad = torch.tensor(g)
        topt.step()
        x = opt.step(x, [g])
        np.testing.assert_allclose(x[0], t.detach().numpy(), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("s", [0, 1])
def test_sum_step_size_change_keeps_the_iterate_difference(s):
    """Eq. (3) under a schedule: the momentum term is beta (y^{s,n+1} - y^{s,n}), a difference of iterates.
    With G^n = 0 the new step size cannot matter: x^{n+1} - x^n = beta (x^n - x^{n-1} + s alpha_{n-1} G^{n-1})."""
    a0, a1, b = Fraction(1, 3), Fraction(1, 30), Fraction(3, 5)
    G = [Fraction(v) for v in (2, -1, 5)]
    opt, xs = O.SUM([Fraction(1)], a0, b, s=s), [Fraction(1)]
    for g in G:
        xs.append(opt.step([xs[-1]], [g])[0])
    opt.alpha = a1
    xs.append(opt.step([xs[-1]], [Fraction(0)])[0])
    assert xs[-1] - xs[-2] == b * (xs[-2] - xs[-3] + s * a0 * G[-1])
    # and one more step with a gradient: the plain step uses the new alpha, the carried term the old iterates
    g = Fraction(7)
    x_next = opt.step([xs[-1]], [g])[0]
    assert x_next - xs[-1] == -a1 * g + b * (xs[-1] - xs[-2] - s * a1 * g)


# ----------------------------------------------------------------------------- layers
CONV_CASES = [(2, 3, 5, 6, 4, 3, 3, 1, 1), (2, 4, 7, 7, 3, 3, 3, 2, 1), (3, 5, 6, 6, 2, 1, 1, 2, 0),
              (1, 2, 9, 8, 3, 7, 7, 2, 3), (2, 3, 4, 4, 5, 1, 1, 1, 0)]


@pytest.mark.parametrize("N,C,H,W,K,R,S,st,pd", CONV_CASES)
def test_conv_matches_torch_and_adjoints(N, C, H, W, K, R, S, st, pd):
    rng = np.random.default_rng(1)
    x, w = rng.standard_normal((N, C, H, W)), rng.standard_normal((K, C, R, S))
    y = O.conv2d_forward(x, w, st, pd)
    yt = torch.nn.functional.conv2d(torch.tensor(x), torch.tensor(w), stride=st, padding=pd).numpy()
    np.testing.assert_allclose(y, yt, rtol=1e-12, atol=1e-12)
    g = rng.standard_normal(y.shape)
    dx = O.conv2d_backward_data(g, w, x.shape, st, pd)
    dw = O.conv2d_backward_weight(x, g, w.shape, st, pd)
    # <conv(x,w), g> = <x, dgrad(g,w)> = <w, wgrad(x,g)>   (the conv is bilinear)
    ip = float((y * g).sum())
    assert abs(ip - float((x * dx).sum())) < 1e-10 * max(1, abs(ip))
    assert abs(ip - float((w * dw).sum())) < 1e-10 * max(1, abs(ip))
    # adjointness must hold against *any* x', w' (pins dx and dw element-wise, not just one inner product)
    x2, w2 = rng.standard_normal(x.shape), rng.standard_normal(w.shape)
    assert abs(float((O.conv2d_forward(x2, w, st, pd) * g).sum()) - float((x2 * dx).sum())) < 1e-9
    assert abs(float((O.conv2d_forward(x, w2, st, pd) * g).sum()) - float((w2 * dw).sum())) < 1e-9


@pytest.mark.parametrize("N,C,H,W,K,R,S,st,pd,G", [(2, 8, 7, 6, 12, 3, 3, 1, 1, 4), (3, 6, 9, 9, 6, 3, 3, 2, 1, 2),
                                                   (2, 6, 5, 5, 6, 1, 1, 1, 0, 6), (1, 4, 8, 7, 8, 5, 5, 2, 2, 2)])
def test_grouped_conv_is_the_block_diagonal_dense_conv(N, C, H, W, K, R, S, st, pd, G):
    """A grouped convolution equals the dense one whose filter bank is zero outside the diagonal channel blocks; its
    two gradients are those of the dense problem (the filter gradient restricted to the blocks).  Also against
    torch's ``groups=`` and the adjoint identities with arbitrary second arguments."""
    rng = np.random.default_rng(40 + G)
    Ci, Co = C // G, K // G
    x, w = rng.standard_normal((N, C, H, W)), rng.standard_normal((K, Ci, R, S))
    dense = np.zeros((K, C, R, S))
    for g in range(G):
        dense[g * Co:(g + 1) * Co, g * Ci:(g + 1) * Ci] = w[g * Co:(g + 1) * Co]
    y = O.conv2d_forward(x, w, st, pd, G)
    np.testing.assert_allclose(y, O.conv2d_forward(x, dense, st, pd), rtol=1e-13, atol=1e-13)
    yt = torch.nn.functional.conv2d(torch.tensor(x), torch.tensor(w), stride=st, padding=pd, groups=G).numpy()
    np.testing.assert_allclose(y, yt, rtol=1e-12, atol=1e-12)
    gy = rng.standard_normal(y.shape)
    dx = O.conv2d_backward_data(gy, w, x.shape, st, pd, G)
    dw = O.conv2d_backward_weight(x, gy, w.shape, st, pd, G)
    np.testing.assert_allclose(dx, O.conv2d_backward_data(gy, dense, x.shape, st, pd), rtol=1e-12, atol=1e-12)
    dwd = O.conv2d_backward_weight(x, gy, dense.shape, st, pd)
    for g in range(G):
        np.testing.assert_allclose(dw[g * Co:(g + 1) * Co], dwd[g * Co:(g + 1) * Co, g * Ci:(g + 1) * Ci], rtol=1e-12, atol=1e-12)
    x2, w2 = rng.standard_normal(x.shape), rng.standard_normal(w.shape)
    assert abs(float((O.conv2d_forward(x2, w, st, pd, G) * gy).sum()) - float((x2 * dx).sum())) < 1e-9
    assert abs(float((O.conv2d_forward(x, w2, st, pd, G) * gy).sum()) - float((w2 * dw).sum())) < 1e-9


def test_conv_1x1_is_matmul_and_delta_is_shift():
    rng = np.random.default_rng(2)
    x, w = rng.standard_normal((2, 5, 4, 3)), rng.standard_normal((6, 5, 1, 1))
    y = O.conv2d_forward(x, w, 1, 0)
    np.testing.assert_allclose(y, np.einsum("nchw,kc->nkhw", x, w[:, :, 0, 0]), rtol=1e-13, atol=1e-13)
    d = np.zeros((1, 1, 3, 3))
    d[0, 0, 0, 2] = 1.0  # tap (r=0, s=2): y[h, w] = x[h-1, w+1]
    x = rng.standard_normal((1, 1, 5, 5))
    y = O.conv2d_forward(x, d, 1, 1)
    ref = np.zeros_like(x)
    ref[0, 0, 1:, :-1] = x[0, 0, :-1, 1:]
    np.testing.assert_array_equal(y, ref)


def test_bn_closed_forms():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((4, 3, 5, 5)) * 3 + 2
    eps = 1e-5
    y, mean, invstd = O.bn_forward(x, np.ones(3), np.zeros(3), eps)
    var = x.var(axis=(0, 2, 3))
    np.testing.assert_allclose(mean, x.mean(axis=(0, 2, 3)), rtol=1e-13)
    np.testing.assert_allclose(invstd, 1 / np.sqrt(var + eps), rtol=1e-13)
    np.testing.assert_allclose(y.mean(axis=(0, 2, 3)), 0, atol=1e-13)
    np.testing.assert_allclose(y.var(axis=(0, 2, 3)), var / (var + eps), rtol=1e-12)
    g, gamma = rng.standard_normal(x.shape), rng.standard_normal(3)
    dx, dg, db = O.bn_backward(g, x, gamma, mean, invstd)
    np.testing.assert_allclose(dx.sum(axis=(0, 2, 3)), 0, atol=1e-12)       # BN output ignores shifts of x
    # ... and scalings of x up to the eps term: sum dx*xhat = gamma*invstd*dgamma*(1 - var/(var+eps))
    np.testing.assert_allclose((dx * y).sum(axis=(0, 2, 3)), gamma * invstd * dg * eps * invstd ** 2,
                               rtol=1e-6, atol=1e-12)
    np.testing.assert_allclose(db, g.sum(axis=(0, 2, 3)), rtol=1e-13)
    xt = torch.tensor(x, requires_grad=True)
    gt = torch.tensor(gamma, requires_grad=True)
    bt = torch.zeros(3, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.batch_norm(xt, None, None, gt, bt, training=True, eps=eps)
    yt.backward(torch.tensor(g))
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dg, gt.grad.numpy(), rtol=1e-10)


def test_maxpool_matches_torch():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2, 3, 9, 10))
    y, arg = O.maxpool_forward(x, 3, 2, 1)
    xt = torch.tensor(x, requires_grad=True)
    yt = torch.nn.functional.max_pool2d(xt, 3, 2, 1)
    np.testing.assert_array_equal(y, yt.detach().numpy())
    g = rng.standard_normal(y.shape)
    yt.backward(torch.tensor(g))
    np.testing.assert_allclose(O.maxpool_backward(g, arg, x.shape), xt.grad.numpy(), rtol=0, atol=1e-15)


@pytest.mark.parametrize("C", [10, 100, 1000])
def test_softmax_ce_closed_forms(C):
    L = O.SoftmaxCE()
    labels = np.arange(6) % C
    loss, g = L.value_and_grad(np.zeros((6, C)), labels)
    assert abs(loss - np.log(C)) < 1e-12
    np.testing.assert_allclose(g.sum(axis=1), 0, atol=1e-15)
    z = np.random.default_rng(5).standard_normal((6, C)) * 30  # large logits: the max-shift matters
    loss, g = L.value_and_grad(z, labels)
    lt = torch.nn.functional.cross_entropy(torch.tensor(z), torch.tensor(labels, dtype=torch.long))
    assert abs(loss - float(lt)) < 1e-10 * max(1.0, abs(float(lt)))
    np.testing.assert_allclose(g.sum(axis=1), 0, atol=1e-13)


# ----------------------------------------------------------------------------- block VJP by finite differences
def _small_cfg(name, batch, hw):
    cfg = get_config(name, batch=batch, hw=hw)
    rng = np.random.default_rng(cfg["seed"])
    params = [perturb_affine(make_params(layers, rng), rng) for layers in cfg["blocks"]]
    return cfg, params, rng


def _block_in_shape(cfg, k):
    from workloads.configs import block_output_shape
    s = cfg["input"]
    for j in range(k):
        s = block_output_shape(cfg["blocks"][j], s)
    return s


@pytest.mark.parametrize("name,k,batch,hw", [("tiny2", 0, 2, 6), ("tiny2", 1, 2, 6), ("resnet20", 1, 2, 8),
                                             ("resnet18", 0, 2, 16), ("resnet50_conv4x", 0, 2, 4),
                                             ("resnet164", 1, 2, 8), ("vgg19", 1, 2, 32), ("resnext_tiny", 0, 2, 8),
                                             ("resnext_tiny", 1, 2, 8)])
def test_block_vjp_finite_differences(name, k, batch, hw):
    """Central differences in fp64 on s(x_k, h_k) = <f_k(h_k; x_k), G> for a fixed random G: this is
    exactly what lines 1-2 of Eq. (5) define.  Probes a few coordinates of every parameter tensor and of h_k."""
    cfg, params, rng = _small_cfg(name, batch, hw)
    if name == "resnet50_conv4x":  # shrink channels: same graph, FD-sized
        for L in cfg["blocks"][0]:
            for key in ("cin", "cout", "c"):
                if key in L:
                    L[key] //= 64
        cfg["input"] = (batch, 8, hw, hw)
        params = [perturb_affine(make_params(cfg["blocks"][0], rng), rng)]
    blk = O.CNNBlock(cfg["blocks"][k], params[k], first_block=False)
    h = rng.standard_normal(_block_in_shape(cfg, k))
    out, cache = blk.forward(h)
    G = rng.standard_normal(out.shape)
    g_h, g_x = blk.backward(cache, G)

    def s_of(hh, plist):
        blk.set_param_list(plist)
        return float((blk.forward(hh)[0] * G).sum())

    base = [a.copy() for a in blk.param_list()]
    eps, checked = 1e-6, 0
    for ti, (arr, ga) in enumerate(zip(base, g_x)):
        for _ in range(3):
            idx = tuple(rng.integers(0, d) for d in arr.shape)
            pp = [a.copy() for a in base]
            pm = [a.copy() for a in base]
            pp[ti][idx] += eps
            pm[ti][idx] -= eps
            fd = (s_of(h, pp) - s_of(h, pm)) / (2 * eps)
            assert abs(fd - ga[idx]) <= 2e-5 * max(1.0, abs(fd)), (ti, idx, fd, ga[idx])
            checked += 1
    for _ in range(6):
        idx = tuple(rng.integers(0, d) for d in h.shape)
        hp, hm = h.copy(), h.copy()
        hp[idx] += eps
        hm[idx] -= eps
        fd = (s_of(hp, base) - s_of(hm, base)) / (2 * eps)
        assert abs(fd - g_h[idx]) <= 2e-5 * max(1.0, abs(fd)), (idx, fd, g_h[idx])
    assert checked > 0


# ----------------------------------------------------------------------------- zero staleness == BP + SGD (torch autograd)
def _torch_net(cfg, params):
    """The same layer lists evaluated by torch's own ops (third-party check of the BP case)."""
    tp = [[{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in d.items()} for d in blk]
          for blk in params]
    F = torch.nn.functional

    def run(x, labels):
        h = x
        for layers, prm in zip(cfg["blocks"], tp):
            T = []
            src = lambda i: h if i == -1 else T[i]  # noqa: E731
            for L, p in zip(layers, prm):
                xin = src(L["in"])
                if L["op"] == "conv":
                    T.append(F.conv2d(xin, p["w"], stride=L["stride"], padding=L["pad"], groups=L.get("groups", 1)))
                elif L["op"] == "bn":
                    z = F.batch_norm(xin, None, None, p["gamma"], p["beta"], training=True, eps=1e-5)
                    if L["res"] is not None:
                        z = z + src(L["res"])
                    T.append(F.relu(z) if L["relu"] else z)
                elif L["op"] == "add":
                    T.append(xin + src(L["res"]))
                elif L["op"] == "maxpool":
                    T.append(F.max_pool2d(xin, L["k"], L["stride"], L["pad"]))
                elif L["op"] == "gap":
                    T.append(xin.mean(dim=(2, 3)))
                elif L["op"] == "linear":
                    T.append(xin @ p["w"].T + p["c"])
                elif L["op"] == "softmax_ce":
                    T.append(F.cross_entropy(xin, labels))
            h = T[-1]
        return h

    leaves = [t for blk in tp for d in blk for t in d.values()]
    return run, leaves, tp


def _torch_bp_sumsq(cfg, template, frozen, x, y):
    """Sum of squares of torch autograd's parameter gradients per block; frozen[k] = flat parameter list."""
    params = []
    for blk, flat in zip(template, frozen):
        it = iter(flat)
        params.append([{key: next(it) for key in d} for d in blk])
    run, leaves, tp = _torch_net(cfg, params)
    run(torch.tensor(x, dtype=torch.float64), torch.tensor(y, dtype=torch.long)).backward()
    return [sum(float((t.grad ** 2).sum()) for d in blk for t in d.values()) for blk in tp]


@pytest.mark.parametrize("name,batch,hw,loose", [("tiny2", 4, 8, 1), ("resnet20", 4, 8, 1), ("resnet18", 2, 64, 1),
                                                 # 164 layers amplify the fp64 rounding differences of two evaluation
                                                 # orders about a thousandfold more than 18 do (gradients still agree to 1e-4: no formula differs)
                                                 ("resnet164", 4, 16, 1000), ("vgg19", 2, 32, 1), ("resnext_tiny", 4, 8, 1)])
def test_zero_staleness_equals_backprop_sgd(name, batch, hw, loose):
    """Section 3.1 remark (a): with Delta t_k = 0 DSP is backpropagation; step for step against
    torch.autograd + torch.optim.SGD(momentum) in fp64 on the same net, data and initial parameters."""
    cfg, params, rng = _small_cfg(name, batch, hw)
    K = cfg["K"]
    orc = O.build_cnn_oracle(cfg, params, p=[0] * K, m=[0] * K)
    run, leaves, tp = _torch_net(cfg, params)
    topt = torch.optim.SGD(leaves, lr=cfg["lr"], momentum=cfg["beta"])
    for _ in range(4):
        x, y = make_batch(rng, cfg["input"], cfg["classes"])
        rec = orc.tick(x, y)
        topt.zero_grad()
        loss = run(torch.tensor(x, dtype=torch.float64), torch.tensor(y, dtype=torch.long))
        loss.backward()
        assert abs(rec["loss"] - loss.item()) < 1e-10 * loose * max(1.0, abs(loss.item()))
        for k in range(K):
            tg = [t.grad.numpy() for d in tp[k] for t in d.values()]
            for a, b in zip(rec["g_x"][k], tg):
                np.testing.assert_allclose(a, b, rtol=1e-7 * loose, atol=1e-9 * loose * max(1.0, float(np.abs(b).max())))
        topt.step()
        for k in range(K):
            for a, d in zip(orc.blocks[k].param_list(), [t for d in tp[k] for t in d.values()]):
                np.testing.assert_allclose(a, d.detach().numpy(), rtol=1e-7 * loose, atol=1e-9 * loose)


def test_lr0_dsp_gradient_equals_bp_gradient():
    """Section 3.2: Eq. (5) coincides with Eq. (4) when forward and backward parameters are equal.
    With alpha = 0 nothing ever changes, so every batch's DSP gradient is its BP gradient at x^0."""
    cfg, params, rng = _small_cfg("resnet20", 4, 8)
    K = cfg["K"]
    dsp = O.build_cnn_oracle(cfg, params, lr=0.0)
    bp = O.build_cnn_oracle(cfg, params, lr=0.0, p=[0] * K, m=[0] * K)
    got = {}
    ref = {}
    for n in range(8):
        x, y = make_batch(rng, cfg["input"], cfg["classes"])
        r1, r2 = dsp.tick(x, y), bp.tick(x, y)
        for k in range(K):
            if r1["bwd"][k] is not None:
                got[(k, r1["bwd"][k])] = r1["g_x"][k]
            ref[(k, r2["bwd"][k])] = r2["g_x"][k]
    assert len(got) >= 8
    for key, gx in got.items():
        for a, b in zip(gx, ref[key]):
            np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)


def test_dsp_differs_from_bp_and_uses_current_parameters():
    """With lr > 0 the recompute must use the block's current parameters on the stored input: check one
    backward of block 0 against a by-hand evaluation from the logged pieces."""
    cfg, params, rng = _small_cfg("tiny2", 4, 8)
    orc = O.build_cnn_oracle(cfg, params, lr=0.1)
    snaps = []
    for n in range(5):
        x, y = make_batch(rng, cfg["input"], cfg["classes"])
        before = [a.copy() for a in orc.blocks[0].param_list()]
        rec = orc.tick(x, y)
        snaps.append((before, rec))
    before, rec = snaps[3]  # tick 3: block 0 backward batch 1 after one update
    assert rec["bwd"][0] == 1 and rec["version"][0] == 1
    chk = O.CNNBlock(cfg["blocks"][0], params[0], first_block=True)
    chk.set_param_list(before)
    _, gx = chk.vjp(rec["h_in_bwd"][0], rec["g_out"][0])
    for a, b in zip(gx, rec["g_x"][0]):
        np.testing.assert_array_equal(a, b)
    chk0 = O.CNNBlock(cfg["blocks"][0], params[0], first_block=True)  # initial (forward-time) parameters
    _, gx0 = chk0.vjp(rec["h_in_bwd"][0], rec["g_out"][0])
    assert max(float(np.abs(a - b).max()) for a, b in zip(gx0, rec["g_x"][0])) > 1e-8


def test_round_bf16_matches_torch():
    """The storage-rounding helper of the oracle's bf16 comparison mode against torch's own conversion."""
    rng = np.random.default_rng(7)
    x = np.concatenate([rng.standard_normal(4096) * 10.0 ** rng.integers(-20, 20, 4096),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -2.5, 65504.0]])
    x = x.astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy().astype(np.float64)
    np.testing.assert_array_equal(O.round_bf16(x), ref)
    # ties go to the even mantissa: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6
    assert O.round_bf16(np.float32(1.00390625)) == 1.0 and O.round_bf16(np.float32(1.01171875)) == 1.015625


def test_bf16_storage_mode_is_close_to_fp64_and_idempotent():
    cfg, params, rng = _small_cfg("resnet20", 4, 8)
    h = O.round_bf16(rng.standard_normal(_block_in_shape(cfg, 1)))
    a = O.CNNBlock(cfg["blocks"][1], params[1], first_block=False)
    b = O.CNNBlock(cfg["blocks"][1], params[1], first_block=False, storage="bf16")
    ya, yb = a.forward(h)[0], b.forward(h)[0]
    assert np.array_equal(O.round_bf16(yb), yb)
    assert np.linalg.norm(ya - yb) / np.linalg.norm(ya) < 2e-2


def test_bf16_gradient_reproducibility_floor():
    """Why bf16 gradient parity through ReLU layers cannot be tight for ANY implementation: inside the
    oracle alone, moving 0.01% of a block's (bf16) inputs by one bf16 ulp changes G_h of an 18-ReLU
    bottleneck stage by more than 5%, while the forward output moves several times less.  (Rounding
    boundaries turn the ulp into ulp-sized changes of a growing share of the activations, and a fixed
    share of pre-activations near zero then takes the other ReLU branch.)"""
    cfg = get_config("resnet50_conv4x", batch=4, hw=14)
    for L in cfg["blocks"][0]:  # thinner, same depth: keeps the CPU test short
        for key in ("cin", "cout", "c"):
            if key in L:
                L[key] //= 8
    rng = np.random.default_rng(3)
    params = [make_params(cfg["blocks"][0], rng)]
    blk = O.CNNBlock(cfg["blocks"][0], params[0], first_block=False, storage="bf16")
    h = O.round_bf16(rng.standard_normal((4, 64, 14, 14)))
    out, _ = blk.forward(h)
    g = O.round_bf16(rng.standard_normal(out.shape) * 0.1)
    gh, _ = blk.vjp(h, g)
    h2 = h.copy().reshape(-1)
    idx = rng.choice(h2.size, size=max(1, h2.size // 10000), replace=False)
    h2[idx] *= 1 + 2.0 ** -8
    h2 = O.round_bf16(h2.reshape(h.shape))
    out2, _ = blk.forward(h2)
    gh2, _ = blk.vjp(h2, g)
    rel = lambda a, b: np.linalg.norm(a - b) / np.linalg.norm(b)  # noqa: E731
    assert rel(out2, out) < 3e-2
    assert rel(gh2, gh) > 5e-2 and rel(gh2, gh) > 3 * rel(out2, out)


@pytest.mark.parametrize("shape", [(2, 5, 9, 8, 4, 3, 3, 1, 1), (3, 4, 10, 10, 6, 3, 3, 2, 1), (2, 3, 12, 11, 5, 7, 7, 2, 3),
                                   (2, 6, 7, 7, 4, 1, 1, 2, 0), (2, 6, 7, 8, 9, 3, 3, 1, 1, 3), (2, 8, 9, 9, 4, 3, 3, 2, 1, 2)])
def test_single_element_convolutions_agree_with_the_full_ones(shape):
    """The per-element definitions used for full-size GPU parity are written independently (numpy slicing)
    of the C loops; on small problems every element of both must agree."""
    N, C, H, W, K, R, S, st, pd = shape[:9]
    G = shape[9] if len(shape) > 9 else 1
    rng = np.random.default_rng(11)
    x = rng.standard_normal((N, C, H, W))
    w = rng.standard_normal((K, C // G, R, S))
    y = O.conv2d_forward(x, w, st, pd, G)
    dy = rng.standard_normal(y.shape)
    dx = O.conv2d_backward_data(dy, w, x.shape, st, pd, G)
    dw = O.conv2d_backward_weight(x, dy, w.shape, st, pd, G)
    iy = [tuple(int(v) for v in np.unravel_index(i, y.shape)) for i in range(y.size)]
    ix = [tuple(int(v) for v in np.unravel_index(i, x.shape)) for i in range(x.size)]
    iw = [tuple(int(v) for v in np.unravel_index(i, w.shape)) for i in range(w.size)]
    np.testing.assert_allclose(O.conv2d_forward_at(x, w, st, pd, iy, G), y.ravel(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(O.conv2d_backward_data_at(dy, w, x.shape, st, pd, ix, G), dx.ravel(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(O.conv2d_backward_weight_at(x, dy, st, pd, iw, G), dw.ravel(), rtol=1e-11, atol=1e-11)


# ----------------------------------------------------------------------------- bf16 storage mode, decisions handed in
def _parse_kv(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            key, vals = line.split(":")
            out[key] = [Fraction(v) for v in vals.split()]
    return out


def test_bf16_storage_mode_worked_example():
    """Where the storage mode rounds is fixed by the library interface (what is bf16 in memory), not by any
    implementation; tests/golden/bf16_storage_worked_example.txt derives a conv -> BN + shortcut + ReLU block by hand
    in dyadic rationals, chosen so that dropping or moving any single rounding changes one of the values."""
    c = _parse_kv(os.path.join(os.path.dirname(__file__), "golden", "bf16_storage_worked_example.txt"))
    f = lambda v: np.array([float(x) for x in v])  # noqa: E731  (dyadic rationals: exact in fp64)
    layers = [dict(op="conv", **{"in": -1}, cin=1, cout=1, r=1, s=1, stride=1, pad=0),
              dict(op="bn", **{"in": 0}, c=1, relu=True, res=-1)]
    params = [{"w": f(c["w"]).reshape(1, 1, 1, 1)}, {"gamma": f(c["gamma"]), "beta": f(c["beta"])}]
    blk = O.CNNBlock(layers, params, first_block=False, eps=float(c["eps"][0]), storage="bf16")
    h = f(c["h"]).reshape(2, 1, 1, 1)
    out, cache = blk.forward(h)
    np.testing.assert_array_equal(out.ravel(), f(c["h_out"]))
    g_h, g_x = blk.backward(cache, f(c["g"]).reshape(2, 1, 1, 1))
    np.testing.assert_array_equal(g_h.ravel(), f(c["G_h"]))
    np.testing.assert_array_equal(g_x[0].ravel(), f(c["G_w"]))
    np.testing.assert_array_equal(g_x[1], f(c["G_gamma"]))
    np.testing.assert_array_equal(g_x[2], f(c["G_beta"]))
    # the same block without storage rounding gives other values everywhere (the example does exercise the roundings)
    ref = O.CNNBlock(layers, params, first_block=False, eps=float(c["eps"][0]))
    out64, cache64 = ref.forward(h)
    gh64, gx64 = ref.backward(cache64, f(c["g"]).reshape(2, 1, 1, 1))
    assert out64.ravel()[0] != out.ravel()[0] and gh64.ravel()[1] != g_h.ravel()[1] and gx64[0].ravel()[0] != g_x[0].ravel()[0]
    # the sum layer stores its result once
    add = O.CNNBlock([dict(op="add", **{"in": -1}, res=-1)], [{}], first_block=False, storage="bf16")
    a, b = float(c["add_a"][0]), float(c["add_b"][0])
    add.layers[0]["res"] = -1
    y, _ = add.forward(np.full((1, 1, 1, 1), (a + b) / 2))  # x + x with x = (a + b) / 2 is a + b exactly
    assert y.ravel()[0] == float(c["add_out"][0])


def test_decisions_handed_to_backward():
    """backward(decisions=...) applies the chain rule with another implementation's ReLU masks / pooling choices.
    Its own decisions handed back change nothing; a flipped decision changes exactly the path of that element and is
    reported with its margin; a max-pool choice moves the gradient to the chosen pixel."""
    rng = np.random.default_rng(5)
    layers = [dict(op="bn", **{"in": -1}, c=2, relu=True, res=None),
              dict(op="maxpool", **{"in": 0}, k=2, stride=2, pad=0)]
    params = [{"gamma": np.array([1.0, 2.0]), "beta": np.array([0.5, -0.25])}, {}]
    blk = O.CNNBlock(layers, params, first_block=False)
    h = rng.standard_normal((2, 2, 4, 4))
    out, cache = blk.forward(h)
    g = rng.standard_normal(out.shape)
    gh0, gx0 = blk.backward(cache, g)
    y, arg = cache[1][0], cache[2][1]
    own = {0: y > 0, 1: arg}
    gh1, gx1 = blk.backward(cache, g, decisions=own)
    np.testing.assert_array_equal(gh1, gh0)
    assert all(np.array_equal(a, b) for a, b in zip(gx1, gx0))
    assert blk.last_decision_report == [(1, 0, 0.0), (0, 0, 0.0)]
    # flip the mask of the element whose pre-activation is closest to zero
    mean, invstd = cache[2][0][0], cache[2][0][1]
    z = params[0]["gamma"].reshape(1, 2, 1, 1) * (h - mean.reshape(1, 2, 1, 1)) * invstd.reshape(1, 2, 1, 1) + params[0]["beta"].reshape(1, 2, 1, 1)
    idx = np.unravel_index(np.argmin(np.abs(z)), z.shape)
    mask = (y > 0).copy()
    mask[idx] = ~mask[idx]
    blk.backward(cache, g, decisions={0: mask})
    (layer, n, worst), = blk.last_decision_report
    cs = idx[1]
    mag = abs(params[0]["gamma"][cs] * invstd[cs]) * (abs(h[idx]) + abs(mean[cs])) + abs(params[0]["beta"][cs])
    assert layer == 0 and n == 1 and worst == pytest.approx(abs(z[idx]) / mag, rel=1e-12)
    # a masked-out output (all decisions "not positive") stops every gradient through the rectifier
    ghz, gxz = blk.backward(cache, g, decisions={0: np.zeros_like(mask)})
    assert not ghz.any() and not gxz[0].any() and not gxz[1].any()
    # pooling: route the first window's gradient to another pixel of the window
    theirs = arg.copy()
    a0 = int(arg[0, 0, 0, 0])
    other = [p for p in (0, 1, 4, 5) if p != a0][0]
    theirs[0, 0, 0, 0] = other
    blk2 = O.CNNBlock([dict(layers[1], **{"in": -1})], [{}], first_block=False)
    o2, c2 = blk2.forward(y)
    d_own, _ = blk2.backward(c2, g)
    d_th, _ = blk2.backward(c2, g, decisions={0: theirs})
    delta = d_th - d_own
    assert delta[0, 0].ravel()[other] == g[0, 0, 0, 0] and delta[0, 0].ravel()[a0] == -g[0, 0, 0, 0]
    assert np.count_nonzero(delta) == 2
    (layer, n, worst), = blk2.last_decision_report
    assert n == 1 and worst == pytest.approx(abs(y[0, 0].ravel()[a0] - y[0, 0].ravel()[other]) / abs(y[0, 0].ravel()[a0]), rel=1e-12)


# ----------------------------------------------------------------------------- trajectories: drift and stored files
def _run_losses(cfg, params, storage, ticks, seed_rng_state):
    rng = np.random.default_rng(0)
    rng.bit_generator.state = seed_rng_state
    orc = O.build_cnn_oracle(cfg, params, storage=storage)
    out = []
    for _ in range(ticks):
        x, y = make_batch(rng, cfg["input"], cfg["classes"])
        rec = orc.tick(x, y)
        if rec["loss"] is not None:
            out.append(rec["loss"])
    return np.array(out), orc


def _read_trajectory(fname):
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", fname)) if not l.startswith("#")]
    rows = [r for r in rows if int(r[1]) >= 0]
    return (np.array([float(r[2]) for r in rows]), np.array([float(r[3]) for r in rows]), np.array([float(r[4]) for r in rows]))


def test_trajectories_of_the_oracle_itself_drift_apart():
    """Why a free-running loss trajectory cannot be held to a fixed 1e-3 over the configured 50 ticks: the DSP
    recursion amplifies rounding-level differences (a rectifier that falls the other way changes the next parameters,
    hence every later decision).  tests/golden/trajectory_resnet20_fp32.txt holds, next to the oracle's losses on the
    full-size ResNet-20 workload, the distance of two more runs of THIS oracle that differ from the first only by
    rounding: every stored tensor rounded to fp32 (column 4), initial parameters moved by one fp32 ulp (column 5).
    Here the first ticks of the stored run and of the fp32-rounded run are recomputed (the file is the oracle's), and
    the stored distances are shown to grow from rounding level to beyond 1e-3; the GPU trajectory tests bound the
    library's distance from the oracle by a small multiple of these distances."""
    stored, gap_b, gap_c = _read_trajectory("trajectory_resnet20_fp32.txt")
    assert len(stored) == 48
    cfg = get_config("resnet20")
    rng = np.random.default_rng(cfg["seed"])
    params = [make_params(layers, rng) for layers in cfg["blocks"]]
    state = rng.bit_generator.state
    a, _ = _run_losses(cfg, params, None, 7, state)
    b, _ = _run_losses(cfg, params, "fp32", 7, state)
    np.testing.assert_allclose(a, stored[:5], rtol=1e-12)
    np.testing.assert_allclose(np.abs(b - a) / np.abs(a), gap_b[:5], rtol=0.05, atol=1e-11)
    # rounding level at first, three to four orders of magnitude more by the end of the configured steps
    assert max(gap_b[:4].max(), gap_c[:4].max()) < 1e-7
    assert gap_b[-10:].max() > 1e-3 and gap_c[-10:].max() > 1e-3
    # bf16 storage: two runs one fp32 ulp apart differ by ~1e-3 from the first loss on and by ~1e-2 later
    _, gb, gc = _read_trajectory("trajectory_resnet56_bf16.txt")
    assert max(gb[:5].max(), gc[:5].max()) > 5e-4 and max(gb.max(), gc.max()) > 5e-3


def test_fp32_storage_mode_rounds_like_numpy_single():
    x = np.array([1.0 + 2.0 ** -30, 1.0 + 2.0 ** -24, 1.0 + 3 * 2.0 ** -24, 1e-50, 3.0e38 * 1.2])
    np.testing.assert_array_equal(O.round_fp32(x), [1.0, 1.0, 1.0 + 2.0 ** -22, 0.0, np.inf])
