"""CPU oracle for Diversely Stale Parameters (DSP) -- TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 statement of what the DSP training step computes, written from the
paper; it shares no code with the HIP library and must never be imported by the product
path (only tests, the smoke check and the benchmark's CPU-baseline leg may use it).

What follows the paper, and where:

* Section 2, Eq. (1): the CNN is K consecutive blocks h_{k+1} = f_k(h_k; x_k), loss L(h_K, l).
  ``CNNBlock`` is one f_k (a list of textbook layers, arithmetic in ``layers.c``/numpy);
  ``SoftmaxCE`` is L.
* Section 2, Eq. (2): the chain rule per block -> ``CNNBlock.vjp``.
* Section 2, Eq. (3): stochastic unified momentum -> ``SUM`` (s = 0 heavy ball, s = 1 Nesterov).
* Lemma 1 / Section 5.4: DSP gradient against the BP gradient at forward-time parameters -> ``GradientDifference``.
* Section 3.1: layer-wise staleness = number of parameter updates between the forward and the
  backward use of a block's parameters for one mini-batch.
* Section 3.2, Eq. (5): the DSP gradient -- block k recomputes f_k on the input it *stored*
  (produced by the lower blocks' forward parameters) with its *current* (backward) parameters
  and applies the chain rule with the delayed error gradient.
* Section 3.3 and Appendix A: the batch pipeline -- block k owns FIFO queues M_k (inputs),
  P_k (outputs), Q_k (gradients) of lengths 1+m_k, 1+p_k, 1+q_k with
  q_k = m_{k-1} - p_{k-1} - m_k, q_0 = 0, p_{K-1} = 0.  ``DSPOracle`` moves real tagged items
  through real queues; it never computes a batch index in closed form.

Readings taken where the paper is silent (all listed in the design notes of the repository):
a queue of length 1+n releases its oldest item once it holds 1+n items, i.e. it delays by n
ticks; inside one tick a block runs forward(a), then recompute+backward(b) with the same
parameters, then its update; ticks in which no gradient has arrived make no update; the
last block may have m = 0 (the paper's own configurations do); all m = p = 0 is ordinary
backpropagation; every p = 0 with stale backward passes is the forward-locked schedule of the
features-replay comparison (Section 6); Q_k holds the gradients block k emits for block k-1; the
mini-batch loss is the mean over the batch; weight decay, if any, is added to the gradient of weight
tensors only; a grouped convolution (ResNeXt) is one ordinary convolution per group of channels.

Two modes beside plain fp64 serve the comparison with a kernel that stores tensors in a narrower
type: ``storage="bf16"`` / ``"fp32"`` round every stored feature map, gradient map and filter where
the C ABI says they are stored (arithmetic stays fp64), and ``CNNBlock.backward(decisions=...)``
applies the chain rule with given rectifier masks / pooling choices instead of its own (a branch
decision is an integer taken on a stored value; both sides must take it in the same precision).

Parity pins (tests/test_oracle_pins.py): exact rational worked examples (the DSP recursion; the bf16
storage mode with every rounding point written out), finite differences, adjoint identities,
grouped = block-diagonal dense convolution, torch's conv2d / autograd / SGD (also Nesterov) for the
zero-staleness case, closed forms for BN / softmax / momentum / the gradient difference, queue
timelines incl. the forward-locked tuples.  No function of this module is without a pin.  The loss
trajectory on the synthetic CNN workloads has no reference other than this oracle (parity unpinned
beyond its pins: the paper prints no numbers for synthetic data).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from collections import deque

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "layers.c")
_SO = os.path.join(_HERE, "_build", "liboracle_layers.so")
_lib_handle = None


def build(force=False):
    """Compiles layers.c with gcc (plain C, -O2, OpenMP on outer loops only)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_SO), exist_ok=True)
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _SO)
    return _SO


def _lib():
    global _lib_handle
    if _lib_handle is None:
        _lib_handle = ctypes.CDLL(build())
    return _lib_handle


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


# --------------------------------------------------------------------------- layers (fp64, NCHW)
def _per_group(groups, x_channels, w):
    """Channel ranges of a grouped convolution: group g maps input channels [g Ci, (g+1) Ci) to output channels
    [g Co, (g+1) Co) with the filters w[g Co : (g+1) Co] (shape Co_total x Ci x R x S)."""
    K, Ci = w.shape[0], w.shape[1]
    assert x_channels == Ci * groups and K % groups == 0, (x_channels, w.shape, groups)
    Co = K // groups
    return [(slice(g * Ci, (g + 1) * Ci), slice(g * Co, (g + 1) * Co)) for g in range(groups)]


def conv2d_forward(x, w, stride, pad, groups=1):
    x, w = _f64(x), _f64(w)
    if groups > 1:  # every group is an ordinary convolution of its own channel range
        return np.concatenate([conv2d_forward(x[:, ci], w[co], stride, pad) for ci, co in _per_group(groups, x.shape[1], w)], axis=1)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    y = np.empty((N, K, Ho, Wo))
    _lib().oracle_conv2d_forward(_p(x), _p(w), _p(y), N, C, H, W, K, R, S, stride, pad)
    return y


def conv2d_backward_data(dy, w, x_shape, stride, pad, groups=1):
    dy, w = _f64(dy), _f64(w)
    if groups > 1:
        N, C, H, W = x_shape
        return np.concatenate([conv2d_backward_data(dy[:, co], w[co], (N, C // groups, H, W), stride, pad)
                               for ci, co in _per_group(groups, C, w)], axis=1)
    N, C, H, W = x_shape
    K, _, R, S = w.shape
    dx = np.empty(x_shape)
    _lib().oracle_conv2d_backward_data(_p(dy), _p(w), _p(dx), N, C, H, W, K, R, S, stride, pad)
    return dx


def conv2d_backward_weight(x, dy, w_shape, stride, pad, groups=1):
    x, dy = _f64(x), _f64(dy)
    if groups > 1:
        K, Ci, R, S = w_shape
        rng = [(slice(g * Ci, (g + 1) * Ci), slice(g * (K // groups), (g + 1) * (K // groups))) for g in range(groups)]
        return np.concatenate([conv2d_backward_weight(x[:, ci], dy[:, co], (K // groups, Ci, R, S), stride, pad) for ci, co in rng], axis=0)
    N, C, H, W = x.shape
    K, _, R, S = w_shape
    dw = np.empty(w_shape)
    _lib().oracle_conv2d_backward_weight(_p(x), _p(dy), _p(dw), N, C, H, W, K, R, S, stride, pad)
    return dw


# ---- single output elements of the three convolutions, straight from the definition ------------------
# For parity checks at sizes where the full fp64 convolution would take minutes: each requested element
# is one sum over its receptive field (forward / backward-data) or over all output pixels
# (backward-weight), written independently of the C loops above.
def conv2d_forward_at(x, w, stride, pad, idx, groups=1):
    """y[n, k, ho, wo] for every (n, k, ho, wo) in idx; y = cross-correlation of x (NCHW) with w (KCRS); with groups,
    output channel k sees only the input channels of its group."""
    _, _, H, W = x.shape
    K, Ci, R, S = w.shape
    out = np.zeros(len(idx))
    for i, (n, k, ho, wo) in enumerate(idx):
        c0 = (k // (K // groups)) * Ci
        acc = 0.0
        for r in range(R):
            hi = ho * stride - pad + r
            if hi < 0 or hi >= H:
                continue
            for s in range(S):
                wi = wo * stride - pad + s
                if wi < 0 or wi >= W:
                    continue
                acc += float(np.dot(x[n, c0:c0 + Ci, hi, wi].astype(np.float64), w[k, :, r, s].astype(np.float64)))
        out[i] = acc
    return out


def conv2d_backward_data_at(dy, w, x_shape, stride, pad, idx, groups=1):
    """dx[n, c, hi, wi] for every (n, c, hi, wi) in idx: sum over the outputs (k, ho, wo) that x[n, c, hi, wi] fed
    (with groups: the output channels of the group of c)."""
    _, _, Ho, Wo = dy.shape
    K, Ci, R, S = w.shape
    Co = K // groups
    out = np.zeros(len(idx))
    for i, (n, c, hi, wi) in enumerate(idx):
        g, cl = c // Ci, c % Ci
        ks = slice(g * Co, (g + 1) * Co)
        acc = 0.0
        for r in range(R):
            th = hi + pad - r
            if th < 0 or th % stride or th // stride >= Ho:
                continue
            for s in range(S):
                tw = wi + pad - s
                if tw < 0 or tw % stride or tw // stride >= Wo:
                    continue
                acc += float(np.dot(dy[n, ks, th // stride, tw // stride].astype(np.float64), w[ks, cl, r, s].astype(np.float64)))
        out[i] = acc
    return out


def conv2d_backward_weight_at(x, dy, stride, pad, idx, groups=1):
    """dw[k, c, r, s] for every (k, c, r, s) in idx: sum over all (n, ho, wo) of dy[n, k, ho, wo] * x[n, c, hi, wi]
    (with groups, c counts inside the group of k: the input channel is (k // (K / groups)) * (C / groups) + c)."""
    _, C, H, W = x.shape
    _, K, Ho, Wo = dy.shape
    out = np.zeros(len(idx))
    for i, (k, c, r, s) in enumerate(idx):
        c = (k // (K // groups)) * (C // groups) + c
        # output pixels whose tap (r, s) falls inside the image
        ho = np.array([o for o in range(Ho) if 0 <= o * stride - pad + r < H], dtype=np.int64)
        wo = np.array([o for o in range(Wo) if 0 <= o * stride - pad + s < W], dtype=np.int64)
        if len(ho) == 0 or len(wo) == 0:
            continue
        xs = x[:, c][:, ho * stride - pad + r][:, :, wo * stride - pad + s].astype(np.float64)
        gs = dy[:, k][:, ho][:, :, wo].astype(np.float64)
        out[i] = float(np.sum(xs * gs))
    return out


def bn_forward(x, gamma, beta, eps):
    x, gamma, beta = _f64(x), _f64(gamma), _f64(beta)
    N, C, H, W = x.shape
    y, mean, invstd = np.empty_like(x), np.empty(C), np.empty(C)
    _lib().oracle_bn_forward(_p(x), _p(gamma), _p(beta), ctypes.c_double(eps), _p(y), _p(mean), _p(invstd),
                             N, C, H * W)
    return y, mean, invstd


def bn_backward(dy, x, gamma, mean, invstd):
    dy, x, gamma = _f64(dy), _f64(x), _f64(gamma)
    N, C, H, W = x.shape
    dx, dg, db = np.empty_like(x), np.empty(C), np.empty(C)
    _lib().oracle_bn_backward(_p(dy), _p(x), _p(gamma), _p(_f64(mean)), _p(_f64(invstd)), _p(dx), _p(dg),
                              _p(db), N, C, H * W)
    return dx, dg, db


def maxpool_forward(x, k, stride, pad):
    x = _f64(x)
    N, C, H, W = x.shape
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    y = np.empty((N, C, Ho, Wo))
    arg = np.empty((N, C, Ho, Wo), np.int32)
    _lib().oracle_maxpool_forward(_p(x), _p(y), _p(arg), N, C, H, W, k, stride, pad)
    return y, arg


def maxpool_backward(dy, arg, x_shape):
    dy = _f64(dy)
    N, C, H, W = x_shape
    dx = np.empty(x_shape)
    _lib().oracle_maxpool_backward(_p(dy), _p(arg), _p(dx), N, C, H, W, dy.shape[2], dy.shape[3])
    return dx


def round_bf16(a):
    """Nearest bfloat16 (8 exponent bits, 7 fraction bits; ties to even), returned as fp64."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    out = r.astype(np.uint32).view(np.float32).astype(np.float64)
    return np.where(np.isfinite(f), out, f.astype(np.float64)).reshape(np.shape(a))


def round_fp32(a):
    """Nearest IEEE single (ties to even), returned as fp64."""
    with np.errstate(over="ignore"):  # beyond the single range: infinity, as the format prescribes
        return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)


class SoftmaxCE:
    """L(h_K, l): mean over the mini-batch of -log softmax(h_K)[l]; returns (loss, dL/dh_K)."""

    def value_and_grad(self, z, labels):
        z = _f64(z)
        n = z.shape[0]
        zs = z - z.max(axis=1, keepdims=True)
        logp = zs - np.log(np.exp(zs).sum(axis=1, keepdims=True))
        loss = -logp[np.arange(n), labels].mean()
        g = np.exp(logp)
        g[np.arange(n), labels] -= 1.0
        return float(loss), g / n


# --------------------------------------------------------------------------- one block f_k
class CNNBlock:
    """f_k(h_k; x_k) for a layer list (see workloads.configs) and its VJP (Eq. (2)).

    ``params`` is a list (one entry per layer) of dicts of fp64 arrays: conv {"w"},
    bn {"gamma", "beta"}, linear {"w", "c"}.  A trailing ``softmax_ce`` layer is not part of
    f_k: it is the loss L and is handled by the pipeline.
    """

    def __init__(self, layers, params, first_block, eps=1e-5, storage=None):
        self.layers = [L for L in layers if L["op"] != "softmax_ce"]
        self.x = [{k: _f64(v).copy() for k, v in d.items()} for d in params[:len(self.layers)]]
        self.first_block = first_block  # no gradient w.r.t. the data h_0 is formed (q_0 = 0)
        self.eps = eps
        # storage = "bf16": every feature map, every error gradient of a feature map and the
        # conv filters are rounded to bfloat16 where a bf16 implementation stores them (the
        # arithmetic stays fp64; master parameters, weight gradients, BN statistics and the
        # pooled head stay unrounded).  A ReLU mask is an integer decision taken on a stored
        # value, so a comparison with a bf16 implementation is only meaningful if both sides
        # take it in the same precision.
        # storage = "fp32": the same roundings to single precision (what an fp32 implementation keeps in memory).
        assert storage in (None, "bf16", "fp32")
        self._rnd = {None: (lambda a: a), "bf16": round_bf16, "fp32": round_fp32}[storage]
        # Filled by backward() when it is handed the branch decisions of another implementation: per layer
        # (layer index, decisions that differ from this block's own, largest |margin| / magnitude among them).
        self.last_decision_report = []

    # -- parameters as one flat list of arrays (what the optimiser sees)
    def param_list(self):
        return [d[k] for d in self.x for k in d]

    def decay_mask(self):
        return [k == "w" for d in self.x for k in d]

    def set_param_list(self, new):
        it = iter(new)
        for d in self.x:
            for k in d:
                d[k] = next(it)

    def forward(self, h, params=None):
        """Returns (h_{k+1}, cache) with every intermediate tensor kept."""
        P = self.x if params is None else params
        rnd = self._rnd
        h = _f64(h)
        T, aux = [], []
        src = lambda i: h if i == -1 else T[i]  # noqa: E731
        for L, prm in zip(self.layers, P):
            x = src(L["in"])
            op = L["op"]
            if op == "conv":
                T.append(rnd(conv2d_forward(x, rnd(prm["w"]), L["stride"], L["pad"], L.get("groups", 1))))
                aux.append(None)
            elif op == "bn":
                z, mean, invstd = bn_forward(x, prm["gamma"], prm["beta"], self.eps)
                if L["res"] is not None:
                    z = z + src(L["res"])
                y = rnd(np.maximum(z, 0.0) if L["relu"] else z)
                T.append(y)
                aux.append((mean, invstd, y))
            elif op == "add":  # element-wise sum of two feature maps (the shortcut of a pre-activation unit)
                T.append(rnd(x + src(L["res"])))
                aux.append(None)
            elif op == "maxpool":
                y, arg = maxpool_forward(x, L["k"], L["stride"], L["pad"])
                T.append(y)
                aux.append(arg)
            elif op == "gap":
                T.append(x.mean(axis=(2, 3)))
                aux.append(None)
            elif op == "linear":
                T.append(x @ prm["w"].T + prm["c"])
                aux.append(None)
            else:
                raise ValueError(op)
        return T[-1], (h, T, aux)

    def backward(self, cache, g_out, params=None, decisions=None):
        """Chain rule through the cached forward: returns (G_{h_k} or None, G_{x_k} as a flat list).

        ``decisions`` (optional): {layer index: array}.  The backward pass of a rectifier and of a max pool
        rests on an integer decision taken on floating-point values (is the output positive; which window
        element is the largest).  Another implementation of the same definition may decide a near-tie the
        other way, after which the two gradients differ although both are correct.  To compare gradients, the
        decisions of that implementation can be handed in: for a bn layer with relu a boolean array
        (output > 0), for a max pool an integer array of source pixels (h * W + w per output element, -1 for
        none); the chain rule is then applied with THOSE decisions and ``last_decision_report`` lists, per
        such layer, how many differ from this block's own and the largest margin by which a differing
        decision contradicts this block's values, relative to the magnitude of the terms the value was
        formed from (the caller judges whether that is rounding noise).  Nothing else changes."""
        P = self.x if params is None else params
        h, T, aux = cache
        dT = [None] * len(T)
        dT[-1] = _f64(g_out)
        dh = [None]
        grads = [dict() for _ in self.layers]
        report = []

        def src(i):
            return h if i == -1 else T[i]

        rnd = self._rnd

        def add(i, v):  # gradients of feature maps are stored (hence rounded) after every contribution
            if i == -1:
                dh[0] = rnd(v if dh[0] is None else dh[0] + v)
            elif T[i].ndim == 4:
                dT[i] = rnd(v if dT[i] is None else dT[i] + v)
            else:
                dT[i] = v if dT[i] is None else dT[i] + v

        for i in reversed(range(len(self.layers))):
            L, prm, g = self.layers[i], P[i], dT[i]
            assert g is not None, "tensor %d has no consumer" % i
            x = src(L["in"])
            op = L["op"]
            if op == "conv":
                grads[i]["w"] = conv2d_backward_weight(x, g, prm["w"].shape, L["stride"], L["pad"], L.get("groups", 1))
                if not (L["in"] == -1 and self.first_block):
                    add(L["in"], conv2d_backward_data(g, rnd(prm["w"]), x.shape, L["stride"], L["pad"], L.get("groups", 1)))
            elif op == "bn":
                mean, invstd, y = aux[i]
                if L["relu"]:
                    own = y > 0.0  # ReLU'(0) = 0, decided on the stored output
                    mask = own
                    if decisions is not None and i in decisions:
                        mask = np.asarray(decisions[i], dtype=bool).reshape(y.shape)
                        diff = mask != own
                        worst = 0.0
                        if diff.any():
                            cs = (1, -1, 1, 1)
                            scale = (prm["gamma"] * invstd).reshape(cs)
                            z = scale * (x - mean.reshape(cs)) + prm["beta"].reshape(cs)
                            mag = np.abs(scale) * (np.abs(x) + np.abs(mean).reshape(cs)) + np.abs(prm["beta"]).reshape(cs)
                            if L["res"] is not None:
                                z = z + src(L["res"])
                                mag = mag + np.abs(src(L["res"]))
                            worst = float((np.abs(z[diff]) / (mag[diff] + 1e-300)).max())
                        report.append((i, int(diff.sum()), worst))
                    g = g * mask
                if L["res"] is not None:
                    add(L["res"], g)
                dx, dg, db = bn_backward(g, x, prm["gamma"], mean, invstd)
                grads[i]["gamma"], grads[i]["beta"] = dg, db
                add(L["in"], dx)
            elif op == "add":
                add(L["res"], g)
                add(L["in"], g)
            elif op == "maxpool":
                arg = aux[i]
                if decisions is not None and i in decisions:
                    theirs = np.ascontiguousarray(np.asarray(decisions[i]).reshape(arg.shape), dtype=np.int32)
                    diff = theirs != arg
                    worst = 0.0
                    if diff.any():
                        n_, c_ = np.nonzero(diff)[:2]
                        flat = x.reshape(x.shape[0], x.shape[1], -1)
                        best, chosen = flat[n_, c_, arg[diff]], flat[n_, c_, theirs[diff]]
                        worst = float((np.abs(best - chosen) / (np.abs(best) + 1e-300)).max())
                    report.append((i, int(diff.sum()), worst))
                    arg = theirs
                add(L["in"], maxpool_backward(g, arg, x.shape))
            elif op == "gap":
                hw = x.shape[2] * x.shape[3]
                add(L["in"], np.broadcast_to(g[:, :, None, None] / hw, x.shape).copy())
            elif op == "linear":
                grads[i]["w"] = g.T @ x
                grads[i]["c"] = g.sum(axis=0)
                add(L["in"], g @ prm["w"])
        self.last_decision_report = report
        flat = [grads[i][k] for i, d in enumerate(self.x) for k in d]
        return (None if self.first_block else dh[0]), flat

    def vjp(self, h, g_out, decisions=None):
        """Eq. (5), lines 1-2: recompute f_k on the stored input with the *current* parameters, then chain rule."""
        _, cache = self.forward(h)
        return self.backward(cache, g_out, decisions=decisions)


# --------------------------------------------------------------------------- Eq. (3)
class SUM:
    """Stochastic unified momentum, Eq. (3):

        y^{n+1}   = x^n - alpha G,     y^{s,n+1} = x^n - s alpha G,
        x^{n+1}   = y^{n+1} + beta (y^{s,n+1} - y^{s,n}),       y^{s,0} = x^0.

    s = 0 is heavy-ball momentum SGD (the optimiser of the paper's experiments), beta = 0 is SGD.
    ``alpha`` may be changed between steps (a learning-rate schedule): the recursion is applied as
    written, so the momentum term stays the difference of the stored iterates y^s.
    Works on any list of objects supporting + - * (numpy arrays, Fractions).
    """

    def __init__(self, x0, alpha, beta, s=0, wd=0, decay_mask=None):
        self.alpha, self.beta, self.s, self.wd = alpha, beta, s, wd
        self.ys = [v * 1 for v in x0]
        self.mask = decay_mask or [True] * len(x0)
        self.n_updates = 0
        self.last_step = None  # x^{n+1} - x^n of the latest update
        self.last_ys_step = None  # y^{s,n+1} - y^{s,n} of the latest update, and the alpha it was taken with
        self.last_alpha = None

    def step(self, x, G):
        new, step, ys_step = [], [], []
        for i, (xi, gi) in enumerate(zip(x, G)):
            if self.wd and self.mask[i]:
                gi = gi + self.wd * xi
            y = xi - self.alpha * gi
            ys = xi - self.s * self.alpha * gi
            xn = y + self.beta * (ys - self.ys[i])
            ys_step.append(ys - self.ys[i])
            self.ys[i] = ys
            new.append(xn)
            step.append(xn - xi)
        self.n_updates += 1
        self.last_step, self.last_ys_step, self.last_alpha = step, ys_step, self.alpha
        return new


# --------------------------------------------------------------------------- the batch pipeline
def queue_lengths(p, m):
    """Appendix A: q_0 = 0, q_k = m_{k-1} - p_{k-1} - m_k; validates the schedule.

    Accepted: (i) the all-zero schedule = ordinary backpropagation (Section 3.1, remark a);
    (ii) p_k > 0 for k < K-1, p_{K-1} = 0, m_k > 0 for k < K-1, m_{K-1} >= 0, q_k > 0 for k >= 1;
    (iii) every p_k = 0 with m_k > 0 for k < K-1 and q_k > 0: no output queue delays anything, so a mini-batch
    runs forward through all blocks within one tick (forward locking) while the backward passes stay stale --
    with m_k = K-1-k this is the schedule of the features-replay comparison of Section 6 (q_k = 1).
    """
    K = len(m)
    if len(p) != K:
        raise ValueError("p and m must have K entries each")
    if all(v == 0 for v in p) and all(v == 0 for v in m):
        return [0] * K
    if p[K - 1] != 0:
        raise ValueError("p_{K-1} must be 0")
    if any(v <= 0 for v in p[:K - 1]) and any(v != 0 for v in p):
        raise ValueError("p_k must be > 0 for k < K-1 (or every p_k = 0)")
    if any(v <= 0 for v in m[:K - 1]) or m[K - 1] < 0:
        raise ValueError("m_k must be > 0 for k < K-1 and >= 0 for the last block")
    q = [0] + [m[k - 1] - p[k - 1] - m[k] for k in range(1, K)]
    if any(v <= 0 for v in q[1:]):
        raise ValueError("q_k = m_{k-1} - p_{k-1} - m_k must be > 0")
    return q


class _Fifo:
    """A FIFO queue of fixed length: once it holds ``length`` items, pop() hands out the oldest."""

    def __init__(self, length):
        self.length = length
        self.items = deque()

    def push(self, item):
        assert len(self.items) < self.length, "queue overflow"
        self.items.append(item)

    def full(self):
        return len(self.items) == self.length

    def pop(self):
        return self.items.popleft()


class DSPOracle:
    """DSP(p_0..p_{K-1}; m_0..m_{K-1}) over K blocks, one ``tick`` per fresh mini-batch.

    ``blocks[k]`` must offer forward(h) -> (h_next, cache), vjp(h, g) -> (g_h, [g_x...]),
    param_list(), set_param_list(list), decay_mask(); ``loss`` offers
    value_and_grad(h_K, label) -> (value, G_{h_K}).
    """

    def __init__(self, blocks, loss, p, m, lr, beta, wd=0, s=0, external_gradient=False):
        self.blocks, self.loss = blocks, loss
        self.K = K = len(blocks)
        self.p, self.m = list(p), list(m)
        self.q = queue_lengths(self.p, self.m)
        self.M = [_Fifo(1 + self.m[k]) for k in range(K)]
        self.P = [_Fifo(1 + self.p[k]) for k in range(K)]
        self.Q = [_Fifo(1 + self.q[k]) for k in range(K)]
        # error gradient at the top of the last block, held until that block's backward (delay m_{K-1})
        self.QK = _Fifo(1 + self.m[K - 1])
        self.opt = [SUM(b.param_list(), lr, beta, s=s, wd=wd, decay_mask=b.decay_mask()) for b in blocks]
        self.external_gradient = external_gradient
        self.tau = 0
        self.log = []  # one dict per tick: what every block did

    def tick(self, h0, label, top_gradient=None):
        """Feeds mini-batch number ``tau``; returns this tick's record.

        ``top_gradient(batch_id, h_K)`` supplies G_{h_K} when the pipeline is a lone block fed
        with an external error gradient instead of a loss.
        """
        K, tau = self.K, self.tau
        rec = {"tau": tau, "fwd": [None] * K, "bwd": [None] * K, "version": [o.n_updates for o in self.opt],
               "loss": None, "loss_batch": None, "out": [None] * K, "g_in": [None] * K, "g_x": [None] * K,
               "h_in_fwd": [None] * K, "h_in_bwd": [None] * K, "g_out": [None] * K}
        pending = [None] * K

        # forward: the data source feeds block 0; block k>0 takes what P_{k-1} releases
        for k in range(K):
            if k == 0:
                item = (tau, h0, label)
            elif self.P[k - 1].full():
                item = self.P[k - 1].pop()
            else:
                continue
            a, h, lab = item
            self.M[k].push(item)
            out, _ = self.blocks[k].forward(h)
            rec["fwd"][k], rec["h_in_fwd"][k], rec["out"][k] = a, h, out
            if k < K - 1:
                self.P[k].push((a, out, lab))
            else:
                if self.external_gradient:
                    g = top_gradient(a, out)
                else:
                    val, g = self.loss.value_and_grad(out, lab)
                    rec["loss"], rec["loss_batch"] = val, a
                self.QK.push((a, g))

        # recompute + backward: the stored input and the delayed error gradient must carry the same tag
        for k in reversed(range(K)):
            if not self.M[k].full():
                continue
            gq = self.QK if k == K - 1 else self.Q[k + 1]
            if not gq.full():
                continue
            b, h, _ = self.M[k].pop()
            bg, g = gq.pop()
            assert b == bg, "block %d: stored input of batch %d met the gradient of batch %d" % (k, b, bg)
            g_h, g_x = self.blocks[k].vjp(h, g)  # same parameters as this tick's forward
            rec["bwd"][k], rec["h_in_bwd"][k], rec["g_out"][k] = b, h, g
            rec["g_in"][k], rec["g_x"][k] = g_h, g_x
            if k > 0:
                self.Q[k].push((b, g_h))
            pending[k] = g_x

        # update last: x_k <- SUM(x_k, G_{x_k})
        for k in range(K):
            if pending[k] is not None:
                self.blocks[k].set_param_list(self.opt[k].step(self.blocks[k].param_list(), pending[k]))
        self.tau += 1
        self.log.append({k: rec[k] for k in ("tau", "fwd", "bwd", "version", "loss", "loss_batch")})
        return rec


# --------------------------------------------------------------------------- Lemma 1 / Section 5.4
def _sumsq(v):
    return (v * v).sum() if hasattr(v, "sum") else v * v


class GradientDifference:
    """The two gradients Lemma 1 compares, per block and mini-batch (the quantity of Section 5.4).

    For mini-batch b let x_i^{fwd(b)} be block i's parameters when it ran the forward pass of b.
    * BP gradient: nabla_{x_k} L(F(h_0(b); x_0^{fwd(b)}, ..., x_{K-1}^{fwd(b)}), label(b)), i.e. ordinary
      backpropagation of batch b through the network frozen at those parameters;
    * DSP gradient: the G_{x_k} block k formed for b (Eq. (5)), with the parameters of its backward tick.
    ``tick`` drives the wrapped pipeline and, once block 0 (the last to finish a batch) has formed its
    gradient of batch b, returns (b, [||DSP_k - BP_k||^2], [||BP_k||^2]) as exact sums of squares.
    """

    def __init__(self, orc):
        assert not orc.external_gradient
        self.orc = orc
        K = orc.K
        self.snap = [dict() for _ in range(K)]          # batch -> parameters block k forwarded it with
        self.data = {}                                  # batch -> (h_0, label)
        self.dsp = [dict() for _ in range(K)]           # batch -> G_{x_k}

    def bp_gradient(self, b):
        """Backpropagation of batch b through the blocks frozen at their forward-time parameters."""
        orc, K = self.orc, self.orc.K
        live = [blk.param_list() for blk in orc.blocks]
        try:
            for k in range(K):
                orc.blocks[k].set_param_list(self.snap[k][b])
            h, lab = self.data[b]
            hs = []
            for k in range(K):
                hs.append(h)
                h, _ = orc.blocks[k].forward(h)
            _, g = orc.loss.value_and_grad(h, lab)
            grads = [None] * K
            for k in reversed(range(K)):
                g, grads[k] = orc.blocks[k].vjp(hs[k], g)
        finally:
            for k in range(K):
                orc.blocks[k].set_param_list(live[k])
        return grads

    def tick(self, h0, label):
        orc, K, tau = self.orc, self.orc.K, self.orc.tau
        self.data[tau] = (h0, label)
        before = [[v * 1 for v in blk.param_list()] for blk in orc.blocks]  # a tick's update comes last
        rec = orc.tick(h0, label)
        for k in range(K):
            if rec["fwd"][k] is not None:
                self.snap[k][rec["fwd"][k]] = before[k]
            if rec["bwd"][k] is not None:
                self.dsp[k][rec["bwd"][k]] = rec["g_x"][k]
        b = rec["bwd"][0]
        if b is None:
            return rec, None
        bp = self.bp_gradient(b)
        diff = [sum(_sumsq(d - r) for d, r in zip(self.dsp[k].pop(b), bp[k])) for k in range(K)]
        ref = [sum(_sumsq(r) for r in bp[k]) for k in range(K)]
        self.last_frozen = [self.snap[k].pop(b) for k in range(K)]  # kept for inspection
        del self.data[b]
        return rec, (b, diff, ref)


def build_cnn_oracle(cfg, params_per_block, lr=None, beta=None, wd=None, p=None, m=None, eps=1e-5, storage=None):
    """A DSPOracle over the CNN blocks of a workload config (see workloads.configs)."""
    blocks = [CNNBlock(layers, prm, first_block=(k == 0 and cfg.get("data_input", True)), eps=eps,
                       storage=storage)
              for k, (layers, prm) in enumerate(zip(cfg["blocks"], params_per_block))]
    ext = cfg.get("classes") is None
    return DSPOracle(blocks, SoftmaxCE(), cfg["p"] if p is None else p, cfg["m"] if m is None else m,
                     cfg["lr"] if lr is None else lr, cfg["beta"] if beta is None else beta,
                     wd=cfg["wd"] if wd is None else wd, external_gradient=ext)
