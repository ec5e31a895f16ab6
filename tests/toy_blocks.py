"""Scalar blocks in exact rationals for the worked example of the DSP pipeline (test helper)."""
from fractions import Fraction


class ScalarBlock:
    """f(h; x) = x^power * h with one scalar parameter."""

    def __init__(self, x0, power):
        self.x, self.power = [Fraction(x0)], power

    def param_list(self):
        return list(self.x)

    def set_param_list(self, new):
        self.x = list(new)

    def decay_mask(self):
        return [True]

    def forward(self, h):
        return self.x[0] ** self.power * h, None

    def vjp(self, h, g):
        x = self.x[0]
        return x ** self.power * g, [self.power * x ** (self.power - 1) * h * g]


class HalfSquare:
    """L(h, l) = (h - l)^2 / 2."""

    def value_and_grad(self, h, l):
        return (h - l) ** 2 / 2, h - l


class CountingBlock:
    """Carries integers only: records which parameter version touched which batch."""

    def __init__(self):
        self.version = 0
        self.fwd_version = {}
        self.bwd_version = {}

    def param_list(self):
        return [self.version]

    def set_param_list(self, new):
        self.version += 1

    def decay_mask(self):
        return [False]

    def forward(self, h):
        self.fwd_version[h] = self.version
        return h, None

    def vjp(self, h, g):
        assert h == g, "stored input and error gradient come from different batches"
        self.bwd_version[h] = self.version
        return g, [0]


class BatchIdLoss:
    def value_and_grad(self, h, l):
        assert h == l
        return h, h
