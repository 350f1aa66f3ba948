"""Pins of the RMSNorm + JVP oracle against things other than itself: a library routine for the primal, library
forward-mode differentiation, finite differences, closed forms and invariants; and planted mistakes that each
pin set must catch."""
import numpy as np
import pytest
import torch

from oracle.rmsnorm_jvp_ref import rmsnorm_jvp_ref


def data(seed, rows=7, d=16):
    g = np.random.default_rng(seed)
    return g.normal(size=(rows, d)) * 1.7, g.normal(size=(rows, d)), g.normal(size=d) + 1.0


PINS = []


def pin(f):
    PINS.append(f)
    return f


@pin
def pin_primal_library(fn):
    x, tx, w = data(1)
    y, _ = fn(x, tx, w, 1e-5)
    lib = torch.nn.functional.rms_norm(torch.from_numpy(x), (x.shape[-1],), torch.from_numpy(w), 1e-5).numpy()
    np.testing.assert_allclose(y, lib, rtol=1e-12, atol=1e-13)


@pin
def pin_forward_mode_library(fn):
    x, tx, w = data(2)
    eps = 1e-3
    f = lambda z: z * torch.rsqrt(z.pow(2).mean(-1, keepdim=True) + eps) * torch.from_numpy(w)
    y_l, ty_l = torch.func.jvp(f, (torch.from_numpy(x),), (torch.from_numpy(tx),))
    y, ty = fn(x, tx, w, eps)
    np.testing.assert_allclose(y, y_l.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ty, ty_l.numpy(), rtol=1e-11, atol=1e-12)


@pin
def pin_finite_differences(fn):
    x, tx, w = data(3)
    eps, h = 0.05, 1e-6
    yp, _ = fn(x + h * tx, tx, w, eps)
    ym, _ = fn(x - h * tx, tx, w, eps)
    _, ty = fn(x, tx, w, eps)
    np.testing.assert_allclose(ty, (yp - ym) / (2 * h), rtol=2e-8, atol=2e-9)


@pin
def pin_scale_invariance(fn):
    """With eps = 0 the output does not change along x itself: tx = x gives ty = 0."""
    x, _, w = data(4)
    _, ty = fn(x, x, w, 0.0)
    assert np.abs(ty).max() < 1e-14


@pin
def pin_tangent_orthogonal_to_normalised_row(fn):
    """With eps = 0, |x r|^2 = d for every x, so (y/w) . (ty/w) = 0."""
    x, tx, w = data(5)
    y, ty = fn(x, tx, w, 0.0)
    np.testing.assert_allclose(((y / w) * (ty / w)).sum(-1), 0.0, atol=1e-12)
    np.testing.assert_allclose(((y / w) ** 2).mean(-1), 1.0, rtol=1e-13)


@pin
def pin_linearity_in_tangent(fn):
    x, t1, w = data(6)
    _, t2, _ = data(7)
    a, b = 0.3, -1.9
    _, ty1 = fn(x, t1, w, 1e-2)
    _, ty2 = fn(x, t2, w, 1e-2)
    _, ty = fn(x, a * t1 + b * t2, w, 1e-2)
    np.testing.assert_allclose(ty, a * ty1 + b * ty2, rtol=1e-12, atol=1e-13)


@pin
def pin_scalar_closed_form(fn):
    """d = 1: y = w x / sqrt(x^2 + eps), dy/dx = w eps / (x^2 + eps)^(3/2)."""
    x = np.array([[0.7], [-2.0], [1e-3]]); tx = np.array([[1.3], [0.4], [-2.0]]); w = np.array([1.5]); eps = 0.25
    y, ty = fn(x, tx, w, eps)
    np.testing.assert_allclose(y, w * x / np.sqrt(x * x + eps), rtol=1e-14)
    np.testing.assert_allclose(ty, w * tx * eps / (x * x + eps) ** 1.5, rtol=1e-13)


@pin
def pin_large_eps_limit(fn):
    """eps >> mean(x^2): r -> eps^-1/2, the layer becomes the linear map x w / sqrt(eps)."""
    x, tx, w = data(8)
    eps = 1e12
    y, ty = fn(x, tx, w, eps)
    np.testing.assert_allclose(y, x * w / np.sqrt(eps), rtol=1e-10)
    np.testing.assert_allclose(ty, tx * w / np.sqrt(eps), rtol=1e-10)


@pytest.mark.parametrize("p", PINS, ids=lambda f: f.__name__)
def test_pin(p):
    p(rmsnorm_jvp_ref)


def _mutant(kind):
    def fn(x, tx, w, eps):
        x, tx, w = np.asarray(x, float), np.asarray(tx, float), np.asarray(w, float)
        ms = np.mean(x * x, -1, keepdims=True)
        if kind == "sum_not_mean":
            ms = np.sum(x * x, -1, keepdims=True)
        r = 1 / np.sqrt(ms + eps)
        if kind == "eps_outside":
            r = 1 / (np.sqrt(ms) + eps)
        xt = np.mean(x * tx, -1, keepdims=True)
        if kind == "xt_sum":
            xt = np.sum(x * tx, -1, keepdims=True)
        power = 2 if kind == "r_squared" else 3
        second = x * r ** power * xt
        if kind == "sign":
            second = -second
        if kind == "dropped_term":
            second = 0 * second
        ty = tx * r - second
        y = x * r * w
        ty = ty * (1.0 if kind == "tangent_without_gain" else w)
        if kind == "gain_inside_mean":
            y = (x * w) / np.sqrt(np.mean((x * w) ** 2, -1, keepdims=True) + eps)
        return y, ty
    return fn


@pytest.mark.parametrize("kind", ["sum_not_mean", "eps_outside", "xt_sum", "r_squared", "sign", "dropped_term",
                                  "tangent_without_gain", "gain_inside_mean"])
def test_planted_mistake_is_caught(kind):
    caught = 0
    for p in PINS:
        try:
            p(_mutant(kind))
        except AssertionError:
            caught += 1
    assert caught >= 1, f"no pin notices the mistake '{kind}'"


def test_mutant_harness_passes_the_unmutated_formula():
    for p in PINS:
        p(_mutant("none"))
