"""Pins for the fp64 oracle: what the mathematics fixes, checked without the oracle's own formula.

Each pin is a function of an implementation `impl(q,k,v,tq,tk,tv,scale) -> (o,to,lse)` on one
head, so the same pins can be turned on deliberately broken variants (test_pins_catch_mutants)
to show that a dropped term, a wrong sign, a missing scale or swapped operands fails at least one.
Library routines used as independent references: scipy.special.softmax / logsumexp and
torch.func.jvp over torch's own softmax attention (forward-mode AD, the paper's fallback, Sec. 3.2).
"""
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle.attn_jvp_ref import attn_jvp_ref, attn_jvp_ref_head
from oracle.alg2_stream import alg2_head


def rand_head(seed, Lq, Lkv, d, tangent_std=1.0):
    rng = np.random.default_rng(seed)
    q, tq = rng.standard_normal((Lq, d)), tangent_std * rng.standard_normal((Lq, d))
    k, tk = rng.standard_normal((Lkv, d)), tangent_std * rng.standard_normal((Lkv, d))
    v, tv = rng.standard_normal((Lkv, d)), tangent_std * rng.standard_normal((Lkv, d))
    return q, k, v, tq, tk, tv


def primal_lib(q, k, v, scale):
    """O and lse from library routines only."""
    s = scale * (q @ k.T)
    return scipy.special.softmax(s, axis=1) @ v, scipy.special.logsumexp(s, axis=1)


# ---------------------------------------------------------------- pins (each takes impl)

def pin_primal_library(impl):
    q, k, v, tq, tk, tv = rand_head(1, 7, 11, 5)
    o, _, lse = impl(q, k, v, tq, tk, tv, 0.37)
    o_ref, lse_ref = primal_lib(q, k, v, 0.37)
    np.testing.assert_allclose(o, o_ref, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, lse_ref, rtol=0, atol=1e-13)


def pin_finite_differences(impl):
    """tO is the directional derivative of O: central differences of the library primal."""
    for seed, (Lq, Lkv, d) in enumerate([(5, 9, 4), (16, 16, 8), (3, 33, 6)]):
        q, k, v, tq, tk, tv = rand_head(10 + seed, Lq, Lkv, d)
        scale = 1.0 / math.sqrt(d)
        _, to, _ = impl(q, k, v, tq, tk, tv, scale)
        eps = 1e-6
        op, _ = primal_lib(q + eps * tq, k + eps * tk, v + eps * tv, scale)
        om, _ = primal_lib(q - eps * tq, k - eps * tk, v - eps * tv, scale)
        fd = (op - om) / (2 * eps)
        np.testing.assert_allclose(to, fd, rtol=0, atol=2e-8 * max(1.0, np.abs(fd).max()))


def pin_torch_forward_ad(impl):
    q, k, v, tq, tk, tv = rand_head(20, 12, 19, 8)
    scale = 0.25

    def attn(q_, k_, v_):
        return torch.softmax(scale * q_ @ k_.T, dim=-1) @ v_

    prim = tuple(torch.from_numpy(x) for x in (q, k, v))
    tang = tuple(torch.from_numpy(x) for x in (tq, tk, tv))
    o_t, to_t = torch.func.jvp(attn, prim, tang)
    o, to, _ = impl(q, k, v, tq, tk, tv, scale)
    np.testing.assert_allclose(o, o_t.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(to, to_t.numpy(), rtol=0, atol=1e-12)


def pin_zero_tangent(impl):
    q, k, v, *_ = rand_head(30, 6, 10, 4)
    z = np.zeros_like
    _, to, _ = impl(q, k, v, z(q), z(k), z(v), 0.5)
    assert np.all(to == 0.0)


def pin_linearity(impl):
    q, k, v, tq1, tk1, tv1 = rand_head(40, 6, 10, 4)
    _, _, _, tq2, tk2, tv2 = rand_head(41, 6, 10, 4)
    a, b = 1.7, -0.3
    _, t1, _ = impl(q, k, v, tq1, tk1, tv1, 0.5)
    _, t2, _ = impl(q, k, v, tq2, tk2, tv2, 0.5)
    _, t12, _ = impl(q, k, v, a * tq1 + b * tq2, a * tk1 + b * tk2, a * tv1 + b * tv2, 0.5)
    np.testing.assert_allclose(t12, a * t1 + b * t2, rtol=0, atol=1e-13)


def pin_value_tangent_is_output(impl):
    """O is linear in V: tV = V with tQ = tK = 0 gives tO = O."""
    q, k, v, *_ = rand_head(50, 6, 10, 4)
    o, to, _ = impl(q, k, v, np.zeros_like(q), np.zeros_like(k), v, 0.5)
    np.testing.assert_allclose(to, o, rtol=0, atol=1e-14)


def pin_temperature_derivative(impl):
    """tQ = Q, tK = tV = 0 makes tS = S, so tO = scale * dO/dscale (FD of the library primal)."""
    q, k, v, *_ = rand_head(60, 6, 10, 4)
    scale = 0.4
    _, to, _ = impl(q, k, v, q, np.zeros_like(k), np.zeros_like(v), scale)
    h = 1e-6
    fd = (primal_lib(q, k, v, scale + h)[0] - primal_lib(q, k, v, scale - h)[0]) / (2 * h)
    np.testing.assert_allclose(to, scale * fd, rtol=0, atol=1e-8)
    # same statement through K: tK = K
    _, to_k, _ = impl(q, k, v, np.zeros_like(q), k, np.zeros_like(v), scale)
    np.testing.assert_allclose(to_k, scale * fd, rtol=0, atol=1e-8)


def pin_row_constant_ts(impl):
    """The same vector u added to every key shifts each score row by a constant: softmax, O unchanged."""
    q, k, v, *_ = rand_head(70, 6, 10, 4)
    u = np.random.default_rng(71).standard_normal(4)
    tk = np.tile(u, (10, 1))
    _, to, _ = impl(q, k, v, np.zeros_like(q), tk, np.zeros_like(v), 0.5)
    np.testing.assert_allclose(to, 0.0, rtol=0, atol=1e-13)


def pin_ones_value(impl):
    """V = 1 gives O = 1 whatever the scores are, so only the P tV term survives."""
    q, k, _, tq, tk, tv = rand_head(80, 6, 10, 4)
    v = np.ones((10, 4))
    o, to, _ = impl(q, k, v, tq, tk, tv, 0.5)
    np.testing.assert_allclose(o, 1.0, rtol=0, atol=1e-14)
    p = scipy.special.softmax(0.5 * q @ k.T, axis=1)
    np.testing.assert_allclose(to, p @ tv, rtol=0, atol=1e-13)


def pin_uniform_and_single_key(impl):
    q, _, v, tq, tk, tv = rand_head(90, 5, 8, 3)
    k = np.zeros((8, 3))
    scale = 0.6
    o, to, lse = impl(q, k, v, tq, tk, tv, scale)
    np.testing.assert_allclose(o, np.tile(v.mean(0), (5, 1)), rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse, math.log(8.0), rtol=0, atol=1e-14)
    ts = scale * q @ tk.T                       # tQ K^T vanishes with K = 0
    cov = (ts - ts.mean(1, keepdims=True)) @ v / 8.0
    np.testing.assert_allclose(to, cov + tv.mean(0), rtol=0, atol=1e-13)
    # a single key: softmax is 1, O = V_0 and tO = tV_0 whatever tQ, tK are
    q, k, v, tq, tk, tv = rand_head(91, 5, 1, 3)
    o, to, lse = impl(q, k, v, tq, tk, tv, scale)
    np.testing.assert_allclose(o, np.tile(v[0], (5, 1)), rtol=0, atol=0)
    np.testing.assert_allclose(to, np.tile(tv[0], (5, 1)), rtol=0, atol=1e-15)
    np.testing.assert_allclose(lse, scale * q @ k[0], rtol=0, atol=1e-14)


def pin_two_key_logistic(impl):
    """Two keys, d = 1: O = sigma(z) v1 + (1 - sigma(z)) v2 with z = scale q (k1 - k2); differentiate by hand."""
    qv, k1, k2, v1, v2 = 0.7, 1.3, -0.4, 2.0, -1.0
    tqv, tk1, tk2, tv1, tv2 = 0.5, -0.2, 0.9, 0.3, -0.6
    scale = 0.8
    z = scale * qv * (k1 - k2)
    dz = scale * (tqv * (k1 - k2) + qv * (tk1 - tk2))
    sig = 1.0 / (1.0 + math.exp(-z))
    o_ref = sig * v1 + (1 - sig) * v2
    to_ref = sig * (1 - sig) * dz * (v1 - v2) + sig * tv1 + (1 - sig) * tv2
    o, to, _ = impl(np.array([[qv]]), np.array([[k1], [k2]]), np.array([[v1], [v2]]),
                    np.array([[tqv]]), np.array([[tk1], [tk2]]), np.array([[tv1], [tv2]]), scale)
    assert abs(o[0, 0] - o_ref) < 1e-15 and abs(to[0, 0] - to_ref) < 1e-15


def pin_bruteforce_jacobian(impl):
    """Scalar loops over the softmax Jacobian dP_ij/dS_ik = P_ij (delta_jk - P_ik)."""
    q, k, v, tq, tk, tv = rand_head(100, 3, 4, 2)
    scale = 0.9
    Lq, Lkv, d = 3, 4, 2
    o, to, _ = impl(q, k, v, tq, tk, tv, scale)
    for i in range(Lq):
        s = [scale * sum(q[i][c] * k[j][c] for c in range(d)) for j in range(Lkv)]
        ts = [scale * sum(tq[i][c] * k[j][c] + q[i][c] * tk[j][c] for c in range(d)) for j in range(Lkv)]
        zsum = sum(math.exp(x) for x in s)
        p = [math.exp(x) / zsum for x in s]
        for c in range(d):
            acc = 0.0
            for j in range(Lkv):
                dp = sum(p[j] * ((1.0 if j == kk else 0.0) - p[kk]) * ts[kk] for kk in range(Lkv))
                acc += dp * v[j][c] + p[j] * tv[j][c]
            assert abs(acc - to[i][c]) < 1e-13
            assert abs(sum(p[j] * v[j][c] for j in range(Lkv)) - o[i][c]) < 1e-13


def pin_kv_permutation(impl):
    q, k, v, tq, tk, tv = rand_head(110, 6, 13, 4)
    perm = np.random.default_rng(111).permutation(13)
    a = impl(q, k, v, tq, tk, tv, 0.5)
    b = impl(q, k[perm], v[perm], tq, tk[perm], tv[perm], 0.5)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=0, atol=1e-13)


def pin_lse_tangent(impl):
    """d lse / d eps along the tangent equals rowsum(P o tS); visible in tO when V holds tS itself.

    With d = 1, V_j = 1 for one key j* and 0 elsewhere, O_i = P_ij*, and
    tO_i = P_ij* (tS_ij* - dlse_i), so dlse follows from tO; compare with FD of the library lse.
    """
    q, k, _, tq, tk, _ = rand_head(120, 5, 7, 3)
    scale = 0.5
    v = np.zeros((7, 3)); v[2, :] = 1.0
    o, to, _ = impl(q, k, v, tq, tk, np.zeros((7, 3)), scale)
    ts = scale * (tq @ k.T + q @ tk.T)
    dlse = ts[:, 2] - to[:, 0] / o[:, 0]
    eps = 1e-6
    fd = (primal_lib(q + eps * tq, k + eps * tk, v, scale)[1]
          - primal_lib(q - eps * tq, k - eps * tk, v, scale)[1]) / (2 * eps)
    np.testing.assert_allclose(dlse, fd, rtol=0, atol=1e-8)


PINS = [pin_primal_library, pin_finite_differences, pin_torch_forward_ad, pin_zero_tangent, pin_linearity,
        pin_value_tangent_is_output, pin_temperature_derivative, pin_row_constant_ts, pin_ones_value,
        pin_uniform_and_single_key, pin_two_key_logistic, pin_bruteforce_jacobian, pin_kv_permutation,
        pin_lse_tangent]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_explicit_oracle(pin):
    pin(attn_jvp_ref_head)


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
@pytest.mark.parametrize("Br,Bc,order", [(4, 3, "forward"), (128, 64, "forward"), (2, 5, "forward"), (4, 3, "tree"),
                                         (5, 2, "backward")])
def test_streaming_oracle(pin, Br, Bc, order):
    pin(lambda *a: alg2_head(*a, Br=Br, Bc=Bc, order=order))


def test_partial_states_merge_in_any_order():
    """The rescale-and-add of Alg. 2's inner loop is an associative, commutative merge of per-block states: folding
    the key blocks forward (the printed loop), backward, as a tree, or in a shuffled order gives the explicit
    definition every time, also when a later block holds the row maxima (the rescale factors are then far from 1)."""
    from oracle.alg2_stream import block_state, finish, merge
    q, k, v, tq, tk, tv = rand_head(77, 9, 50, 8)
    k[37] *= 6.0                                        # one key far above the rest for most rows
    ref = attn_jvp_ref_head(q, k, v, tq, tk, tv, 0.4)
    for order in ("forward", "backward", "tree"):
        for x, y in zip(alg2_head(q, k, v, tq, tk, tv, 0.4, 4, 7, order=order), ref):
            np.testing.assert_allclose(x, y, rtol=1e-12, atol=1e-13)
    states = [block_state(q, tq, k[j:j + 6], v[j:j + 6], tk[j:j + 6], tv[j:j + 6], 0.4) for j in range(0, 50, 6)]
    perm = np.random.default_rng(5).permutation(len(states))
    acc = states[perm[0]]
    for i in perm[1:]:
        acc = merge(states[i], acc)
    for x, y in zip(finish(acc), ref):
        np.testing.assert_allclose(x, y, rtol=1e-12, atol=1e-13)
    # a mistake in the merge must show: forgetting to rescale the tangent-side sums
    def bad_merge(a, b):
        good = merge(a, b)
        return good[0], good[1], good[2], a[3] + b[3], good[4]
    wrong = finish(bad_merge(states[0], bad_merge(states[1], states[7])))
    right = finish(merge(states[0], merge(states[1], states[7])))
    assert np.abs(wrong[1] - right[1]).max() > 1e-6


# ---------------------------------------------------------------- mutants: every planted mistake must be caught

def _mutant(kind):
    def impl(q, k, v, tq, tk, tv, scale):
        s = scale * (q @ k.T)
        if kind == "misindexed_scores":
            s = scale * (k @ q.T).T[:, ::-1] if q.shape[0] == k.shape[0] else s[:, ::-1]
        p = scipy.special.softmax(s, axis=1)
        lse = scipy.special.logsumexp(s, axis=1)
        ts = scale * (tq @ k.T + q @ tk.T)
        if kind == "ts_unscaled":
            ts = tq @ k.T + q @ tk.T
        if kind == "ts_drop_tk":
            ts = scale * (tq @ k.T)
        if kind == "ts_drop_tq":
            ts = scale * (q @ tk.T)
        if kind == "ts_minus":
            ts = scale * (tq @ k.T - q @ tk.T)
        h = p * ts
        rs = h.sum(1, keepdims=True)
        if kind == "no_rowsum":
            rs = 0 * rs
        if kind == "rowsum_of_ts":
            rs = ts.sum(1, keepdims=True)
        tp = h - p * rs
        if kind == "tp_plus":
            tp = h + p * rs
        to = tp @ v + p @ tv
        if kind == "drop_ptv":
            to = tp @ v
        if kind == "ptv_uses_v":
            to = tp @ v + p @ v
        if kind == "tpv_uses_tv":
            to = tp @ tv + p @ tv
        if kind == "lse_no_max":
            lse = np.log(np.exp(s).sum(1)) + 1e-9
        if kind == "o_unnormalised":
            return np.exp(s - s.max(1, keepdims=True)) @ v, to, lse
        return p @ v, to, lse
    return impl


MUTANTS = ["misindexed_scores", "ts_unscaled", "ts_drop_tk", "ts_drop_tq", "ts_minus", "no_rowsum",
           "rowsum_of_ts", "tp_plus", "drop_ptv", "ptv_uses_v", "tpv_uses_tv", "lse_no_max", "o_unnormalised"]


@pytest.mark.parametrize("kind", MUTANTS)
def test_pins_catch_mutants(kind):
    caught = []
    for pin in PINS:
        try:
            pin(_mutant(kind))
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake '{kind}'"


def test_unmutated_reference_of_mutant_harness_passes():
    for pin in PINS:
        pin(_mutant("none"))


# ---------------------------------------------------------------- batched wrapper, dtypes, row subsets

def test_batched_wrapper_rows_and_dtypes():
    g = torch.Generator().manual_seed(5)
    B, H, Lq, Lkv, d = 2, 3, 10, 14, 8
    mk = lambda L: torch.randn(B, H, L, d, generator=g).to(torch.bfloat16)
    q, tq = mk(Lq), mk(Lq)
    k, v, tk, tv = mk(Lkv), mk(Lkv), mk(Lkv), mk(Lkv)
    o, to, lse = attn_jvp_ref(q, k, v, tq, tk, tv, 0.3)
    assert o.dtype == np.float64 and o.shape == (B, H, Lq, d) and lse.shape == (B, H, Lq)
    rows = np.array([0, 3, 9])
    o_r, to_r, lse_r = attn_jvp_ref(q, k, v, tq, tk, tv, 0.3, rows=rows)
    np.testing.assert_array_equal(o_r, o[:, :, rows])
    np.testing.assert_array_equal(to_r, to[:, :, rows])
    np.testing.assert_array_equal(lse_r, lse[:, :, rows])
    # bf16 values are upcast exactly: same result from the float64 copies
    f = lambda x: x.double().numpy()
    o2, to2, _ = attn_jvp_ref(f(q), f(k), f(v), f(tq), f(tk), f(tv), 0.3)
    np.testing.assert_array_equal(o2, o)
    np.testing.assert_array_equal(to2, to)
    # per-head result equals the single-head routine
    oh, toh, _ = attn_jvp_ref_head(f(q)[1, 2], f(k)[1, 2], f(v)[1, 2], f(tq)[1, 2], f(tk)[1, 2], f(tv)[1, 2], 0.3)
    np.testing.assert_array_equal(oh, o[1, 2])
    np.testing.assert_array_equal(toh, to[1, 2])


def test_streaming_equals_explicit_config1_shape():
    """Config-1 sized head (L=256, d=64): the streamed result equals the explicit one for ragged tiles."""
    q, k, v, tq, tk, tv = rand_head(200, 256, 256, 64)
    ref = attn_jvp_ref_head(q, k, v, tq, tk, tv, 0.125)
    for Br, Bc in [(128, 64), (96, 40), (256, 256)]:
        got = alg2_head(q, k, v, tq, tk, tv, 0.125, Br, Bc)
        for x, y in zip(got, ref):
            np.testing.assert_allclose(x, y, rtol=0, atol=1e-12)


def test_frozen_tiny_example_still_matches():
    """tests/golden/attn_jvp_tiny.json (written by tests/golden/make_attn_jvp_tiny.py from the oracle alone) freezes
    the oracle's answers on a 3 x 5 x 4 problem: both oracles must still reproduce it, the streaming walk too."""
    import json
    import os
    from oracle.rmsnorm_jvp_ref import rmsnorm_jvp_ref
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "attn_jvp_tiny.json")) as f:
        gold = json.load(f)
    a = {n: np.array(x) for n, x in gold["inputs"].items()}
    o, to, lse = attn_jvp_ref_head(a["q"], a["k"], a["v"], a["tq"], a["tk"], a["tv"], gold["scale"])
    for got, name in ((o, "o"), (to, "to"), (lse, "lse")):
        np.testing.assert_allclose(got, np.array(gold["attention"][name]), rtol=1e-13, atol=1e-15)
    o2, to2, lse2 = alg2_head(a["q"], a["k"], a["v"], a["tq"], a["tk"], a["tv"], gold["scale"], 2, 2)
    np.testing.assert_allclose(o2, np.array(gold["attention"]["o"]), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(to2, np.array(gold["attention"]["to"]), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse2, np.array(gold["attention"]["lse"]), rtol=1e-12, atol=1e-14)
    y, ty = rmsnorm_jvp_ref(a["q"], a["tq"], a["w"], gold["eps"])
    np.testing.assert_allclose(y, np.array(gold["rmsnorm_of_q"]["y"]), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(ty, np.array(gold["rmsnorm_of_q"]["ty"]), rtol=1e-13, atol=1e-15)
