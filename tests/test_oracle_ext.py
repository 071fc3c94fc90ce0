"""Pins for the oracle's extensions: weight decay, the uncorrected gradient-averaging variant
the paper rejects (Sec. 3.2), the final global average (Algorithm 1, last line), the
replica-consistency diagnostics, and the communication-time model (Sec. 2.2, Sec. 3.1)."""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import brute
from paper_2007_00433_amd import workloads as wl

from util import TOL, bit_mismatches, layer_error

GA = oracle.FLAG_GRAD_AVG


def fresh(n, P, seed, distinct=True, v_std=0.01):
    x = wl.host_params(n, P, 0.05, seed)
    if distinct:
        x += wl.host_grads(n, P, 0.01, seed, 10 ** 6)
    v = wl.host_grads(n, P, v_std, seed, 10 ** 6 + 1) if v_std else np.zeros_like(x)
    return x, v


def test_general_step_reduces_to_the_basic_step():
    for n, m in [(8, 4), (6, 3), (16, 1), (5, 5)]:
        xa, va = fresh(n, 300, 1)
        xb, vb = xa.copy(), va.copy()
        for t in range(4):
            g = wl.host_grads(n, 300, 1e-2, 1, t)
            oracle.step(xa, g, va, m, t, 0.1, 0.9, seed=3)
            oracle.step_ex(xb, g, vb, m, t, 0.1, 0.9, 0.0, 0, seed=3)
        assert bit_mismatches(xa, xb) == 0 and bit_mismatches(va, vb) == 0


def test_gradient_averaging_over_all_workers_is_ring_sgd():
    """The uncorrected variant with one group is exactly the DSGD equation."""
    n, P = 8, 257
    for use_v in (True, False):
        xa, va = fresh(n, P, 2)
        xb, vb = xa.copy(), va.copy()
        if not use_v:
            va = vb = None
        for t in range(3):
            g = wl.host_grads(n, P, 1e-2, 2, t, "bf16" if t == 1 else "f32")
            oracle.step_ex(xa, g, va, n, t, 0.1, 0.9, 0.0, GA)
            oracle.ring_step(xb, g, vb, 0.1, 0.9)
        assert bit_mismatches(xa, xb) == 0
        if use_v:
            assert bit_mismatches(va, vb) == 0


def test_without_groups_both_variants_are_local_sgd():
    n, P = 4, 100
    xa, va = fresh(n, P, 3)
    xb, vb = xa.copy(), va.copy()
    g = wl.host_grads(n, P, 1e-2, 3, 0)
    oracle.step_ex(xa, g, va, 1, 0, 0.1, 0.9, 5e-4, 0)
    oracle.step_ex(xb, g, vb, 1, 0, 0.1, 0.9, 5e-4, GA)
    assert bit_mismatches(xa, xb) == 0 and bit_mismatches(va, vb) == 0


@pytest.mark.parametrize("n", [2, 4, 6])
def test_general_step_against_exact_rational_brute_force(n):
    rng = np.random.default_rng(300 + n)
    P = 5
    for m in [d for d in range(1, n + 1) if n % d == 0]:
        for grad_avg in (False, True):
            for use_v in (True, False):
                x = (rng.standard_normal((n, P))).astype(np.float32)
                v = (rng.standard_normal((n, P)) * 0.1).astype(np.float32) if use_v else None
                g = (rng.standard_normal((n, P)) * 0.01).astype(np.float32)
                it = int(rng.integers(0, 1000))
                group_of = oracle.plan(n, m, it)["group_of"].tolist()
                wd = np.float32(5e-4)
                want_x, want_v = brute.brute_step_ex(x, g, v, group_of, m, np.float32(0.1),
                                                     np.float32(0.9), wd, grad_avg)
                oracle.step_ex(x, g, v, m, it, 0.1, 0.9, float(wd), GA if grad_avg else 0)
                assert np.array_equal(x, want_x)
                if use_v:
                    assert np.array_equal(v, want_v)


def test_weight_decay_is_the_library_optimizer_convention():
    """m = 1 with weight decay against torch.optim.SGD(weight_decay=...) in float64."""
    n, P, T, wd = 2, 400, 10, 5e-4
    x, _ = fresh(n, P, 4, v_std=0.0)
    v = np.zeros_like(x)
    p = torch.nn.Parameter(torch.from_numpy(x.astype(np.float64)))
    opt = torch.optim.SGD([p], lr=0.1, momentum=0.9, weight_decay=wd)
    for t in range(T):
        g = wl.host_grads(n, P, 1e-2, 4, t)
        oracle.step_ex(x, g, v, 1, t, 0.1, 0.9, wd, 0)
        p.grad = torch.from_numpy(g.astype(np.float64))
        opt.step()
    assert layer_error(x, p.detach().numpy(), [0, P]) < TOL
    # decay matters at this tolerance: without it the result is measurably different
    y, _ = fresh(n, P, 4, v_std=0.0)
    w = np.zeros_like(y)
    for t in range(T):
        oracle.step_ex(y, wl.host_grads(n, P, 1e-2, 4, t), w, 1, t, 0.1, 0.9, 0.0, 0)
    assert layer_error(y, p.detach().numpy(), [0, P]) > 50 * TOL


def test_uncorrected_variant_diverges_as_the_paper_states():
    """Sec. 3.2 divergence equation: without correction x_i - x_j accumulates the differences
    of the group-mean gradients.  With i.i.d. N(0, sigma^2) gradients, no momentum, and S
    iterations in which i and j sit in different groups, E (x_i - x_j)^2 = lr^2 * S * 2 sigma^2/m
    per coordinate.  With the correction the distance stays bounded instead."""
    n, m, P, lr, sigma = 16, 4, 20000, 0.1, 1e-2
    for T in (40, 160):
        xn = wl.host_params(n, P, 0.05, 5)
        xc = xn.copy()
        sep = 0
        for t in range(T):
            g = wl.host_grads(n, P, sigma, 5, t)
            oracle.step_ex(xn, g, None, m, t, lr, 0.0, 0.0, GA, seed=5)
            oracle.step_ex(xc, g, None, m, t, lr, 0.0, 0.0, 0, seed=5)
            go = oracle.plan(n, m, t, seed=5)["group_of"]
            sep += int(go[0] != go[1])
        got = float(np.mean((xn[0].astype(np.float64) - xn[1]) ** 2))
        want = lr ** 2 * sep * 2 * sigma ** 2 / m
        assert abs(got - want) < 0.05 * want, (T, got, want)
        # appendix probability: sep / T is near n(k-1)/(k(n-1)) = 0.8
        assert abs(sep / T - 0.8) < 0.15
        dn, _ = oracle.consensus(xn)
        dc, _ = oracle.consensus(xc)
        if T == 40:
            first = (dn, dc)
    assert dn > 3.0 * first[0]               # random walk: grows ~ linearly in T (x4 here)
    assert dc < 1.5 * first[1]               # corrected: stationary
    assert dc < dn / 10


def test_global_average_pins():
    n, P = 7, 333
    x, _ = fresh(n, P, 6)
    want64 = x.astype(np.float64).mean(axis=0)
    y = x.copy()
    oracle.step(y, np.zeros_like(y), None, n, 0, 0.0, 0.0)      # averaging-only SESGD step
    z = x.copy()
    oracle.global_average(z)
    assert bit_mismatches(z, y) == 0
    assert all(bit_mismatches(z[0], z[i]) == 0 for i in range(n))
    assert np.max(np.abs(z[0] - want64)) / np.max(np.abs(want64)) < TOL
    assert np.array_equal(z[:, :9], brute.brute_global_average(x[:, :9]))
    # columns outside the range are untouched
    w = x.copy()
    oracle.global_average(w, cols=(10, 20))
    assert bit_mismatches(w[:, :10], x[:, :10]) == 0 and bit_mismatches(w[:, 20:], x[:, 20:]) == 0
    assert bit_mismatches(w[:, 10:20], z[:, 10:20]) == 0


def test_consensus_closed_forms():
    n, P = 5, 64
    a = np.array([1.0, 2.0, 4.0, -3.0, 1.0], np.float32)     # mean 1, deviations 0,1,3,-4,0
    x = np.repeat(a[:, None], P, axis=1).copy()
    d, s = oracle.consensus(x)
    assert d == P * 26.0
    assert s == P * 5.0
    y, _ = fresh(16, 1000, 7)
    d, s = oracle.consensus(y)
    y64 = y.astype(np.float64)
    assert math.isclose(d, float(((y64 - y64.mean(axis=0)) ** 2).sum()), rel_tol=1e-12)
    assert math.isclose(s, float(y64.sum()), rel_tol=1e-12, abs_tol=1e-12)
    d2, _ = oracle.consensus(y, cols=(100, 200))
    assert math.isclose(d2, float(((y64[:, 100:200] - y64[:, 100:200].mean(axis=0)) ** 2).sum()), rel_tol=1e-12)
    oracle.global_average(y)
    assert oracle.consensus(y)[0] == 0.0
    # from identical starts a full-group SESGD step leaves the replicas identical
    z = wl.host_params(8, 100, 0.05, 8)
    oracle.step(z, wl.host_grads(8, 100, 1e-2, 8, 0), np.zeros_like(z), 8, 0, 0.1, 0.9)
    assert oracle.consensus(z)[0] == 0.0


def test_cost_model_numbers_of_the_paper():
    """Sec. 2.3: 50 layers on 16 workers -> 50*2*(16-1) = 1500 handshakes.  Sec. 2.2 / 3.1:
    ring time 2(w-1)(G/(w nu) + t); approximations 2G/nu + 2 n t and 2G/nu + 2 sqrt(n) t."""
    assert oracle.handshakes(50, 16) == 1500
    assert oracle.handshakes(50, 4) == 300           # SESGD, 4 groups of 4
    G, nu = 4 * 2359296.0, 125e6                     # a 3x3x512x512 conv layer on 1 Gbps
    for t_tau in (1e-4, 5e-3):
        ring = oracle.ring_time(G, 16, nu, t_tau)
        se = oracle.ring_time(G, 4, nu, t_tau)
        assert math.isclose(ring, 2 * 15 * (G / (16 * nu) + t_tau), rel_tol=1e-15)
        approx_ring = 2 * G / nu + 2 * 16 * t_tau
        approx_se = 2 * G / nu + 2 * math.sqrt(16) * t_tau
        assert abs(ring - approx_ring) / approx_ring < 0.07
        assert abs(se - approx_se) / approx_se < 0.26     # (m-1)/m is a coarser approximation at m = 4
        assert se < ring
    # latency-dominated limit: communication speed-up -> (n-1)/(n/k-1) = 5 for n=16, k=4,
    # the "almost 5x" the paper reports at 5 ms
    tiny_layer = 4 * 64.0
    assert math.isclose(oracle.ring_time(tiny_layer, 16, nu, 5e-3) / oracle.ring_time(tiny_layer, 4, nu, 5e-3),
                        5.0, rel_tol=1e-3)
    assert oracle.ring_time(1.0, 0, nu, 0.0) < 0
