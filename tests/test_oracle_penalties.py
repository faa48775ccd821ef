"""Pins of the oracle's adaptive penalty tuning (Section 3.4, last paragraph; Algorithm 1 Phase 5: residual
balancing per layer and level, duals rescaled) and of the per-layer rescaling of an arena.  CPU only.

The rule's constants (mu, tau) are not in the paper; the tests pass the values the ADMM reference it cites suggests
(mu = 10, tau = 2) or exactly representable ones where a boundary is probed."""
import math

import numpy as np
import pytest

import oracle
import workloads as wk
from tests.test_oracle_pins import random_table


def _sq(rows):
    return np.array(rows, dtype=np.float64)


def test_handworked_balancing_both_levels_and_the_cap():
    # four layers, P = 4 replicas, the node's own view of the inter-node residuals (n_out = 1), mu = 10, tau = 2.
    # intra: ||r|| = sqrt(row 0), ||s|| = rho_1 sqrt(4 row 1)
    #   l0: r = 2,    s = 1 * sqrt(4e-4) = 0.02   -> r > 10 s : rho_1 1 -> 2,   u scaled by 1/2
    #   l1: r = 1e-3, s = 1 * sqrt(4)    = 2      -> s > 10 r : rho_1 1 -> 1/2, u scaled by 2
    #   l2: r = 1,    s = 1 * sqrt(0.04) = 0.2    -> neither  : unchanged,      scale 1
    #   l3: r = 3,    s = 8 * 0 = 0               -> raise, 16 capped at 10,    scale 8/10
    # inter: ||r|| = sqrt(row 2), ||s|| = rho_2 sqrt(row 3)
    #   l0: r = 0.5,  s = 0.25 * 1 = 0.25 -> neither;  l1: r = 5, s = 0.25 * 0.04 = 0.01 -> raise 0.25 -> 0.5
    #   l2: r = 0, s = 0 -> unchanged;  l3: r = 0.01, s = 4 * 0.5 = 2 -> lower 4 -> 2, v scaled by 2
    sq = _sq([[4.0, 1e-6, 1.0, 9.0], [1e-4, 1.0, 1e-2, 0.0], [0.25, 25.0, 0.0, 1e-4], [1.0, 1.6e-3, 0.0, 0.25]])
    r1, r2, su, sv = oracle.adapt_penalties(sq, [1.0, 1.0, 1.0, 8.0], [0.25, 0.25, 0.25, 4.0], 4, 1, 10.0, 2.0, 2.0,
                                            10.0, 10.0)
    assert r1.tolist() == [2.0, 0.5, 1.0, 10.0]
    assert su.tolist() == [0.5, 2.0, 1.0, np.float32(0.8)]
    assert r2.tolist() == [0.25, 0.5, 0.25, 2.0]
    assert sv.tolist() == [1.0, 0.5, 1.0, 2.0]


def test_the_inequalities_are_strict_and_the_dual_norm_counts_the_copies():
    # r = 2; s = rho sqrt(P sq_s) = 0.5 * sqrt(4 / 64) = 0.125; mu = 16 -> mu s = 2 = r exactly: unchanged
    base = [[4.0], [1.0 / 64.0], [0.0], [0.0]]
    r1, _, su, _ = oracle.adapt_penalties(_sq(base), [0.5], [1.0], 4, 1, 16.0, 2.0, 2.0, 10.0, 10.0)
    assert r1.tolist() == [0.5] and su.tolist() == [1.0]
    up = [[4.0 * (1.0 + 2.0 ** -51)], [1.0 / 64.0], [0.0], [0.0]]     # two ulps: its root is the next double after 2
    r1, _, su, _ = oracle.adapt_penalties(_sq(up), [0.5], [1.0], 4, 1, 16.0, 2.0, 2.0, 10.0, 10.0)
    assert r1.tolist() == [1.0] and su.tolist() == [0.5]
    # the same numbers with one replica: s = 0.5 * 0.125 = 0.0625, mu s = 1 < r = 2 -> raised
    r1, _, _, _ = oracle.adapt_penalties(_sq(base), [0.5], [1.0], 1, 1, 16.0, 2.0, 2.0, 10.0, 10.0)
    assert r1.tolist() == [1.0]
    # mirror case on the dual side: s = mu r exactly -> unchanged; two ulps more under the root -> lowered
    # r = 0.125, mu = 16 -> 2;  s = 1 * sqrt(4 * 1) = 2
    r1, _, _, _ = oracle.adapt_penalties(_sq([[1.0 / 64.0], [1.0], [0.0], [0.0]]), [1.0], [1.0], 4, 1, 16.0, 2.0, 4.0,
                                         10.0, 10.0)
    assert r1.tolist() == [1.0]
    r1, _, su, _ = oracle.adapt_penalties(_sq([[1.0 / 64.0], [1.0 + 2.0 ** -51], [0.0], [0.0]]), [1.0], [1.0], 4,
                                          1, 16.0, 2.0, 4.0, 10.0, 10.0)
    assert r1.tolist() == [0.25] and su.tolist() == [4.0]
    # inter level: the number of nodes summed into the primal row enters the dual norm the same way
    inter = [[0.0], [0.0], [4.0], [1.0 / 64.0]]
    _, r2, _, _ = oracle.adapt_penalties(_sq(inter), [1.0], [0.5], 1, 4, 16.0, 2.0, 2.0, 10.0, 10.0)
    assert r2.tolist() == [0.5]
    _, r2, _, sv = oracle.adapt_penalties(_sq(inter), [1.0], [0.5], 1, 1, 16.0, 2.0, 2.0, 10.0, 10.0)
    assert r2.tolist() == [1.0] and sv.tolist() == [0.5]


def test_repeated_raises_follow_the_closed_form_count():
    """With fixed residual sums and ||r|| far above ||s||, rho grows by tau per call until mu ||s|| (which grows with
    rho) reaches ||r|| or the cap is hit: n = ceil(log_tau(||r|| / (mu rho_0 sqrt(P sq_s)))) raises, counted here from
    that closed form and not from the rule."""
    rng = np.random.default_rng(11)
    for _ in range(50):
        P = int(rng.integers(1, 9))
        tau = float(rng.choice([1.5, 2.0, 3.0]))
        mu = float(rng.choice([2.0, 10.0]))
        rho0 = float(10.0 ** rng.uniform(-4, -2))
        sq_r = float(10.0 ** rng.uniform(-2, 2))
        sq_s = float(10.0 ** rng.uniform(-6, -2))
        ratio = math.sqrt(sq_r) / (mu * rho0 * math.sqrt(P * sq_s))
        want = max(0, math.ceil(math.log(ratio) / math.log(tau) - 1e-12)) if ratio > 1.0 else 0
        if abs(math.log(ratio) / math.log(tau) - round(math.log(ratio) / math.log(tau))) < 1e-9:
            continue                                            # on a boundary the count is a matter of rounding
        rho, n = rho0, 0
        for _ in range(200):
            r1, _, su, _ = oracle.adapt_penalties(_sq([[sq_r], [sq_s], [0.0], [0.0]]), [rho], [1.0], P, 1, mu, tau, tau,
                                                  1e30, 1e30)
            if r1[0] == rho:
                break
            assert r1[0] == tau * rho and su[0] == np.float32(rho / (tau * rho))
            rho, n = float(r1[0]), n + 1
        assert n == want, (n, want, ratio, tau)


def test_layers_and_levels_are_independent_and_neutral_constants_change_nothing():
    rng = np.random.default_rng(3)
    L = 9
    sq = 10.0 ** rng.uniform(-8, 2, (4, L))
    rho1 = 10.0 ** rng.uniform(-3, 0, L)
    rho2 = 10.0 ** rng.uniform(-4, 0, L)
    args = (3, 2, 10.0, 2.0, 2.0, 10.0, 10.0)
    r1, r2, su, sv = oracle.adapt_penalties(sq, rho1, rho2, *args)
    assert (r1 != rho1).any() and (r2 != rho2).any()              # the draw exercises the rule
    perm = rng.permutation(L)
    p1, p2, pu, pv = oracle.adapt_penalties(sq[:, perm], rho1[perm], rho2[perm], *args)
    assert np.array_equal(p1, r1[perm]) and np.array_equal(p2, r2[perm])
    assert np.array_equal(pu, su[perm]) and np.array_equal(pv, sv[perm])
    other = sq.copy()
    other[2:] = 10.0 ** rng.uniform(-8, 2, (2, L))                # inter-node rows replaced: intra results stay
    q1, _, qu, _ = oracle.adapt_penalties(other, rho1, rho2, *args)
    assert np.array_equal(q1, r1) and np.array_equal(qu, su)
    other = sq.copy()
    other[:2] = 10.0 ** rng.uniform(-8, 2, (2, L))
    _, q2, _, qv = oracle.adapt_penalties(other, rho1, rho2, *args)
    assert np.array_equal(q2, r2) and np.array_equal(qv, sv)
    for mu, ti, td in ((1e300, 2.0, 2.0), (10.0, 1.0, 1.0)):      # nothing ever out of balance / unit steps
        n1, n2, nu, nv = oracle.adapt_penalties(sq, rho1, rho2, 3, 2, mu, ti, td, 10.0, 10.0)
        assert np.array_equal(n1, rho1) and np.array_equal(n2, rho2)
        assert (nu == 1.0).all() and (nv == 1.0).all()
    # rho_new * scale = rho_old (the unscaled dual y = rho u is what must survive the change)
    np.testing.assert_allclose(r1 * su.astype(np.float64), rho1, rtol=2.0 ** -23)
    np.testing.assert_allclose(r2 * sv.astype(np.float64), rho2, rtol=2.0 ** -23)


def test_rescaled_dual_keeps_a_converged_scaled_admm_at_its_fixed_point():
    """A two-block consensus problem solved by scaled ADMM in this test: min (x - a)^2 / 2 + c (z - b)^2 / 2 s.t.
    x = z.  At convergence the unscaled dual y = rho u does not depend on rho, so after a change of rho the iteration
    stays at its fixed point exactly when u is multiplied by rho_old / rho_new -- the factor the oracle returns."""
    a, b, c = 3.0, -1.0, 2.0

    def iterate(x, z, u, rho, n):
        for _ in range(n):
            x = (a + rho * (z - u)) / (1.0 + rho)
            z = (c * b + rho * (x + u)) / (c + rho)
            u = u + x - z
        return x, z, u

    rho = 0.5
    x, z, u = iterate(0.0, 0.0, 0.0, rho, 400)
    fixed = (a + c * b) / (1.0 + c)
    assert abs(x - fixed) < 1e-12 and abs(z - fixed) < 1e-12
    # residual sums that call for a raise, then for a cut
    for sq, expect in (([[1.0], [1e-8], [0.0], [0.0]], 1.0), ([[1e-8], [1.0], [0.0], [0.0]], 0.25)):
        r1, _, su, _ = oracle.adapt_penalties(_sq(sq), [rho], [1.0], 1, 1, 10.0, 2.0, 2.0, 10.0, 10.0)
        assert r1[0] == expect
        x2, z2, _ = iterate(x, z, u * float(su[0]), float(r1[0]), 1)
        assert abs(x2 - fixed) < 1e-6 and abs(z2 - fixed) < 1e-6
        x3, z3, _ = iterate(x, z, u / float(su[0]), float(r1[0]), 1)      # the inverse factor leaves the fixed point
        assert abs(x3 - fixed) > 1e-2


def test_penalty_arguments_are_checked():
    ok = ([[1.0], [1.0], [1.0], [1.0]], [1.0], [1.0], 2, 1, 10.0, 2.0, 2.0, 10.0, 10.0)
    oracle.adapt_penalties(_sq(ok[0]), *ok[1:])
    for pos, bad in ((1, [0.0]), (1, [11.0]), (2, [-1.0]), (3, 0), (4, 0), (5, 0.0), (6, 0.5), (7, 0.99)):
        args = list(ok)
        args[pos] = bad
        with pytest.raises(ValueError):
            oracle.adapt_penalties(_sq(args[0]), *args[1:])
    with pytest.raises(ValueError):
        oracle.adapt_penalties(_sq([[1.0], [-1.0], [1.0], [1.0]]), *ok[1:])


def test_scale_layers_is_a_per_layer_float32_multiply():
    rng = np.random.default_rng(5)
    wl = wk.custom_workload(random_table(rng, 6), R=1, seed=2)
    t = wl.table()
    X = rng.standard_normal(wl.n_arena).astype(np.float32)
    f = rng.uniform(0.25, 4.0, len(wl.layers)).astype(np.float32)
    f[2] = 1.0
    out = oracle.scale_layers(t, X, f)
    want = X.copy()
    for li, l in enumerate(wl.layers):
        sl = slice(l.elem_off, l.elem_off + l.n)
        want[sl] = X[sl] * f[li]                                 # NumPy's float32 product: one rounding
    assert np.array_equal(out.view(np.uint32), want.view(np.uint32))
    assert np.array_equal(oracle.scale_layers(t, X, np.ones(len(wl.layers), np.float32)).view(np.uint32),
                          X.view(np.uint32))
