"""Pins of the oracle's full node update (Eq. (9) with the rho_2 (z - v) term), the inter-node dual update
(Eq. (13)) and the pre-transmission sum c = z_i + v_i (Section 4.4.1).  CPU only."""
import json

import numpy as np
import pytest

import oracle
import workloads as wk
from tests.test_oracle_pins import one_layer_table, random_table, GOLDEN

G = json.load(open(GOLDEN))["weighted_cases"]


def test_coefficients_of_eq_9():
    c = G["coefficients"]
    a, b = oracle.node_coefficients([c["rho1"]], [c["rho2"]], c["lambda"], c["M"], c["P"])
    assert a[0] == np.float32(c["a"]) and b[0] == np.float32(c["b"])
    gamma = c["lambda"] / c["M"] + c["P"] * c["rho1"] + c["rho2"]
    assert gamma == pytest.approx(c["gamma"], rel=1e-15)
    # lambda = 0 and rho_2 = 0: the plain mean (a = 1, b = 0), whatever rho_1 and P are
    a, b = oracle.node_coefficients([0.3, 7.0], [0.0, 0.0], 0.0, 5, 8)
    assert a.tolist() == [1.0, 1.0] and b.tolist() == [0.0, 0.0]
    # the three weights of Eq. (9) sum to one: a + b + (lambda/M)/gamma = 1
    rng = np.random.default_rng(0)
    r1, r2 = rng.uniform(1e-4, 10, 50), rng.uniform(0, 10, 50)
    a, b = oracle.node_coefficients(r1, r2, 3e-4, 16, 4)
    gam = 3e-4 / 16 + 4 * r1 + r2
    np.testing.assert_allclose(a.astype(np.float64) + b + (3e-4 / 16) / gam, 1.0, atol=2e-7)
    np.testing.assert_allclose(a, 4 * r1 / gam, rtol=1e-7)
    with pytest.raises(ValueError):
        oracle.node_coefficients([0.0], [0.0], 0.0, 1, 1)          # gamma = 0


def test_handworked_weighted_projection():
    c = G["project"]
    t = one_layer_table(c["c_out"], c["c_in"], c["khw"], c["mode"], c["k"])
    W = np.array(c["W"], np.float32)
    U = np.array(c["U"], np.float32)
    out = oracle.project_weighted(t, W, U, np.array(c["Zg"], np.float32), np.array(c["Vd"], np.float32),
                                  [c["a"]], [c["b"]], want_wbar=True)
    assert out["key"].tolist() == c["key"] and out["mask"].tolist() == c["mask"]
    assert out["Z"].tolist() == c["Z"] and out["U"].tolist() == c["U_new"]
    assert oracle.project(t, W, U)["mask"].tolist() == c["mask_without_global_term"]


@pytest.mark.parametrize("seed", range(3))
def test_weights_one_and_zero_give_the_base_projection(seed):
    rng = np.random.default_rng(seed)
    wl = wk.custom_workload(random_table(rng, 7), R=int(rng.integers(1, 5)), seed=seed, sigma_replica=0.03)
    W, U = wk.generate(wl)
    Zg = rng.standard_normal(wl.n_arena).astype(np.float32)
    Vd = rng.standard_normal(wl.n_arena).astype(np.float32)
    L = len(wl.layers)
    a = oracle.project(wl.table(), W, U, want_wbar=True)
    b = oracle.project_weighted(wl.table(), W, U, Zg, Vd, np.ones(L), np.zeros(L), want_wbar=True)
    assert np.array_equal(a["mask"], b["mask"])
    for name in ("Z", "U", "Wbar"):
        assert np.array_equal(a[name], b[name]), name          # == : a zero may change sign through + (0 * q)
    assert np.array_equal(a["key"].view(np.uint64), b["key"].view(np.uint64))


def test_eq_9_printed_formula_with_per_replica_duals():
    """z~ = (1/gamma) [rho_1 sum_j (theta_j + u_j) + rho_2 (z - v)] in float64 against the oracle's candidate on
    an unconstrained layer (where Z = z~), with U = mean_j u_j."""
    rng = np.random.default_rng(5)
    P, M, lam, rho1, rho2 = 4, 16, 1e-4, 1.5e-3, 1.5e-4
    n = 48
    theta = rng.standard_normal((P, n)).astype(np.float32)
    u = (0.05 * rng.standard_normal((P, n))).astype(np.float32)
    z = rng.standard_normal(n).astype(np.float32)
    v = (0.1 * rng.standard_normal(n)).astype(np.float32)
    gamma = lam / M + P * rho1 + rho2
    z_tilde = (rho1 * np.sum(theta.astype(np.float64) + u, axis=0) + rho2 * (z.astype(np.float64) - v)) / gamma
    ubar = np.mean(u.astype(np.float64), axis=0).astype(np.float32)
    a, b = oracle.node_coefficients([rho1], [rho2], lam, M, P)
    t = one_layer_table(6, 8, 1, wk.MODE_NONE, 6)
    out = oracle.project_weighted(t, theta, ubar, z, v, a, b)
    np.testing.assert_allclose(out["Z"], z_tilde, rtol=0, atol=2e-6)


@pytest.mark.parametrize("seed", range(3))
def test_weighted_against_numpy(seed):
    rng = np.random.default_rng(20 + seed)
    wl = wk.custom_workload(random_table(rng, 6), R=3, seed=seed, sigma_replica=0.03)
    W, U = wk.generate(wl)
    Zg = rng.standard_normal(wl.n_arena).astype(np.float32)
    Vd = (0.3 * rng.standard_normal(wl.n_arena)).astype(np.float32)
    L = len(wl.layers)
    a = rng.uniform(0.5, 1.0, L).astype(np.float32)
    b = rng.uniform(0.0, 0.5, L).astype(np.float32)
    out = oracle.project_weighted(wl.table(), W, U, Zg, Vd, a, b, want_wbar=True)
    acc = W[0].copy()
    for r in range(1, 3):
        acc = (acc + W[r]).astype(np.float32)
    wbar = (acc * (np.float32(1) / np.float32(3))).astype(np.float32)
    for li, l in enumerate(wl.layers):
        sl = slice(l.elem_off, l.elem_off + l.n)
        t = (wbar[sl] + U[sl]).astype(np.float32)
        q = (Zg[sl] - Vd[sl]).astype(np.float32)
        v = ((a[li] * t).astype(np.float32) + (b[li] * q).astype(np.float32)).astype(np.float32)
        v3 = v.reshape(l.c_out, l.c_in, l.khw).astype(np.float64)
        key = np.sum(v3 * v3, axis=(0, 2) if l.mode == wk.MODE_CHANNEL else (1, 2))
        np.testing.assert_allclose(out["key"][l.group_base:l.group_base + l.groups], key, rtol=1e-12)
        if l.mode == wk.MODE_NONE:
            m = np.ones(l.groups, np.uint8)
        else:
            m = np.zeros(l.groups, np.uint8)
            m[np.argsort(-key, kind="stable")[:l.k]] = 1
        assert np.array_equal(out["mask"][l.group_base:l.group_base + l.groups], m)
        m3 = m[None, :, None] if l.mode == wk.MODE_CHANNEL else m[:, None, None]
        z = np.where(np.broadcast_to(m3.astype(bool), v3.shape), v.reshape(v3.shape), np.float32(0)).reshape(-1)
        assert np.array_equal(out["Z"][sl].view(np.uint32), z.astype(np.float32).view(np.uint32))
        un = (U[sl] + (wbar[sl] - z).astype(np.float32)).astype(np.float32)
        assert np.array_equal(out["U"][sl].view(np.uint32), un.view(np.uint32))


def test_inter_node_dual_update_and_transmission_sum():
    c = G["dual_inter"]
    t = one_layer_table(2, 2, 1, wk.MODE_FILTER, 1)
    vn = oracle.dual_inter(t, np.array(c["Zi"], np.float32), np.array(c["Zg"], np.float32), np.array(c["Vd"], np.float32))
    assert vn.tolist() == c["Vd_new"]
    rng = np.random.default_rng(3)
    wl = wk.custom_workload([(5, 3, 4, wk.MODE_FILTER, 2), (3, 3, 1, wk.MODE_CHANNEL, 1)], R=1, seed=0)
    Zi = rng.standard_normal(wl.n_arena).astype(np.float32)
    Vd = rng.standard_normal(wl.n_arena).astype(np.float32)
    assert np.array_equal(oracle.dual_inter(wl.table(), Zi, Zi, Vd), Vd)          # z == z_i: v unchanged
    Zg = rng.standard_normal(wl.n_arena).astype(np.float32)
    assert np.array_equal(oracle.dual_inter(wl.table(), Zi, Zg, Vd), (Vd + (Zi - Zg).astype(np.float32)).astype(np.float32))
    C = oracle.add_arenas(wl.table(), Zi, Vd)
    pad = np.ones(wl.n_arena, bool)
    for l in wl.layers:
        pad[l.elem_off:l.elem_off + l.n] = False
    assert np.array_equal(C[~pad], (Zi + Vd).astype(np.float32)[~pad]) and not C[pad].any()
    # one node (M = 1): Eq. (11) gives z = z_i + v_i = c, and Eq. (13) then returns v to zero (exact values)
    zi = np.array([3, 0, -2, 8], np.float32)
    v = np.array([1, 4, 0.5, -8], np.float32)
    t2 = one_layer_table(2, 2, 1, wk.MODE_FILTER, 1)
    c2 = oracle.add_arenas(t2, zi, v)
    assert oracle.dual_inter(t2, zi, c2, v).tolist() == [0, 0, 0, 0]


# ---------------------------------------------------------------- retraining branch with the full candidate

def _mixed_workload(rng, seed):
    from tests.test_oracle_composite import random_table_with_both
    return wk.custom_workload(random_table_with_both(rng, 8), R=int(rng.integers(1, 5)), seed=seed, sigma_replica=0.03)


@pytest.mark.parametrize("seed", range(3))
def test_weighted_frozen_with_its_own_mask_is_the_dynamic_weighted_projection(seed):
    """Algorithm 1, Phase 3: both branches form the same candidate; under the mask the dynamic branch selects, the
    frozen branch must reproduce its Z, U and Wbar bit for bit."""
    rng = np.random.default_rng(300 + seed)
    wl = _mixed_workload(rng, seed)
    W, U = wk.generate(wl)
    L = len(wl.layers)
    Zg = (rng.standard_normal(wl.n_arena) * 0.05).astype(np.float32)
    Vd = (rng.standard_normal(wl.n_arena) * 0.01).astype(np.float32)
    a = rng.uniform(0.3, 1.0, L).astype(np.float32)
    b = rng.uniform(0.0, 0.7, L).astype(np.float32)
    dyn = oracle.project_weighted(wl.table(), W, U, Zg, Vd, a, b, want_wbar=True)
    frz = oracle.project_weighted_frozen(wl.table(), W, U, Zg, Vd, a, b, dyn["mask"] * 200, want_wbar=True)
    for name in ("Z", "U", "Wbar"):
        assert np.array_equal(dyn[name].view(np.uint32), frz[name].view(np.uint32)), name


@pytest.mark.parametrize("seed", range(3))
def test_weighted_frozen_with_weights_one_and_zero_is_the_base_frozen_projection(seed):
    rng = np.random.default_rng(400 + seed)
    wl = _mixed_workload(rng, seed)
    W, U = wk.generate(wl)
    L = len(wl.layers)
    Zg = rng.standard_normal(wl.n_arena).astype(np.float32)
    Vd = rng.standard_normal(wl.n_arena).astype(np.float32)
    mask = (rng.random(wl.groups_total) < 0.5).astype(np.uint8)
    base = oracle.project_frozen(wl.table(), W, U, mask, want_wbar=True)
    wtd = oracle.project_weighted_frozen(wl.table(), W, U, Zg, Vd, np.ones(L), np.zeros(L), mask, want_wbar=True)
    for name in ("Z", "U", "Wbar"):
        assert np.array_equal(base[name], wtd[name]), name     # == : a zero may change sign through + (0 * q)


def test_weighted_frozen_against_the_printed_formulas_in_float64():
    """z~ = a (Wbar + U) + b (z - v) (Eq. (9)), z_i = z~ (.) m (Algorithm 1, Phase 3, retraining branch),
    u <- u + (Wbar - z_i) (Eq. (12)), written out in NumPy float64 on values where fp32 is exact."""
    rng = np.random.default_rng(9)
    co, ci, s = 6, 5, 4
    from tests.test_oracle_composite import both_table
    t = both_table(co, ci, s, 3, 2)
    n = co * ci * s
    W = (rng.integers(-8, 9, (2, n)) / 4.0).astype(np.float32)          # quarters: all sums below are exact in fp32
    U = (rng.integers(-8, 9, n) / 4.0).astype(np.float32)
    Zg = (rng.integers(-8, 9, n) / 4.0).astype(np.float32)
    Vd = (rng.integers(-8, 9, n) / 4.0).astype(np.float32)
    a, b = np.float32(0.5), np.float32(0.25)
    mask = np.array([1, 0, 1, 1, 0, 1] + [0, 1, 1, 0, 1], np.uint8)      # filters, then channels
    out = oracle.project_weighted_frozen(t, W, U, Zg, Vd, [a], [b], mask, want_wbar=True)
    wbar = W.astype(np.float64).mean(axis=0)
    zt = 0.5 * (wbar + U) + 0.25 * (Zg.astype(np.float64) - Vd)
    keep = (mask[:co, None, None] != 0) & (mask[co:][None, :, None] != 0)
    z = np.where(np.broadcast_to(keep, (co, ci, s)).reshape(-1), zt, 0.0)
    assert np.array_equal(out["Wbar"].astype(np.float64), wbar)
    assert np.array_equal(out["Z"].astype(np.float64), z)
    assert np.array_equal(out["U"].astype(np.float64), U + (wbar - z))
    # a pruned filter's row and a pruned channel's columns are exactly +0
    Z3 = out["Z"].reshape(co, ci, s)
    assert not Z3[1].any() and not Z3[:, 0].any() and not np.signbit(Z3[1]).any()
    # filter and channel masks alone
    for mode, m in ((wk.MODE_FILTER, mask[:co]), (wk.MODE_CHANNEL, mask[co:])):
        o = oracle.project_weighted_frozen(one_layer_table(co, ci, s, mode, 1), W, U, Zg, Vd, [a], [b], m)
        k3 = (m[:, None, None] != 0) if mode == wk.MODE_FILTER else (m[None, :, None] != 0)
        assert np.array_equal(o["Z"].astype(np.float64), np.where(np.broadcast_to(k3, (co, ci, s)).reshape(-1), zt, 0.0))
    # an unconstrained layer ignores its mask bytes
    o = oracle.project_weighted_frozen(one_layer_table(co, ci, s, wk.MODE_NONE, co), W, U, Zg, Vd, [a], [b],
                                       np.zeros(co, np.uint8))
    assert np.array_equal(o["Z"].astype(np.float64), zt)
