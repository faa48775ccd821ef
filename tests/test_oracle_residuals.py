"""Pins of the oracle's layer-wise residual norms (Section 3.4, last paragraph; Algorithm 1 Phase 5).  CPU only."""
import numpy as np

import oracle
import workloads as wk
from tests.test_oracle_pins import one_layer_table, random_table


def test_handworked_residuals():
    # one layer [2,1,1,2]; two replicas; all values exact.  theta_1 - z_i = [1,0,0,2], theta_2 - z_i = [0,-1,3,0]
    t = one_layer_table(2, 1, 2, wk.MODE_FILTER, 1)
    W = np.array([[2, 0, 1, 2], [1, -1, 4, 0]], np.float32)
    Zi = np.array([1, 0, 1, 0], np.float32)
    Zp = np.array([0, 0, 3, 0], np.float32)          # z_i - z_i_prev = [1,0,-2,0]
    Zg = np.array([1, 1, 1, -1], np.float32)         # z_i - z = [0,-1,0,1]
    Zgp = np.array([0, 1, 1, 1], np.float32)         # z - z_prev = [1,0,0,-2]
    out = oracle.residuals(t, W, Zi, Zp, Zg, Zgp)
    assert out[:, 0].tolist() == [1 + 4 + 1 + 9, 1 + 4, 1 + 1, 1 + 4]
    out = oracle.residuals(t, W, Zi)
    assert out[:, 0].tolist() == [15, 0, 0, 0]


def test_residuals_against_numpy_and_their_zero_cases():
    rng = np.random.default_rng(2)
    wl = wk.custom_workload(random_table(rng, 7), R=3, seed=4, sigma_replica=0.03)
    W, U = wk.generate(wl)
    p = oracle.project(wl.table(), W, U)
    Zi = p["Z"]
    Zp = rng.standard_normal(wl.n_arena).astype(np.float32)
    Zg = rng.standard_normal(wl.n_arena).astype(np.float32)
    Zgp = rng.standard_normal(wl.n_arena).astype(np.float32)
    out = oracle.residuals(wl.table(), W, Zi, Zp, Zg, Zgp)
    for li, l in enumerate(wl.layers):
        sl = slice(l.elem_off, l.elem_off + l.n)
        f = lambda a, b: float(np.sum((a[sl].astype(np.float64) - b[sl].astype(np.float64)) ** 2))
        np.testing.assert_allclose(out[0, li], sum(f(W[r], Zi) for r in range(3)), rtol=1e-12)
        np.testing.assert_allclose(out[1, li], f(Zi, Zp), rtol=1e-12)
        np.testing.assert_allclose(out[2, li], f(Zi, Zg), rtol=1e-12)
        np.testing.assert_allclose(out[3, li], f(Zg, Zgp), rtol=1e-12)
    # consensus reached: every replica equals z_i, z_i is unchanged and equals z -> all residuals vanish
    Wc = np.stack([Zi, Zi, Zi])
    assert not oracle.residuals(wl.table(), Wc, Zi, Zi, Zi, Zi).any()
    # pruned groups contribute their whole weight to the primal residual: with U = 0 and R = 1,
    # ||theta - z_i||^2 is the sum of the pruned groups' squared norms (the keys of the projection)
    W1, _ = wk.generate(wk.custom_workload([(9, 4, 4, wk.MODE_FILTER, 3)], R=1, seed=1))
    t = one_layer_table(9, 4, 4, wk.MODE_FILTER, 3)
    p1 = oracle.project(t, W1, np.zeros(W1.shape[1], np.float32))
    r = oracle.residuals(t, W1, p1["Z"])
    np.testing.assert_allclose(r[0, 0], p1["key"][p1["mask"] == 0].sum(), rtol=1e-12)
