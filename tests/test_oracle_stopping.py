"""Pins of the oracle's stopping test (Section 3.4, last paragraph; Algorithm 1 Phase 5: break once the total primal
and dual residual norms are below eps_pri and eps_dual) and of the layer-wise squared norms it is relative to.  CPU
only.

The tolerances are not in the paper (it defers to the absolute / relative tolerances of the ADMM reference it
cites); the tests pass exactly representable ones so that boundaries can be probed."""
import math

import numpy as np
import pytest

import oracle
import workloads as wk
from tests.test_oracle_pins import random_table


def _col(*rows):
    return np.array(rows, dtype=np.float64).reshape(len(rows), -1)


def test_handworked_thresholds_one_layer():
    # n = 16 elements, P = 3 replicas, the node's own view (n_out = 1): p = (3 + 1) * 16 = 64, sqrt(p) = 8
    # residual sums: intra primal 9, intra dual 1/16, inter primal 16, inter dual 1/4;  rho_1 = 2, rho_2 = 4
    #   R_pri  = sqrt(9 + 16) = 5
    #   R_dual = sqrt(3 * 4 * 1/16 + 1 * 16 * 1/4) = sqrt(3/4 + 4) = sqrt(4.75)
    # magnitudes: sum_j ||theta_j||^2 = 300, ||z_i||^2 = 100, ||z||^2 = 144, sum_j ||u_j||^2 = 9, ||v||^2 = 4
    #   ||A x|| = sqrt(300 + 100) = 20;  ||B z|| = sqrt(3 * 100 + 144) = sqrt(444) = 21.07...;  max = sqrt(444)
    #   ||A^T y|| = sqrt(4 * 9 + 16 * 4) = 10
    # eps_abs = 1/2, eps_rel = 1/8:  eps_pri = 4 + sqrt(444)/8 = 6.63... > 5;  eps_dual = 4 + 10/8 = 5.25 > sqrt(4.75)
    sq, mag = _col([9.0], [1.0 / 16.0], [16.0], [0.25]), _col([300.0], [100.0], [144.0], [9.0], [4.0])
    done, every = oracle.stopping_test([16], 3, 1, [2.0], [4.0], sq, mag, 0.5, 0.125)
    assert done.tolist() == [1] and every
    # eps_abs = 1/8: eps_pri = 1 + 2.63 = 3.63 < 5 -> not converged (the primal side alone decides)
    done, every = oracle.stopping_test([16], 3, 1, [2.0], [4.0], sq, mag, 0.125, 0.125)
    assert done.tolist() == [0] and not every
    # a large dual residual alone also prevents it: inter dual sum 4 -> R_dual = sqrt(0.75 + 64) > 5.25
    sq2 = _col([9.0], [1.0 / 16.0], [16.0], [4.0])
    assert oracle.stopping_test([16], 3, 1, [2.0], [4.0], sq2, mag, 0.5, 0.125)[0].tolist() == [0]


def test_both_comparisons_are_strict():
    # absolute tolerance only (eps_rel = 0): eps = sqrt(p) eps_abs with p = (1 + 1) * 8 = 16 -> 4 eps_abs
    mag = _col([1.0], [1.0], [1.0], [1.0], [1.0])
    at = _col([9.0], [0.0], [7.0], [0.0])            # R_pri = 4 exactly, R_dual = 0
    assert oracle.stopping_test([8], 1, 1, [1.0], [1.0], at, mag, 1.0, 0.0)[0].tolist() == [0]      # 4 < 4 is false
    below = _col([9.0], [0.0], [7.0 * (1.0 - 2.0 ** -50)], [0.0])
    assert oracle.stopping_test([8], 1, 1, [1.0], [1.0], below, mag, 1.0, 0.0)[0].tolist() == [1]
    # the dual side: R_dual = rho_1 sqrt(P sq_1) = 2 * sqrt(4) = 4 = eps_dual -> not converged
    dual_at = _col([0.0], [4.0], [0.0], [0.0])
    assert oracle.stopping_test([8], 1, 1, [2.0], [1.0], dual_at, mag, 1.0, 0.0)[0].tolist() == [0]
    dual_below = _col([0.0], [4.0 * (1.0 - 2.0 ** -50)], [0.0], [0.0])
    assert oracle.stopping_test([8], 1, 1, [2.0], [1.0], dual_below, mag, 1.0, 0.0)[0].tolist() == [1]
    # zero residuals with zero tolerances: 0 < 0 is false
    zero = _col([0.0], [0.0], [0.0], [0.0])
    assert oracle.stopping_test([8], 1, 1, [1.0], [1.0], zero, mag, 0.0, 0.0)[0].tolist() == [0]
    assert oracle.stopping_test([8], 1, 1, [1.0], [1.0], zero, mag, 0.0, 2.0 ** -20)[0].tolist() == [1]


def test_relative_part_takes_the_larger_of_the_two_stacks_and_the_unscaled_duals():
    # eps_abs = 0.  P = 4, n_out = 1.
    # ||A x||^2 = 64 + 36 = 100 (10);  ||B z||^2 = 4 * 36 + 81 = 225 (15) -> eps_pri = 15 eps_rel
    sq = _col([49.0], [0.0], [0.0], [0.0])           # R_pri = 7
    mag = _col([64.0], [36.0], [81.0], [0.0], [0.0])
    assert oracle.stopping_test([5], 4, 1, [1.0], [1.0], sq, mag, 0.0, 0.5)[0].tolist() == [0]      # 7 < 7.5 but R_dual = 0 < 0 fails
    mag[3, 0] = 1.0                                   # any dual magnitude makes eps_dual positive
    assert oracle.stopping_test([5], 4, 1, [1.0], [1.0], sq, mag, 0.0, 0.5)[0].tolist() == [1]      # 7 < 7.5
    assert oracle.stopping_test([5], 4, 1, [1.0], [1.0], sq, mag, 0.0, 0.4375)[0].tolist() == [0]   # 7 < 6.5625 fails
    # with the stacks the other way round (||A x|| larger) the threshold follows ||A x||
    mag2 = _col([400.0], [0.0], [81.0], [1.0], [0.0])        # ||A x|| = 20, ||B z|| = 9
    assert oracle.stopping_test([5], 4, 1, [1.0], [1.0], sq, mag2, 0.0, 0.375)[0].tolist() == [1]   # 7 < 7.5
    assert oracle.stopping_test([5], 4, 1, [1.0], [1.0], sq, mag2, 0.0, 0.3125)[0].tolist() == [0]  # 7 < 6.25 fails
    # dual threshold: ||A^T y|| = sqrt(rho_1^2 * 16 + rho_2^2 * 9) with rho_1 = 3, rho_2 = 4 -> sqrt(144 + 144) = 12 sqrt 2
    dsq = _col([0.0], [0.0], [0.0], [4.0])            # R_dual = rho_2 * 2 = 8
    dmag = _col([1.0], [1.0], [1.0], [16.0], [9.0])
    assert oracle.stopping_test([5], 4, 1, [3.0], [4.0], dsq, dmag, 0.0, 0.5)[0].tolist() == [1]    # 8 < 8.485
    assert oracle.stopping_test([5], 4, 1, [3.0], [4.0], dsq, dmag, 0.0, 0.46875)[0].tolist() == [0]  # 8 < 7.95 fails
    # were the duals taken scaled (without rho), the threshold would be 0.5 * 5 = 2.5 and the first case would fail


def test_the_residual_totals_count_replicas_and_nodes():
    mag = _col([0.0], [0.0], [0.0], [0.0], [0.0])
    # eps = sqrt((P + 1) n n_out) eps_abs.  P = 3, n = 3, n_out = 1: p = 12 -> eps = sqrt(12) = 3.46 with eps_abs = 1
    # R_dual = sqrt(P rho_1^2 sq_1) = sqrt(3 * 1 * 4) = 3.46.. equal to eps: compare squares exactly: 12 < 12 false
    sq = _col([0.0], [4.0], [0.0], [0.0])
    assert oracle.stopping_test([3], 3, 1, [1.0], [1.0], sq, mag, 1.0, 0.0)[0].tolist() == [0]
    assert oracle.stopping_test([3], 3, 1, [1.0], [1.0], _col([0.0], [3.9], [0.0], [0.0]), mag, 1.0, 0.0)[0].tolist() == [1]
    # without the factor P the first case would read sqrt(4) = 2 < 3.46 and pass
    # two nodes: p = (3 + 1) * 3 * 2 = 24; inter dual counts n_out: R_dual = sqrt(2 * 1 * 12) = sqrt(24): not below
    sq = _col([0.0], [0.0], [0.0], [12.0])
    assert oracle.stopping_test([3], 3, 2, [1.0], [1.0], sq, mag, 1.0, 0.0)[0].tolist() == [0]
    assert oracle.stopping_test([3], 3, 2, [1.0], [1.0], _col([0.0], [0.0], [0.0], [11.9]), mag, 1.0, 0.0)[0].tolist() == [1]
    # the same sum seen by one node: sqrt(12) < sqrt(12) fails as well, sqrt(11.9) passes
    assert oracle.stopping_test([3], 3, 1, [1.0], [1.0], sq, mag, 1.0, 0.0)[0].tolist() == [0]


def test_layers_are_judged_separately_and_the_overall_flag_needs_all_of_them():
    sq = _col([1.0, 100.0, 1.0], [0.0, 0.0, 0.0], [0.0, 0.0, 0.0], [0.0, 0.0, 0.0])
    mag = np.ones((5, 3))
    done, every = oracle.stopping_test([4, 4, 4], 1, 1, [1.0] * 3, [1.0] * 3, sq, mag, 1.0, 0.0)     # eps = sqrt(8)
    assert done.tolist() == [1, 0, 1] and not every
    done, every = oracle.stopping_test([4, 400, 4], 1, 1, [1.0] * 3, [1.0] * 3, sq, mag, 1.0, 0.0)   # layer 1: eps = sqrt(800)
    assert done.tolist() == [1, 1, 1] and every


def test_against_the_formulas_in_numpy_on_random_inputs():
    rng = np.random.default_rng(5)
    for trial in range(50):
        L = int(rng.integers(1, 20))
        P, n_out = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        n = rng.integers(1, 10 ** 6, L)
        rho1, rho2 = 10.0 ** rng.uniform(-3, 1, L), 10.0 ** rng.uniform(-4, 1, L)
        sq, mag = 10.0 ** rng.uniform(-8, 2, (4, L)), 10.0 ** rng.uniform(-2, 4, (5, L))
        ea, er = float(10.0 ** rng.uniform(-6, -2)), float(10.0 ** rng.uniform(-5, -1))
        done, every = oracle.stopping_test(n, P, n_out, rho1, rho2, sq, mag, ea, er)
        r_pri = np.sqrt(sq[0] + sq[2])
        r_dual = np.sqrt(P * rho1 ** 2 * sq[1] + n_out * rho2 ** 2 * sq[3])
        root_p = np.sqrt((P + 1.0) * n * n_out)
        e_pri = root_p * ea + er * np.maximum(np.sqrt(mag[0] + mag[1]), np.sqrt(P * mag[1] + n_out * mag[2]))
        e_dual = root_p * ea + er * np.sqrt(rho1 ** 2 * mag[3] + rho2 ** 2 * mag[4])
        clear = (np.abs(r_pri - e_pri) > 1e-12 * e_pri) & (np.abs(r_dual - e_dual) > 1e-12 * e_dual)
        want = (r_pri < e_pri) & (r_dual < e_dual)
        assert np.array_equal(done[clear] != 0, want[clear]), trial
        if clear.all():
            assert every == bool(want.all())


def test_scale_invariance_and_monotony():
    """Multiplying every vector of the iteration by c multiplies residual norms and relative thresholds by c; with the
    absolute tolerance multiplied by c as well, no decision changes.  A looser tolerance never un-converges a layer."""
    rng = np.random.default_rng(9)
    L = 40
    n = rng.integers(10, 10 ** 5, L)
    rho1, rho2 = 10.0 ** rng.uniform(-3, 1, L), 10.0 ** rng.uniform(-4, 1, L)
    sq, mag = 10.0 ** rng.uniform(-6, 0, (4, L)), 10.0 ** rng.uniform(-2, 2, (5, L))
    base, _ = oracle.stopping_test(n, 4, 1, rho1, rho2, sq, mag, 1e-3, 1e-2)
    assert 0 < base.sum() < L                                 # the inputs do split the layers
    for c in (4.0, 0.25):
        again, _ = oracle.stopping_test(n, 4, 1, rho1, rho2, sq * c * c, mag * c * c, 1e-3 * c, 1e-2)
        assert np.array_equal(again, base)
    looser, _ = oracle.stopping_test(n, 4, 1, rho1, rho2, sq, mag, 2e-3, 2e-2)
    assert np.all(looser >= base) and looser.sum() > base.sum()


def test_rejects_bad_arguments():
    ok = dict(n_elems=[4], P=1, n_out=1, rho1=[1.0], rho2=[1.0], sq=np.zeros((4, 1)), mag=np.ones((5, 1)),
              eps_abs=1e-3, eps_rel=1e-3)
    oracle.stopping_test(**ok)
    for key, bad in (("P", 0), ("n_out", 0), ("rho1", [0.0]), ("rho2", [-1.0]), ("eps_abs", -1.0),
                     ("eps_rel", float("nan")), ("n_elems", [0]), ("sq", -np.ones((4, 1))),
                     ("mag", np.full((5, 1), np.nan))):
        args = dict(ok)
        args[key] = bad
        with pytest.raises(ValueError):
            oracle.stopping_test(**args)


# ------------------------------------------------------------------ layer-wise squared norms

def test_layer_sqnorms_handworked_and_against_numpy():
    # two layers [2,1,2] and [1,3,1] at offsets 0 and 4: sums of squares 1 + 4 + 9 + 16 = 30 and 0.25 + 4 + 36 = 40.25
    t = {"elem_off": np.array([0, 4], np.int64), "c_out": np.array([2, 1], np.int32), "c_in": np.array([1, 3], np.int32),
         "khw": np.array([2, 1], np.int32), "mode": np.array([1, 0], np.int32), "k": np.array([1, 1], np.int32)}
    X = np.array([1, -2, 3, 4, 0.5, 2, -6, 1e30], np.float32)           # the last element is arena padding
    assert oracle.layer_sqnorms(t, X).tolist() == [30.0, 40.25]
    rng = np.random.default_rng(2)
    for trial in range(5):
        wl = wk.custom_workload(random_table(rng, 6), R=1, seed=trial)
        X = rng.standard_normal(wl.n_arena).astype(np.float32)
        got = oracle.layer_sqnorms(wl.table(), X)
        for li, l in enumerate(wl.layers):
            seg = X[l.elem_off:l.elem_off + l.n].astype(np.float64)
            assert got[li] == pytest.approx(float(np.sum(seg * seg)), rel=1e-13)
            assert got[li] == pytest.approx(math.fsum((seg * seg).tolist()), rel=1e-13)


def test_layer_sqnorms_tie_the_residual_rows_together():
    """||z_i - 0||^2 through the residual function equals the layer norms of z_i: the two functions agree where their
    definitions meet."""
    rng = np.random.default_rng(4)
    wl = wk.custom_workload(random_table(rng, 5), R=1, seed=3)
    t = wl.table()
    Zi = rng.standard_normal(wl.n_arena).astype(np.float32)
    zero = np.zeros(wl.n_arena, np.float32)
    sq = oracle.residuals(t, Zi[None, :], zero, Zi, None, None)            # row 0: ||theta - 0||^2 with theta = z_i
    assert np.array_equal(sq[0], oracle.layer_sqnorms(t, Zi))
