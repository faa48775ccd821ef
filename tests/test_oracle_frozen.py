"""Pins of the oracle's frozen-mask projection (Algorithm 1 Phase 3, retraining branch; Section 4.5) and of the
mask union (Eq. (14)).  CPU only."""
import json
import os

import numpy as np
import pytest

import oracle
import workloads as wk
from tests.test_oracle_pins import one_layer_table, random_table, GOLDEN


def test_handworked_frozen_masks():
    g = json.load(open(GOLDEN))
    base = {c["name"]: c for c in g["cases"]}[g["frozen_cases"]["base"]]
    t = one_layer_table(base["c_out"], base["c_in"], base["khw"], base["mode"], base["k"])
    W = np.array(base["W"], dtype=np.float32)
    U = np.array(base["U"], dtype=np.float32)
    for c in g["frozen_cases"]["cases"]:
        out = oracle.project_frozen(t, W, U, np.array(c["mask"], np.uint8), want_wbar=True)
        assert out["Z"].tolist() == [float(x) for x in c["Z"]]
        assert out["U"].tolist() == [float(x) for x in c["U_new"]]
        assert out["Wbar"].tolist() == [float(x) for x in base["Wbar"]]


@pytest.mark.parametrize("seed", range(4))
def test_frozen_with_the_projections_own_mask_is_the_projection(seed):
    """Applying the mask the projection selected gives the projection back (Z, U, Wbar bit for bit)."""
    rng = np.random.default_rng(40 + seed)
    wl = wk.custom_workload(random_table(rng, 8), R=int(rng.integers(1, 5)), seed=seed, sigma_replica=0.03)
    W, U = wk.generate(wl)
    a = oracle.project(wl.table(), W, U, want_wbar=True)
    b = oracle.project_frozen(wl.table(), W, U, a["mask"], want_wbar=True)
    for name in ("Z", "U", "Wbar"):
        assert np.array_equal(a[name].view(np.uint32), b[name].view(np.uint32)), name


@pytest.mark.parametrize("seed", range(4))
def test_frozen_against_the_printed_formula_in_numpy(seed):
    """z = z~ (.) m evaluated with a broadcast multiply; values equal, masked-out entries carry a + sign."""
    rng = np.random.default_rng(60 + seed)
    wl = wk.custom_workload(random_table(rng, 6, allow_none=False), R=3, seed=seed, sigma_replica=0.03)
    W, U = wk.generate(wl)
    mask = (rng.random(wl.groups_total) < 0.5).astype(np.uint8) * 5      # any nonzero byte = kept
    out = oracle.project_frozen(wl.table(), W, U, mask, want_wbar=True)
    acc = W[0].copy()
    for r in range(1, 3):
        acc = (acc + W[r]).astype(np.float32)
    wbar = (acc * (np.float32(1) / np.float32(3))).astype(np.float32)
    V = (wbar + U).astype(np.float32)
    for l in wl.layers:
        sl = slice(l.elem_off, l.elem_off + l.n)
        m = (mask[l.group_base:l.group_base + l.groups] != 0).astype(np.float32)
        m3 = m[None, :, None] if l.mode == wk.MODE_CHANNEL else m[:, None, None]
        z_formula = (V[sl].reshape(l.c_out, l.c_in, l.khw) * m3).reshape(-1)
        z = out["Z"][sl]
        assert np.array_equal(z, z_formula)                        # -0 == +0 here
        pruned = np.broadcast_to(m3 == 0, (l.c_out, l.c_in, l.khw)).reshape(-1)
        assert not np.signbit(z[pruned]).any()                     # exactly +0 where masked out
        u_formula = (U[sl] + (wbar[sl] - z).astype(np.float32)).astype(np.float32)
        assert np.array_equal(out["U"][sl].view(np.uint32), u_formula.view(np.uint32))


def test_all_ones_mask_and_unconstrained_layers():
    """m_global is initialised to all ones (Algorithm 1, Initialize): then z = z~.  An unconstrained layer keeps
    everything whatever its mask bytes are."""
    wl = wk.custom_workload([(6, 5, 4, wk.MODE_FILTER, 2), (4, 6, 1, wk.MODE_CHANNEL, 2), (3, 3, 1, wk.MODE_NONE, 3)],
                            R=2, seed=3, sigma_replica=0.03)
    W, U = wk.generate(wl)
    ones = np.ones(wl.groups_total, np.uint8)
    out = oracle.project_frozen(wl.table(), W, U, ones, want_wbar=True)
    assert np.array_equal(out["Z"].view(np.uint32), (out["Wbar"] + U).astype(np.float32).view(np.uint32))
    zeros = np.zeros(wl.groups_total, np.uint8)
    out0 = oracle.project_frozen(wl.table(), W, U, zeros)
    last = wl.layers[2]
    sl = slice(last.elem_off, last.elem_off + last.n)
    assert np.array_equal(out0["Z"][sl], out["Z"][sl])             # mode none ignores the mask
    assert not out0["Z"][:wl.layers[2].elem_off].any()


def test_mask_union_is_the_logical_or():
    rng = np.random.default_rng(8)
    masks = [(rng.random(1000) < p).astype(np.uint8) * v for p, v in ((0.2, 1), (0.3, 7), (0.1, 255), (0.0, 1))]
    out = oracle.mask_or(masks)
    assert np.array_equal(out, np.logical_or.reduce([m != 0 for m in masks]).astype(np.uint8))
    assert set(np.unique(out)) <= {0, 1}
    assert np.array_equal(oracle.mask_or([masks[0], masks[0]]), (masks[0] != 0).astype(np.uint8))
    # union of two top-k masks keeps at least k and at most 2k groups per layer, and contains both
    wl = wk.make_workload("tiny")
    W, U = wk.generate(wl)
    a = oracle.project(wl.table(), W, U)["mask"]
    wl2 = wk.make_workload("tiny", seed=5)
    W2, U2 = wk.generate(wl2)
    b = oracle.project(wl.table(), W2, U2)["mask"]
    u = oracle.mask_or([a, b])
    assert np.all(u >= a) and np.all(u >= b)
    for l in wl.layers:
        c = int(u[l.group_base:l.group_base + l.groups].sum())
        assert l.k <= c <= min(2 * l.k, l.groups)


def test_mask_drift_counts_changed_groups_per_layer():
    """Section 4.5: stability of the sparsity pattern = no group changes its kept flag between iterations."""
    wl = wk.custom_workload([(6, 2, 1, wk.MODE_FILTER, 3), (2, 5, 4, wk.MODE_CHANNEL, 2), (3, 3, 1, wk.MODE_NONE, 3),
                             (4, 3, 1, wk.MODE_BOTH, 2, 2)], R=1)
    a = np.array([1, 1, 1, 0, 0, 0] + [1, 0, 1, 0, 0] + [0, 0, 0] + [1, 1, 0, 0, 1, 1, 0], np.uint8)
    b = np.array([1, 0, 1, 9, 0, 0] + [0, 1, 1, 0, 0] + [1, 1, 1] + [1, 1, 0, 0, 0, 1, 7], np.uint8)
    assert oracle.mask_drift(wl.table(), a, b).tolist() == [2, 2, 0, 2]
    assert oracle.mask_drift(wl.table(), a, a * 200).tolist() == [0, 0, 0, 0]     # any nonzero byte is "kept"
    rng = np.random.default_rng(2)
    wl2 = wk.custom_workload(random_table(rng, 9), R=1)
    x = (rng.random(wl2.groups_total) < 0.5).astype(np.uint8)
    y = (rng.random(wl2.groups_total) < 0.5).astype(np.uint8) * 3
    d = oracle.mask_drift(wl2.table(), x, y)
    for l, dl in zip(wl2.layers, d):
        sl = slice(l.group_base, l.group_base + l.groups)
        assert dl == (0 if l.mode == wk.MODE_NONE else int(np.count_nonzero((x[sl] != 0) ^ (y[sl] != 0))))
    # two successive projections of the same inputs select the same groups: no drift
    W, U = wk.generate(wl2)
    m = oracle.project(wl2.table(), W, U)["mask"]
    assert not oracle.mask_drift(wl2.table(), m, m).any()
