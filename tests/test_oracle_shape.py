"""Pins of the oracle's shape-sparsity mode (Section 2.1: groups W[:, b, u, v], one per input channel and spatial
position).  CPU only.  Such a group is one column of the layer's [c_out][c_in*khw] GEMM view, so the mode must agree
bit for bit with the (separately pinned) channel mode applied to the layer declared as (c_out, c_in*khw, khw = 1)."""
import json

import numpy as np
import pytest

import oracle
import workloads as wk
from tests.test_oracle_pins import GOLDEN, one_layer_table

CASE = json.load(open(GOLDEN))["shape_case"]


def _random_shape_workload(rng, seed, R):
    shapes = []
    for _ in range(7):
        co, ci = int(rng.integers(1, 30)), int(rng.integers(1, 20))
        khw = int(rng.choice([1, 4, 9, 49]))
        mode = int(rng.choice([0, 1, 2, 4, 4, 4]))
        G = {0: co, 1: co, 2: ci, 4: ci * khw}[mode]
        shapes.append((co, ci, khw, mode, int(rng.integers(1, G + 1))))
    return wk.custom_workload(shapes, R=R, seed=seed, sigma_replica=0.04)


def test_handworked_shape_layer():
    c = CASE
    t = one_layer_table(c["c_out"], c["c_in"], c["khw"], c["mode"], c["k"])
    W = np.array(c["W"], np.float32)
    U = np.array(c["U"], np.float32)
    out = oracle.project(t, W, U)
    assert out["key"].tolist() == [float(x) for x in c["key"]]
    assert out["mask"].tolist() == c["mask"]
    assert out["Z"].tolist() == [float(x) for x in c["Z"]]
    assert out["U"].tolist() == [float(x) for x in c["U_new"]]
    p = oracle.compact(t, out["Z"], out["mask"])
    assert p["packed"].tolist() == [float(x) for x in c["packed"]]
    assert p["layer_off"].tolist() == c["layer_off"] and p["kept_idx"].tolist() == c["kept_idx"]
    assert oracle.expand(t, p["packed"], out["mask"], W.shape[1]).tolist() == [float(x) for x in c["Z"]]
    f = oracle.project_frozen(t, W, U, np.array(c["frozen"]["mask"], np.uint8))
    assert f["Z"].tolist() == [float(x) for x in c["frozen"]["Z"]]
    assert f["U"].tolist() == [float(x) for x in c["frozen"]["U_new"]]


@pytest.mark.parametrize("seed", range(4))
def test_shape_groups_are_the_columns_of_the_gemm_view(seed):
    rng = np.random.default_rng(700 + seed)
    wl = _random_shape_workload(rng, seed, R=int(rng.integers(1, 4)))
    W, U = wk.generate(wl)
    a = oracle.project(wl.table(), W, U, want_wbar=True)
    b = oracle.project(wl.gemm_view_table(), W, U, want_wbar=True)
    assert np.array_equal(a["mask"], b["mask"])
    assert np.array_equal(a["key"].view(np.uint64), b["key"].view(np.uint64))
    for name in ("Z", "U", "Wbar"):
        assert np.array_equal(a[name].view(np.uint32), b[name].view(np.uint32)), name
    for align in (1, 5):
        ca = oracle.compact(wl.table(), a["Z"], a["mask"], pack_align=align)
        cb = oracle.compact(wl.gemm_view_table(), a["Z"], a["mask"], pack_align=align)
        for name in ("packed", "layer_off", "kept_idx"):
            assert np.array_equal(ca[name], cb[name]), name
        ea = oracle.expand(wl.table(), ca["packed"], a["mask"], wl.n_arena, pack_align=align)
        assert np.array_equal(ea.view(np.uint32), a["Z"].view(np.uint32))
    m = (rng.random(wl.groups_total) < 0.5).astype(np.uint8) * 2
    fa = oracle.project_frozen(wl.table(), W, U, m)
    fb = oracle.project_frozen(wl.gemm_view_table(), W, U, m)
    assert np.array_equal(fa["Z"].view(np.uint32), fb["Z"].view(np.uint32))
    assert np.array_equal(fa["U"].view(np.uint32), fb["U"].view(np.uint32))
    L = len(wl.layers)
    Zg = (0.05 * rng.standard_normal(wl.n_arena)).astype(np.float32)
    Vd = (0.01 * rng.standard_normal(wl.n_arena)).astype(np.float32)
    ca_, cb_ = rng.uniform(0.5, 1, L).astype(np.float32), rng.uniform(0, 0.5, L).astype(np.float32)
    wa = oracle.project_weighted(wl.table(), W, U, Zg, Vd, ca_, cb_)
    wb = oracle.project_weighted(wl.gemm_view_table(), W, U, Zg, Vd, ca_, cb_)
    assert np.array_equal(wa["mask"], wb["mask"]) and np.array_equal(wa["Z"].view(np.uint32), wb["Z"].view(np.uint32))


@pytest.mark.parametrize("seed", range(3))
def test_shape_against_numpy(seed):
    """Keys by numpy.sum over the filter axis, selection by stable argsort, zeroing by broadcasting (c_in, khw) masks."""
    rng = np.random.default_rng(800 + seed)
    co, ci, khw = int(rng.integers(2, 20)), int(rng.integers(1, 12)), int(rng.choice([4, 9]))
    k = int(rng.integers(1, ci * khw + 1))
    wl = wk.custom_workload([(co, ci, khw, wk.MODE_SHAPE, k)], R=2, seed=seed, sigma_replica=0.05)
    W, U = wk.generate(wl)
    out = oracle.project(wl.table(), W, U, want_wbar=True)
    V = (out["Wbar"] + U).astype(np.float32).reshape(co, ci, khw)
    key = np.sum(V.astype(np.float64) ** 2, axis=0).reshape(-1)
    np.testing.assert_allclose(out["key"], key, rtol=1e-12)
    m = np.zeros(ci * khw, np.uint8)
    m[np.argsort(-key, kind="stable")[:k]] = 1
    assert np.array_equal(out["mask"], m)
    Z = np.where(m.reshape(1, ci, khw).astype(bool), V, np.float32(0)).reshape(-1)
    assert np.array_equal(out["Z"].view(np.uint32), Z.astype(np.float32).view(np.uint32))
    assert int((np.abs(out["Z"].reshape(co, ci * khw)).sum(axis=0) > 0).sum()) <= k
    c = oracle.compact(wl.table(), out["Z"], out["mask"])
    assert np.array_equal(c["packed"], out["Z"].reshape(co, ci * khw)[:, m.astype(bool)].reshape(-1))


def test_shape_with_unit_spatial_extent_is_channel_sparsity():
    wl = wk.custom_workload([(9, 13, 1, wk.MODE_SHAPE, 5)], R=2, seed=1, sigma_replica=0.05)
    wc = wk.custom_workload([(9, 13, 1, wk.MODE_CHANNEL, 5)], R=2, seed=1, sigma_replica=0.05)
    W, U = wk.generate(wl)
    a, b = oracle.project(wl.table(), W, U), oracle.project(wc.table(), W, U)
    assert np.array_equal(a["mask"], b["mask"]) and np.array_equal(a["Z"], b["Z"]) and np.array_equal(a["U"], b["U"])
