"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP path.  Each is chosen so that a plausible
mistake in oracle/hsadmm_oracle.c (dropped term, wrong sign or index, transposed
group axis, wrong tie rule, wrong parenthesisation) fails at least one.
"""
import itertools
import json
import os

import numpy as np
import pytest

import oracle
import workloads as wk
from tests import ref_numpy as ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "handworked_layers.json")


def one_layer_table(co, ci, khw, mode, k, off=0):
    return {"elem_off": np.array([off], np.int64), "c_out": np.array([co], np.int32),
            "c_in": np.array([ci], np.int32), "khw": np.array([khw], np.int32),
            "mode": np.array([mode], np.int32), "k": np.array([k], np.int32)}


def load_cases():
    with open(GOLDEN) as f:
        return json.load(f)


CASES = load_cases()["cases"]


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
def test_handworked_layer(case):
    t = one_layer_table(case["c_out"], case["c_in"], case["khw"], case["mode"], case["k"])
    W = np.array(case["W"], dtype=np.float32)
    U = np.array(case["U"], dtype=np.float32)
    out = oracle.project(t, W, U, want_wbar=True)
    assert out["key"].tolist() == [float(x) for x in case["key"]]
    assert out["mask"].tolist() == case["mask"]
    assert out["Wbar"].tolist() == [float(x) for x in case["Wbar"]]
    assert out["Z"].tolist() == [float(x) for x in case["Z"]]
    assert out["U"].tolist() == [float(x) for x in case["U_new"]]
    c = oracle.compact(t, out["Z"], out["mask"])
    assert c["packed"].tolist() == [float(x) for x in case["packed"]]
    assert c["layer_off"].tolist() == case["layer_off"]
    assert c["kept_idx"].tolist() == case["kept_idx"]
    back = oracle.expand(t, c["packed"], out["mask"], W.shape[1])
    assert back.tolist() == [float(x) for x in case["Z"]]


def test_handworked_two_layer_offsets_and_alignment():
    g = load_cases()
    by_name = {c["name"]: c for c in g["cases"]}
    a, e = (by_name[n] for n in g["two_layer_offsets"]["layers"])
    # layer A at element 0, layer E at element 8 of one arena
    t = {"elem_off": np.array([0, 8], np.int64),
         "c_out": np.array([a["c_out"], e["c_out"]], np.int32),
         "c_in": np.array([a["c_in"], e["c_in"]], np.int32),
         "khw": np.array([a["khw"], e["khw"]], np.int32),
         "mode": np.array([a["mode"], e["mode"]], np.int32),
         "k": np.array([a["k"], e["k"]], np.int32)}
    W = np.array([a["W"][0] + e["W"][0]], dtype=np.float32)
    U = np.zeros(W.shape[1], dtype=np.float32)
    out = oracle.project(t, W, U)
    assert out["mask"].tolist() == a["mask"] + e["mask"]
    assert out["Z"].tolist() == [float(x) for x in a["Z"] + e["Z"]]
    for align, offs in g["two_layer_offsets"]["by_pack_align"].items():
        c = oracle.compact(t, out["Z"], out["mask"], pack_align=int(align))
        assert c["layer_off"].tolist() == offs
        assert c["kept_idx"].tolist() == g["two_layer_offsets"]["kept_idx"]
        assert c["packed"][offs[0]:offs[0] + 4].tolist() == [float(x) for x in a["packed"]]
        assert c["packed"][offs[1]:offs[1] + 8].tolist() == [float(x) for x in e["packed"]]
        back = oracle.expand(t, c["packed"], out["mask"], W.shape[1], pack_align=int(align))
        assert np.array_equal(back, out["Z"])


@pytest.mark.parametrize("mode", [wk.MODE_FILTER, wk.MODE_CHANNEL])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_projection_is_the_euclidean_projection_by_brute_force(mode, seed):
    """Eq. (10): Z is the closest point (Frobenius) with at most k nonzero groups.

    Every support of size k is enumerated on a tiny layer; the oracle's distance must be the minimum
    and must equal the sum of the G-k smallest squared group norms."""
    rng = np.random.default_rng(seed)
    co, ci, khw = (6, 3, 2) if mode == wk.MODE_FILTER else (3, 7, 2)
    G = co if mode == wk.MODE_FILTER else ci
    for k in range(1, G + 1):
        t = one_layer_table(co, ci, khw, mode, k)
        W = rng.standard_normal((1, co * ci * khw)).astype(np.float32)
        U = (0.1 * rng.standard_normal(co * ci * khw)).astype(np.float32)
        out = oracle.project(t, W, U)
        V = (W[0] + U).astype(np.float32).astype(np.float64).reshape(co, ci, khw)
        Z = out["Z"].astype(np.float64).reshape(co, ci, khw)
        d_oracle = np.sum((V - Z) ** 2)
        best = np.inf
        for keep in itertools.combinations(range(G), k):
            m = np.zeros(G)
            m[list(keep)] = 1
            m3 = m[:, None, None] if mode == wk.MODE_FILTER else m[None, :, None]
            best = min(best, np.sum((V - V * m3) ** 2))
        assert d_oracle == pytest.approx(best, rel=1e-12, abs=1e-300)
        axis = (1, 2) if mode == wk.MODE_FILTER else (0, 2)
        keys = np.sort(np.sum(V * V, axis=axis))
        assert d_oracle == pytest.approx(np.sum(keys[:G - k]), rel=1e-12, abs=1e-300)
        assert int(out["mask"].sum()) == k


def random_table(rng, n_layers, allow_none=True):
    shapes = []
    for _ in range(n_layers):
        co = int(rng.integers(1, 40))
        ci = int(rng.integers(1, 40))
        khw = int(rng.choice([1, 1, 4, 9, 49]))
        mode = int(rng.choice([0, 1, 2] if allow_none else [1, 2]))
        G = ci if mode == wk.MODE_CHANNEL else co
        k = int(rng.integers(1, G + 1))
        shapes.append((co, ci, khw, mode, k))
    return shapes


@pytest.mark.parametrize("seed", range(6))
def test_against_numpy_library_routines(seed):
    """Keys vs numpy.sum in float64, selection vs stable argsort, pack vs numpy.ix_, expand vs index assignment."""
    rng = np.random.default_rng(100 + seed)
    R = int(rng.integers(1, 6))
    wl = wk.custom_workload(random_table(rng, 7), R=R, seed=seed, sigma_replica=0.03)
    W, U = wk.generate(wl)
    t = wl.table()
    a = oracle.project(t, W, U, want_wbar=True)
    b = ref.project(t, W, U)
    np.testing.assert_allclose(a["key"], b["key"], rtol=1e-12)
    assert np.array_equal(a["mask"], b["mask"])
    for name in ("Wbar", "Z", "U"):
        assert np.array_equal(a[name].view(np.uint32), b[name].view(np.uint32)), name
    for align in (1, 4, 7):
        ca = oracle.compact(t, a["Z"], a["mask"], pack_align=align)
        cb = ref.compact(t, a["Z"], a["mask"], pack_align=align)
        assert np.array_equal(ca["layer_off"], cb["layer_off"])
        assert np.array_equal(ca["kept_idx"], cb["kept_idx"])
        assert np.array_equal(ca["packed"].view(np.uint32), cb["packed"].view(np.uint32))
        ea = oracle.expand(t, ca["packed"], a["mask"], wl.n_arena, pack_align=align)
        eb = ref.expand(t, ca["packed"], a["mask"], wl.n_arena, pack_align=align)
        assert np.array_equal(ea.view(np.uint32), eb.view(np.uint32))
        assert np.array_equal(ea.view(np.uint32), a["Z"].view(np.uint32))   # expand(compact(Z)) == Z


def test_compact_takes_an_arbitrary_source_and_mask():
    """Compaction under a mask that is not the layer's own top-k (a union of masks keeps more than k)."""
    rng = np.random.default_rng(5)
    wl = wk.custom_workload([(9, 5, 4, wk.MODE_FILTER, 3), (6, 11, 1, wk.MODE_CHANNEL, 2),
                             (4, 4, 9, wk.MODE_NONE, 4)], R=1, seed=3)
    t = wl.table()
    src = rng.standard_normal(wl.n_arena).astype(np.float32)
    mask = (rng.random(wl.groups_total) < 0.6).astype(np.uint8)
    mask[9 + 11:] = 1
    ca = oracle.compact(t, src, mask)
    cb = ref.compact(t, src, mask)
    assert np.array_equal(ca["layer_off"], cb["layer_off"])
    assert np.array_equal(ca["kept_idx"], cb["kept_idx"])
    assert np.array_equal(ca["packed"], cb["packed"])
    # all-zero mask on a constrained layer: nothing packed, expansion is all zeros
    mask0 = mask.copy()
    mask0[:9] = 0
    c0 = oracle.compact(t, src, mask0)
    assert c0["layer_off"][1] == 0
    e0 = oracle.expand(t, c0["packed"], mask0, wl.n_arena)
    assert not e0[:9 * 5 * 4].any()


def test_ties_identical_groups_resolve_by_lower_index():
    co, ci, khw = 8, 5, 4
    rng = np.random.default_rng(7)
    base = rng.standard_normal((co, ci * khw)).astype(np.float32)
    base[5] = base[1]
    base[6] = base[1]
    base[1] *= 1.0
    # make group 1/5/6 straddle the cut: find k so that the k-th slot falls inside the tie
    keys = np.sum(base.astype(np.float64) ** 2, axis=1)
    n_greater = int(np.sum(keys > keys[1]))
    for k, expect in ((n_greater + 1, [1]), (n_greater + 2, [1, 5]), (n_greater + 3, [1, 5, 6])):
        t = one_layer_table(co, ci, khw, wk.MODE_FILTER, k)
        out = oracle.project(t, base.reshape(1, -1), np.zeros(co * ci * khw, np.float32))
        tied_kept = [g for g in (1, 5, 6) if out["mask"][g]]
        assert tied_kept == expect
        assert int(out["mask"].sum()) == k
    # channel mode, same idea
    basec = rng.standard_normal((6, 7, 3)).astype(np.float32)
    basec[:, 4, :] = basec[:, 2, :]
    keysc = np.sum(basec.astype(np.float64) ** 2, axis=(0, 2))
    ng = int(np.sum(keysc > keysc[2]))
    t = one_layer_table(6, 7, 3, wk.MODE_CHANNEL, ng + 1)
    out = oracle.project(t, basec.reshape(1, -1), np.zeros(6 * 7 * 3, np.float32))
    assert out["mask"][2] == 1 and out["mask"][4] == 0


def test_dual_update_parenthesisation_of_eq_12():
    """u+ = u + (theta - z): with theta = 1, u = 1e-8 the kept candidate rounds to 1, theta - z = 0 and
    u+ = u.  The other grouping, (u + theta) - z, would give 0."""
    t = one_layer_table(1, 1, 1, wk.MODE_FILTER, 1)
    W = np.array([[1.0]], dtype=np.float32)
    U = np.array([1e-8], dtype=np.float32)
    out = oracle.project(t, W, U)
    assert out["Z"][0] == np.float32(1.0)
    assert out["U"][0] == np.float32(1e-8)
    assert out["U"][0] != 0


def test_mean_is_left_to_right_sum_times_reciprocal():
    """Reading of Eq. (9)'s normalisation: fp32 sum in replica order, then times fl32(1/R)."""
    t = one_layer_table(1, 1, 1, wk.MODE_NONE, 1)
    W = np.array([[1.0], [2.0], [2.0]], dtype=np.float32)       # sum 5, R = 3
    out = oracle.project(t, W, np.zeros(1, np.float32), want_wbar=True)
    expect = np.float32(5.0) * (np.float32(1.0) / np.float32(3.0))
    assert out["Wbar"][0] == expect
    assert out["Wbar"][0] != np.float32(5.0) / np.float32(3.0)   # the case separates the two readings
    # left-to-right: (2^24 + 1) + 1 loses both ones, 1 + 1 + 2^24 keeps them
    big = np.float32(2 ** 24)
    W1 = np.array([[big], [1.0], [1.0], [0.0]], dtype=np.float32)
    W2 = np.array([[1.0], [1.0], [big], [0.0]], dtype=np.float32)
    o1 = oracle.project(t, W1, np.zeros(1, np.float32), want_wbar=True)["Wbar"][0]
    o2 = oracle.project(t, W2, np.zeros(1, np.float32), want_wbar=True)["Wbar"][0]
    assert o1 == np.float32(2 ** 22) and o2 == np.float32((2 ** 24 + 2) / 4)
    # powers of two: exact division
    for R in (1, 2, 4, 8):
        Wr = np.full((R, 1), 3.25, dtype=np.float32)
        assert oracle.project(t, Wr, np.zeros(1, np.float32), want_wbar=True)["Wbar"][0] == np.float32(3.25)


def test_eq_9_reduces_to_plain_mean_plus_mean_dual():
    """Eq. (9) with lambda = 0 and rho_2 = 0: (1/gamma) rho_1 sum_j (theta_j + u_j), gamma = P rho_1,
    i.e. mean(theta) + mean(u).  Evaluated in float64 from the printed formula and compared with V = Z
    of an unconstrained layer."""
    rng = np.random.default_rng(11)
    P, n = 4, 24
    theta = rng.standard_normal((P, n)).astype(np.float32)
    u = (0.01 * rng.standard_normal((P, n))).astype(np.float32)
    rho1, rho2, lam, M = 1.5e-3, 0.0, 0.0, 16
    gamma = lam / M + P * rho1 + rho2
    z_tilde = (rho1 * np.sum(theta.astype(np.float64) + u.astype(np.float64), axis=0)) / gamma
    ubar = np.mean(u.astype(np.float64), axis=0).astype(np.float32)
    t = one_layer_table(4, 6, 1, wk.MODE_NONE, 4)
    out = oracle.project(t, theta, ubar)
    np.testing.assert_allclose(out["Z"], z_tilde, rtol=0, atol=1e-6)


def test_invariants_on_tiny_and_random_workloads():
    for wl in (wk.make_workload("tiny"),
               wk.custom_workload(random_table(np.random.default_rng(3), 9, allow_none=True), R=3,
                                  seed=9, sigma_replica=0.03)):
        W, U = wk.generate(wl)
        t = wl.table()
        out = oracle.project(t, W, U, want_wbar=True)
        V = (out["Wbar"] + U).astype(np.float32)
        for l in wl.layers:
            m = out["mask"][l.group_base:l.group_base + l.groups]
            key = out["key"][l.group_base:l.group_base + l.groups]
            assert int(m.sum()) == (l.groups if l.mode == wk.MODE_NONE else l.k)
            sl = slice(l.elem_off, l.elem_off + l.n)
            z3 = out["Z"][sl].reshape(l.c_out, l.c_in, l.khw)
            v3 = V[sl].reshape(l.c_out, l.c_in, l.khw)
            u3 = out["U"][sl].reshape(l.c_out, l.c_in, l.khw)
            m3 = m[None, :, None] if l.mode == wk.MODE_CHANNEL else m[:, None, None]
            m3 = np.broadcast_to(m3.astype(bool), z3.shape)
            # kept groups: Z == V bit for bit; pruned groups: Z == +0 and U+ == V bit for bit
            assert np.array_equal(z3[m3].view(np.uint32), v3[m3].view(np.uint32))
            assert not z3[~m3].view(np.uint32).any()
            assert np.array_equal(u3[~m3].view(np.uint32), v3[~m3].view(np.uint32))
            # whole rows / whole columns of the GEMM view are zero (Section 5.5, structured support)
            nz_groups = (np.abs(z3).sum(axis=(0, 2)) > 0) if l.mode == wk.MODE_CHANNEL \
                else (np.abs(z3).sum(axis=(1, 2)) > 0)
            assert int(nz_groups.sum()) == int(m.sum())
            if l.mode != wk.MODE_NONE and l.k < l.groups:
                assert key[m == 1].min() >= key[m == 0].max()
        # conservation: Z + U+ == Wbar + U within one rounding of each side
        lhs = out["Z"].astype(np.float64) + out["U"].astype(np.float64)
        rhs = out["Wbar"].astype(np.float64) + U.astype(np.float64)
        scale = np.maximum(np.abs(out["Wbar"]), np.abs(U)).astype(np.float64)
        assert np.all(np.abs(lhs - rhs) <= 2.0 ** -22 * np.maximum(scale, 1e-30))
        c = oracle.compact(t, out["Z"], out["mask"])
        assert c["layer_off"][0] == 0 and np.all(np.diff(c["layer_off"]) >= 0)
        assert c["layer_off"][-1] == wl.n_kept == c["packed"].size
        p = 0
        for l in wl.layers:
            cnt = l.groups if l.mode == wk.MODE_NONE else l.k
            idx = c["kept_idx"][p:p + cnt]
            assert np.all(np.diff(idx) > 0)
            p += cnt
        assert p == c["kept_idx"].size
        back = oracle.expand(t, c["packed"], out["mask"], wl.n_arena)
        assert np.array_equal(back.view(np.uint32), out["Z"].view(np.uint32))


def test_identity_cases():
    """k = G (and mode none): Z = V, mask all ones, packed = src, expand = identity; R = 1: Wbar = W_0 bitwise.
    Dual variable is unchanged wherever Wbar == Z."""
    wl = wk.custom_workload([(12, 7, 9, wk.MODE_FILTER, 12), (5, 9, 1, wk.MODE_CHANNEL, 9),
                             (3, 4, 4, wk.MODE_NONE, 3)], R=1, seed=2)
    W, U = wk.generate(wl)
    out = oracle.project(wl.table(), W, U, want_wbar=True)
    assert np.array_equal(out["Wbar"].view(np.uint32), W[0].view(np.uint32))
    assert out["mask"].all()
    assert np.array_equal(out["Z"], (W[0] + U).astype(np.float32))
    c = oracle.compact(wl.table(), out["Z"], out["mask"])
    dense = np.concatenate([out["Z"][l.elem_off:l.elem_off + l.n] for l in wl.layers])
    assert np.array_equal(c["packed"], dense)      # arena padding is not packed
    assert np.array_equal(oracle.expand(wl.table(), c["packed"], out["mask"], wl.n_arena), out["Z"])
    U0 = np.zeros_like(U)
    out0 = oracle.project(wl.table(), W, U0)
    assert np.array_equal(out0["Z"], W[0]) and not out0["U"].any()


def test_thread_count_does_not_change_any_bit():
    wl = wk.make_workload("tiny")
    W, U = wk.generate(wl)
    oracle.set_threads(1)
    a = oracle.project(wl.table(), W, U, want_wbar=True)
    ca = oracle.compact(wl.table(), a["Z"], a["mask"])
    oracle.set_threads(5)
    b = oracle.project(wl.table(), W, U, want_wbar=True)
    cb = oracle.compact(wl.table(), b["Z"], b["mask"])
    oracle.set_threads(1)
    for name in ("U", "Z", "Wbar", "mask"):
        assert np.array_equal(a[name], b[name])
    assert np.array_equal(a["key"].view(np.uint64), b["key"].view(np.uint64))
    assert np.array_equal(ca["packed"], cb["packed"])


def test_rejects_bad_arguments_and_non_finite_inputs():
    t = one_layer_table(4, 2, 1, wk.MODE_FILTER, 5)     # k > G
    with pytest.raises(ValueError):
        oracle.project(t, np.zeros((1, 8), np.float32), np.zeros(8, np.float32))
    t = one_layer_table(4, 2, 1, wk.MODE_FILTER, 2)
    W = np.zeros((1, 8), np.float32)
    W[0, 3] = np.nan
    with pytest.raises(ValueError):
        oracle.project(t, W, np.zeros(8, np.float32))
