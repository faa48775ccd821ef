"""Pins of the oracle's modes for the composite sets that involve shape groups together with channels (Section 2.1:
S_c ^ S_s and S_f ^ S_c ^ S_s; the projections applied one after the other, Section 3, paragraph after Eq. (10), in
the order the paper lists the sets: filters, channels, shape groups).  CPU only.

What fixes the modes: hand-worked layers, the special cases that reduce to modes pinned elsewhere (all channels kept:
the shape mode; all positions of the kept channels kept: the channel mode / both constraints; all filters kept: mode
5), the single projections applied literally one after the other with NumPy, brute force over the shape supports, and
invariants (feasibility, conservation, idempotence)."""
import itertools
import json

import numpy as np
import pytest

import oracle
import workloads as wk
from tests.test_oracle_pins import GOLDEN

CASES = json.load(open(GOLDEN))["nested_cases"]


def _table(co, ci, khw, mode, k, k_in, k_kern):
    return {"elem_off": np.array([0], np.int64), "c_out": np.array([co], np.int32), "c_in": np.array([ci], np.int32),
            "khw": np.array([khw], np.int32), "mode": np.array([mode], np.int32), "k": np.array([k], np.int32),
            "k_in": np.array([k_in], np.int32), "k_kern": np.array([k_kern], np.int32)}


def _random_nested_workload(rng, seed, R, modes=(5, 6)):
    shapes = []
    for _ in range(6):
        co, ci = int(rng.integers(1, 24)), int(rng.integers(1, 12))
        khw = int(rng.choice([1, 4, 9]))
        mode = int(rng.choice(modes))
        k_in = int(rng.integers(1, ci + 1))
        shapes.append((co, ci, khw, mode, int(rng.integers(1, co + 1)) if mode == 6 else 0, k_in,
                       int(rng.integers(1, k_in * khw + 1))))
    return wk.custom_workload(shapes, R=R, seed=seed, sigma_replica=0.04)


@pytest.mark.parametrize("c", CASES, ids=[str(i) for i in range(len(CASES))])
def test_handworked_nested_layer(c):
    t = _table(c["c_out"], c["c_in"], c["khw"], c["mode"], c["k"], c["k_in"], c["k_kern"])
    out = oracle.project(t, np.array(c["W"], np.float32), np.array(c["U"], np.float32))
    assert out["key"].tolist() == [float(x) for x in c["key"]]
    assert out["mask"].tolist() == c["mask"]
    assert out["Z"].tolist() == [float(x) for x in c["Z"]]
    assert out["U"].tolist() == [float(x) for x in c["U_new"]]


def _as_mode(wl, fn):
    """A copy of the workload whose layers fn(layer) rewrote (mode and counts)."""
    shapes = [fn(l) for l in wl.layers]
    out = wk.custom_workload(shapes, R=wl.R, seed=wl.seed, sigma_replica=wl.sigma_replica)
    assert [l.elem_off for l in out.layers] == [l.elem_off for l in wl.layers]
    return out


@pytest.mark.parametrize("seed", range(3))
def test_special_cases_reduce_to_the_modes_pinned_elsewhere(seed):
    rng = np.random.default_rng(4100 + seed)
    wl = _random_nested_workload(rng, seed, R=int(rng.integers(1, 4)))
    W, U = wk.generate(wl)

    def same(a, b):
        for name in ("Z", "U"):
            assert np.array_equal(a[name].view(np.uint32), b[name].view(np.uint32)), name

    # every channel kept: the channel projection changes nothing; modes 5 / 6 are the shape mode / filters with shapes
    full = _as_mode(wl, lambda l: (l.c_out, l.c_in, l.khw, l.mode, l.k, l.c_in, l.k_kern))
    a = oracle.project(full.table(), W, U)
    five = _as_mode(wl, lambda l: (l.c_out, l.c_in, l.khw, l.mode, l.k, l.c_in, l.k_kern))
    plain = _as_mode(wl, lambda l: (l.c_out, l.c_in, l.khw, 4, l.k_kern) if l.mode == 5
                     else (l.c_out, l.c_in * l.khw, 1, 3, l.k, l.k_kern))
    b = oracle.project(plain.table(), W, U)
    same(a, b)
    for la, lb in zip(five.layers, plain.layers):
        ma = a["mask"][la.group_base:la.group_base + la.groups]
        mb = b["mask"][lb.group_base:lb.group_base + lb.groups]
        if la.mode == 5:
            assert np.all(ma[:la.c_in] == 1) and np.array_equal(ma[la.c_in:], mb)
        else:
            assert np.array_equal(ma[:la.c_out], mb[:la.c_out]) and np.all(ma[la.c_out:la.c_out + la.c_in] == 1)
            assert np.array_equal(ma[la.c_out + la.c_in:], mb[la.c_out:])

    # every position of the kept channels kept: the shape projection changes nothing; the channel mode / both
    allpos = _as_mode(wl, lambda l: (l.c_out, l.c_in, l.khw, l.mode, l.k, l.k_in, l.k_in * l.khw))
    a = oracle.project(allpos.table(), W, U)
    plain = _as_mode(wl, lambda l: (l.c_out, l.c_in, l.khw, 2, l.k_in) if l.mode == 5
                     else (l.c_out, l.c_in, l.khw, 3, l.k, l.k_in))
    b = oracle.project(plain.table(), W, U)
    same(a, b)
    for la, lb in zip(allpos.layers, plain.layers):
        ma = a["mask"][la.group_base:la.group_base + la.groups]
        mb = b["mask"][lb.group_base:lb.group_base + lb.groups]
        head = la.c_in if la.mode == 5 else la.c_out + la.c_in
        assert np.array_equal(ma[:head], mb)
        chan = ma[head - la.c_in:head]
        assert np.array_equal(ma[head:], np.repeat(chan, la.khw))       # exactly the positions of the kept channels
        ka = a["key"][la.group_base:la.group_base + la.groups]
        kb = b["key"][lb.group_base:lb.group_base + lb.groups]
        assert np.array_equal(ka[:head].view(np.uint64), kb.view(np.uint64))

    # every filter kept: mode 6 is mode 5
    six = _as_mode(wl, lambda l: (l.c_out, l.c_in, l.khw, 6, l.c_out, l.k_in, l.k_kern))
    five = _as_mode(wl, lambda l: (l.c_out, l.c_in, l.khw, 5, 0, l.k_in, l.k_kern))
    a, b = oracle.project(six.table(), W, U), oracle.project(five.table(), W, U)
    same(a, b)
    for la, lb in zip(six.layers, five.layers):
        ma = a["mask"][la.group_base:la.group_base + la.groups]
        assert np.all(ma[:la.c_out] == 1)
        assert np.array_equal(ma[la.c_out:], b["mask"][lb.group_base:lb.group_base + lb.groups])
        assert np.array_equal(a["key"][la.group_base + la.c_out:la.group_base + la.groups].view(np.uint64),
                              b["key"][lb.group_base:lb.group_base + lb.groups].view(np.uint64))


def _topk_mask(key, k):
    order = np.argsort(-key, kind="stable")           # larger key first, lower index first among equals
    m = np.zeros(key.size, np.uint8)
    m[order[:k]] = 1
    return m


@pytest.mark.parametrize("seed", range(3))
def test_against_the_single_projections_applied_literally_with_numpy(seed):
    """Pi_s(Pi_c(Pi_f(V))) with each projection ranking all of its groups on the tensor it is given.  The values
    must agree bit for bit; the masks agree too as long as no zero position is ranked into the kept set."""
    rng = np.random.default_rng(4200 + seed)
    R = int(rng.integers(1, 4))
    wl = _random_nested_workload(rng, seed, R)
    W, U = wk.generate(wl)
    out = oracle.project(wl.table(), W, U, want_wbar=True)
    for l in wl.layers:
        sl = slice(l.elem_off, l.elem_off + l.n)
        acc = W[0][sl].copy()
        for r in range(1, R):
            acc = acc + W[r][sl]
        wbar = acc * np.float32(1.0 / R)
        x = (wbar + U[sl]).reshape(l.c_out, l.c_in, l.khw).copy()
        masks = []
        if l.mode == 6:
            m = _topk_mask(np.einsum("oct,oct->o", x.astype(np.float64), x.astype(np.float64)), l.k)
            x[m == 0] = 0
            masks.append(m)
        m = _topk_mask(np.einsum("oct,oct->c", x.astype(np.float64), x.astype(np.float64)), l.k_in)
        x[:, m == 0, :] = 0
        masks.append(m)
        ks = np.einsum("oct,oct->ct", x.astype(np.float64), x.astype(np.float64)).reshape(-1)
        ms = _topk_mask(ks, l.k_kern)
        x.reshape(l.c_out, -1)[:, ms == 0] = 0
        assert np.array_equal(out["Z"][sl].view(np.uint32), x.reshape(-1).view(np.uint32)), l.name
        assert np.array_equal(out["U"][sl].view(np.uint32), (U[sl] + (wbar - x.reshape(-1))).view(np.uint32))
        got = out["mask"][l.group_base:l.group_base + l.groups]
        head = np.concatenate(masks)
        assert np.array_equal(got[:head.size], head)
        if np.count_nonzero(ks) >= l.k_kern:
            assert np.array_equal(got[head.size:], ms)
        np.testing.assert_allclose(out["key"][l.group_base + head.size:l.group_base + l.groups], ks, rtol=1e-13)


def test_the_shape_selection_is_the_best_one_inside_the_kept_channels_by_brute_force():
    rng = np.random.default_rng(4300)
    for _ in range(12):
        co, ci, khw = int(rng.integers(1, 4)), int(rng.integers(2, 4)), int(rng.integers(1, 4))
        k_in = int(rng.integers(1, ci + 1))
        k_kern = int(rng.integers(1, k_in * khw + 1))
        wl = wk.custom_workload([(co, ci, khw, 5, 0, k_in, k_kern)], R=1, seed=int(rng.integers(1 << 30)))
        W, U = wk.generate(wl)
        out = oracle.project(wl.table(), W, U)
        v = (W[0][:wl.layers[0].n] + U[:wl.layers[0].n]).astype(np.float64).reshape(co, ci * khw)
        mc, ms = out["mask"][:ci], out["mask"][ci:]
        assert int(mc.sum()) == k_in and int(ms.sum()) == k_kern
        cand = [g for g in range(ci * khw) if mc[g // khw]]
        assert all(mc[g // khw] for g in np.flatnonzero(ms))
        col = (v * v).sum(axis=0)
        kept_energy = col[ms != 0].sum()
        best = max(col[list(s)].sum() for s in itertools.combinations(cand, k_kern))
        assert kept_energy >= best * (1 - 1e-12)
        # and the channels are the best k_in channels of V
        chan = col.reshape(ci, khw).sum(axis=1)
        assert chan[mc != 0].sum() >= max(chan[list(s)].sum() for s in itertools.combinations(range(ci), k_in)) * (1 - 1e-12)


@pytest.mark.parametrize("seed", range(2))
def test_invariants_feasibility_conservation_idempotence(seed):
    rng = np.random.default_rng(4400 + seed)
    wl = _random_nested_workload(rng, seed, R=2)
    W, U = wk.generate(wl)
    out = oracle.project(wl.table(), W, U, want_wbar=True)
    for l in wl.layers:
        sl = slice(l.elem_off, l.elem_off + l.n)
        z = out["Z"][sl].reshape(l.c_out, l.c_in, l.khw)
        m = out["mask"][l.group_base:l.group_base + l.groups]
        head = 0
        if l.mode == 6:
            assert int(m[:l.c_out].sum()) == l.k
            assert np.count_nonzero(np.abs(z).sum(axis=(1, 2))) <= l.k
            head = l.c_out
        mc, ms = m[head:head + l.c_in], m[head + l.c_in:]
        assert int(mc.sum()) == l.k_in and int(ms.sum()) == l.k_kern
        assert np.count_nonzero(np.abs(z).sum(axis=(0, 2))) <= l.k_in            # in S_c
        assert np.count_nonzero(np.abs(z).sum(axis=0)) <= l.k_kern               # in S_s
        assert np.all(mc[np.flatnonzero(ms) // l.khw] == 1)                        # shapes inside kept channels
        # Z is V on the support the three masks name, +0 elsewhere; U + Z is conserved: U_new + Z = U + Wbar
        v = (out["Wbar"][sl] + U[sl]).reshape(l.c_out, l.c_in, l.khw)
        keep = ms.reshape(l.c_in, l.khw)[None] != 0
        if l.mode == 6:
            keep = keep & (m[:l.c_out, None, None] != 0)
        want = np.where(keep, v, np.float32(0))
        assert np.array_equal(z.view(np.uint32), want.view(np.uint32))
    # projecting the projected tensor again changes nothing (R = 1, U = 0)
    again = oracle.project(wl.table(), out["Z"][None, :], np.zeros_like(U))
    assert np.array_equal(again["Z"].view(np.uint32), out["Z"].view(np.uint32))


def test_ties_between_identical_channels_and_positions_go_to_the_lower_index():
    co, ci, khw = 3, 4, 2
    wl = wk.custom_workload([(co, ci, khw, 5, 0, 2, 3)], R=1, seed=5)
    W, U = wk.generate(wl)
    w = W[0][:co * ci * khw].reshape(co, ci, khw)
    w[:] = w[:, :1, :1]                                # every position identical: all keys tie
    U[:] = 0
    out = oracle.project(wl.table(), W, U)
    assert out["mask"].tolist() == [1, 1, 0, 0, 1, 1, 1, 0, 0, 0, 0, 0]


def test_weighted_candidate_under_the_nested_modes():
    """The weighted projection takes the same selection code: weights (1, 0) give the base projection; in general
    it is the base projection of one replica equal to the candidate (R = 1, U = 0), with the dual of Eq. (12)."""
    rng = np.random.default_rng(4500)
    wl = _random_nested_workload(rng, 3, R=2)
    W, U = wk.generate(wl)
    L = len(wl.layers)
    Zg = rng.standard_normal(wl.n_arena).astype(np.float32) * 0.05
    Vd = rng.standard_normal(wl.n_arena).astype(np.float32) * 0.01
    one, zero = np.ones(L, np.float32), np.zeros(L, np.float32)
    base = oracle.project(wl.table(), W, U)
    w10 = oracle.project_weighted(wl.table(), W, U, Zg, Vd, one, zero)
    assert np.array_equal(base["mask"], w10["mask"])
    assert np.array_equal(base["Z"].view(np.uint32), w10["Z"].view(np.uint32))
    a = rng.uniform(0.3, 0.9, L).astype(np.float32)
    b = rng.uniform(0.1, 0.7, L).astype(np.float32)
    w = oracle.project_weighted(wl.table(), W, U, Zg, Vd, a, b, want_wbar=True)
    cand = np.zeros(wl.n_arena, np.float32)
    for i, l in enumerate(wl.layers):
        sl = slice(l.elem_off, l.elem_off + l.n)
        t = w["Wbar"][sl] + U[sl]
        q = Zg[sl] - Vd[sl]
        cand[sl] = a[i] * t + b[i] * q
    ref = oracle.project(wl.table(), cand[None, :], np.zeros_like(U))
    assert np.array_equal(ref["mask"], w["mask"])
    for l in wl.layers:
        sl = slice(l.elem_off, l.elem_off + l.n)
        assert np.array_equal(ref["Z"][sl].view(np.uint32), w["Z"][sl].view(np.uint32))
        assert np.array_equal(w["U"][sl].view(np.uint32), (U[sl] + (w["Wbar"][sl] - w["Z"][sl])).view(np.uint32))


def test_bad_counts_and_the_functions_that_do_not_take_these_modes():
    W = np.zeros((1, 8), np.float32)
    U = np.zeros(8, np.float32)
    for k, k_in, k_kern in ((0, 3, 1), (0, 0, 1), (0, 1, 0), (0, 1, 3)):        # c_in = 2, khw = 2
        with pytest.raises(ValueError):
            oracle.project(_table(2, 2, 2, 5, k, k_in, k_kern), W, U)
    with pytest.raises(ValueError):
        oracle.project(_table(2, 2, 2, 6, 3, 1, 1), W, U)
    t = _table(2, 2, 2, 5, 0, 1, 1)
    out = oracle.project(t, W, U)
    with pytest.raises(ValueError):
        oracle.compact(t, out["Z"], out["mask"])
    with pytest.raises(ValueError):
        oracle.project_frozen(t, W, U, out["mask"])
