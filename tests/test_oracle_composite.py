"""Pins of the oracle's composite projection: both constraints on one layer, S = S_f ^ S_c (Section 2.1),
projected by applying the filter projection and then the channel projection to its output (Section 3, the
paragraph after Eq. (10)); packing by the K_out x K_in slicing of Section 4.4.1 (Eq. (15)).  CPU only.

The pins: hand-worked layers, the already pinned single-constraint oracle applied twice, NumPy library
routines, structure where the answer is known in closed form (separable magnitudes), the reductions to a
single constraint, feasibility and conservation invariants."""
import json

import numpy as np
import pytest

import oracle
import workloads as wk
from tests import ref_numpy as ref
from tests.test_oracle_pins import GOLDEN, one_layer_table

G = json.load(open(GOLDEN))["composite_cases"]
CASES = G["cases"]


def both_table(co, ci, khw, k, k_in, off=0):
    t = one_layer_table(co, ci, khw, wk.MODE_BOTH, k, off)
    t["k_in"] = np.array([k_in], np.int32)
    return t


def random_table_with_both(rng, n_layers):
    shapes = []
    for _ in range(n_layers):
        co = int(rng.integers(1, 40))
        ci = int(rng.integers(1, 40))
        khw = int(rng.choice([1, 1, 4, 9, 49]))
        mode = int(rng.choice([0, 1, 2, 3, 3, 3]))
        if mode == wk.MODE_BOTH:
            shapes.append((co, ci, khw, mode, int(rng.integers(1, co + 1)), int(rng.integers(1, ci + 1))))
        else:
            Gn = ci if mode == wk.MODE_CHANNEL else co
            shapes.append((co, ci, khw, mode, int(rng.integers(1, Gn + 1))))
    return shapes


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
def test_handworked_composite_layer(case):
    t = both_table(case["c_out"], case["c_in"], case["khw"], case["k"], case["k_in"])
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


def test_the_selection_depends_on_the_order_and_the_oracle_takes_filters_first():
    """Case G is a counterexample to reading the order remark as a statement about the selection: the channel
    projection followed by the filter projection (both from the single-constraint oracle) ends on another
    support.  The composite oracle must agree with filters-first."""
    case = CASES[0]
    co, ci, khw, k, k_in = (case[x] for x in ("c_out", "c_in", "khw", "k", "k_in"))
    W = np.array(case["W"], dtype=np.float32)
    zero = np.zeros(W.shape[1], np.float32)
    c_first = oracle.project(one_layer_table(co, ci, khw, wk.MODE_CHANNEL, k_in), W, zero)
    then_f = oracle.project(one_layer_table(co, ci, khw, wk.MODE_FILTER, k), c_first["Z"][None, :], zero)
    opp = case["opposite_order_support"]
    assert np.nonzero(then_f["mask"])[0].tolist() == opp["filters"]
    assert np.nonzero(c_first["mask"])[0].tolist() == opp["channels"]
    out = oracle.project(both_table(co, ci, khw, k, k_in), W, zero)
    assert not np.array_equal(out["Z"], then_f["Z"])
    assert out["Z"].tolist() == [float(x) for x in case["Z"]]


@pytest.mark.parametrize("seed", range(5))
def test_composite_is_the_two_single_projections_applied_in_sequence(seed):
    """Pi_S = Pi_{S_c} o Pi_{S_f}: the pinned single-constraint oracle run twice (the second time on the first
    one's Z as the only replica, with a zero dual) gives Z, both mask halves and both key halves bit for bit."""
    rng = np.random.default_rng(300 + seed)
    co, ci, khw = int(rng.integers(2, 30)), int(rng.integers(2, 30)), int(rng.choice([1, 4, 9]))
    k, k_in = int(rng.integers(1, co + 1)), int(rng.integers(1, ci + 1))
    R = int(rng.integers(1, 4))
    wl = wk.custom_workload([(co, ci, khw, wk.MODE_BOTH, k, k_in)], R=R, seed=seed, sigma_replica=0.05)
    W, U = wk.generate(wl)
    out = oracle.project(wl.table(), W, U, want_wbar=True)
    f = oracle.project(one_layer_table(co, ci, khw, wk.MODE_FILTER, k), W, U, want_wbar=True)
    zero = np.zeros_like(U)
    c = oracle.project(one_layer_table(co, ci, khw, wk.MODE_CHANNEL, k_in), f["Z"][None, :], zero)
    assert np.array_equal(out["Z"].view(np.uint32), c["Z"].view(np.uint32))
    assert np.array_equal(out["mask"], np.concatenate([f["mask"], c["mask"]]))
    assert np.array_equal(out["key"].view(np.uint64), np.concatenate([f["key"], c["key"]]).view(np.uint64))
    assert np.array_equal(out["Wbar"].view(np.uint32), f["Wbar"].view(np.uint32))
    # Eq. (12) with the final z
    u = (U + (out["Wbar"] - out["Z"]).astype(np.float32)).astype(np.float32)
    assert np.array_equal(out["U"].view(np.uint32), u.view(np.uint32))


@pytest.mark.parametrize("seed", range(5))
def test_composite_against_numpy_library_routines(seed):
    rng = np.random.default_rng(400 + seed)
    R = int(rng.integers(1, 5))
    wl = wk.custom_workload(random_table_with_both(rng, 8), R=R, seed=seed, sigma_replica=0.03)
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
        assert np.array_equal(ea.view(np.uint32), ref.expand(t, ca["packed"], a["mask"], wl.n_arena, align).view(np.uint32))
        assert np.array_equal(ea.view(np.uint32), a["Z"].view(np.uint32))
    assert int(ca["layer_off"][-1]) >= wl.n_kept          # n_kept counts k * k_in * khw per composite layer
    # an arbitrary source under an arbitrary (union-like) mask
    src = rng.standard_normal(wl.n_arena).astype(np.float32)
    m = (rng.random(wl.groups_total) < 0.6).astype(np.uint8) * 3
    ca, cb = oracle.compact(t, src, m), ref.compact(t, src, m)
    assert np.array_equal(ca["layer_off"], cb["layer_off"]) and np.array_equal(ca["kept_idx"], cb["kept_idx"])
    assert np.array_equal(ca["packed"].view(np.uint32), cb["packed"].view(np.uint32))
    assert np.array_equal(oracle.expand(t, ca["packed"], m, wl.n_arena), ref.expand(t, ca["packed"], m, wl.n_arena))


def test_separable_magnitudes_have_a_closed_form_answer():
    """|V[o,c,t]| = a_o b_c: every filter norm is a_o ||b|| sqrt(khw) and every channel norm over any filter
    subset is b_c times a constant, so the composite projection keeps the k largest a and the k_in largest b,
    whatever the order (here the paper's order remark does hold)."""
    rng = np.random.default_rng(12)
    co, ci, khw, k, k_in = 9, 7, 4, 4, 3
    a = rng.permutation(np.arange(1, co + 1)).astype(np.float32)
    b = rng.permutation(np.arange(1, ci + 1)).astype(np.float32)
    sign = rng.choice([-1.0, 1.0], size=(co, ci, khw)).astype(np.float32)
    V = (a[:, None, None] * b[None, :, None] * sign).astype(np.float32)
    out = oracle.project(both_table(co, ci, khw, k, k_in), V.reshape(1, -1), np.zeros(V.size, np.float32))
    mf, mc = out["mask"][:co], out["mask"][co:]
    assert sorted(np.nonzero(mf)[0].tolist()) == sorted(np.argsort(-a)[:k].tolist())
    assert sorted(np.nonzero(mc)[0].tolist()) == sorted(np.argsort(-b)[:k_in].tolist())
    expect = V * mf[:, None, None] * mc[None, :, None]
    assert np.array_equal(out["Z"].reshape(V.shape), expect)
    kf = (a.astype(np.float64) ** 2) * np.sum(b.astype(np.float64) ** 2) * khw
    kc = (b.astype(np.float64) ** 2) * np.sum((a.astype(np.float64) ** 2)[mf == 1]) * khw
    assert out["key"].tolist() == np.concatenate([kf, kc]).tolist()       # small integers: exact


@pytest.mark.parametrize("seed", range(3))
def test_reductions_to_a_single_constraint(seed):
    """k_in = c_in: the channel projection keeps everything and the result is the filter projection;
    k = c_out: it is the channel projection."""
    rng = np.random.default_rng(500 + seed)
    co, ci, khw = int(rng.integers(2, 20)), int(rng.integers(2, 20)), int(rng.choice([1, 9]))
    wl = wk.custom_workload([(co, ci, khw, wk.MODE_BOTH, 1, 1)], R=2, seed=seed, sigma_replica=0.05)
    W, U = wk.generate(wl)
    k = int(rng.integers(1, co + 1))
    a = oracle.project(both_table(co, ci, khw, k, ci), W, U)
    f = oracle.project(one_layer_table(co, ci, khw, wk.MODE_FILTER, k), W, U)
    assert np.array_equal(a["mask"], np.concatenate([f["mask"], np.ones(ci, np.uint8)]))
    assert np.array_equal(a["Z"].view(np.uint32), f["Z"].view(np.uint32))
    assert np.array_equal(a["U"].view(np.uint32), f["U"].view(np.uint32))
    k_in = int(rng.integers(1, ci + 1))
    b = oracle.project(both_table(co, ci, khw, co, k_in), W, U)
    c = oracle.project(one_layer_table(co, ci, khw, wk.MODE_CHANNEL, k_in), W, U)
    assert np.array_equal(b["mask"], np.concatenate([np.ones(co, np.uint8), c["mask"]]))
    assert np.array_equal(b["key"][co:].view(np.uint64), c["key"].view(np.uint64))
    assert np.array_equal(b["Z"].view(np.uint32), c["Z"].view(np.uint32))
    assert np.array_equal(b["U"].view(np.uint32), c["U"].view(np.uint32))


def test_invariants_feasibility_conservation_idempotence():
    rng = np.random.default_rng(21)
    wl = wk.custom_workload(random_table_with_both(rng, 10), R=3, seed=4, sigma_replica=0.03)
    W, U = wk.generate(wl)
    t = wl.table()
    out = oracle.project(t, W, U, want_wbar=True)
    V = (out["Wbar"] + U).astype(np.float32)
    seen_both = 0
    for l in wl.layers:
        if l.mode != wk.MODE_BOTH:
            continue
        seen_both += 1
        m = out["mask"][l.group_base:l.group_base + l.groups]
        mf, mc = m[:l.c_out], m[l.c_out:]
        assert int(mf.sum()) == l.k and int(mc.sum()) == l.k_in
        sl = slice(l.elem_off, l.elem_off + l.n)
        z3 = out["Z"][sl].reshape(l.c_out, l.c_in, l.khw)
        v3 = V[sl].reshape(z3.shape)
        u3 = out["U"][sl].reshape(z3.shape)
        keep = np.broadcast_to((mf[:, None, None] & mc[None, :, None]).astype(bool), z3.shape)
        assert np.array_equal(z3[keep].view(np.uint32), v3[keep].view(np.uint32))
        assert not z3[~keep].view(np.uint32).any()
        assert np.array_equal(u3[~keep].view(np.uint32), v3[~keep].view(np.uint32))
        # the result lies in S_f ^ S_c
        assert int((np.abs(z3).sum(axis=(1, 2)) > 0).sum()) <= l.k
        assert int((np.abs(z3).sum(axis=(0, 2)) > 0).sum()) <= l.k_in
        # each stage is optimal for its input: kept keys dominate pruned keys
        key = out["key"][l.group_base:l.group_base + l.groups]
        kf, kc = key[:l.c_out], key[l.c_out:]
        if l.k < l.c_out:
            assert kf[mf == 1].min() >= kf[mf == 0].max()
        if l.k_in < l.c_in:
            assert kc[mc == 1].min() >= kc[mc == 0].max()
        # channel keys are those of the filter-pruned tensor
        x = v3.astype(np.float64) * mf[:, None, None]
        np.testing.assert_allclose(kc, np.sum(x * x, axis=(0, 2)), rtol=1e-12)
    assert seen_both >= 3
    # a point of S projects to itself (replica = Z, zero dual): same mask support, Z unchanged, dual stays zero
    again = oracle.project(t, out["Z"][None, :], np.zeros_like(U))
    assert np.array_equal(again["Z"].view(np.uint32), out["Z"].view(np.uint32))
    assert not again["U"].any()
    c = oracle.compact(t, out["Z"], out["mask"])
    assert int(c["layer_off"][-1]) == wl.n_kept
    assert c["kept_idx"].size == sum((l.k + l.k_in) if l.mode == wk.MODE_BOTH else
                                     (l.groups if l.mode == wk.MODE_NONE else l.k) for l in wl.layers)


def test_frozen_mask_under_both_constraints():
    """z = z~ (.) m with m the outer product of the filter bytes and the channel bytes (Section 4.5)."""
    base = CASES[0]
    fz = G["frozen"]
    t = both_table(base["c_out"], base["c_in"], base["khw"], base["k"], base["k_in"])
    W = np.array(base["W"], np.float32)
    out = oracle.project_frozen(t, W, np.array(base["U"], np.float32), np.array(fz["mask"], np.uint8))
    assert out["Z"].tolist() == [float(x) for x in fz["Z"]]
    assert out["U"].tolist() == [float(x) for x in fz["U_new"]]
    rng = np.random.default_rng(33)
    wl = wk.custom_workload(random_table_with_both(rng, 8), R=3, seed=2, sigma_replica=0.03)
    Wr, U = wk.generate(wl)
    mask = (rng.random(wl.groups_total) < 0.6).astype(np.uint8) * 9
    got = oracle.project_frozen(wl.table(), Wr, U, mask, want_wbar=True)
    V = (got["Wbar"] + U).astype(np.float32)
    for l in wl.layers:
        if l.mode != wk.MODE_BOTH:
            continue
        m = (mask[l.group_base:l.group_base + l.groups] != 0).astype(np.float32)
        m3 = m[:l.c_out, None, None] * m[None, l.c_out:, None]
        sl = slice(l.elem_off, l.elem_off + l.n)
        z = (V[sl].reshape(l.c_out, l.c_in, l.khw) * m3).reshape(-1)
        assert np.array_equal(got["Z"][sl], z) and not np.signbit(got["Z"][sl][z == 0]).any()
        u = (U[sl] + (got["Wbar"][sl] - got["Z"][sl]).astype(np.float32)).astype(np.float32)
        assert np.array_equal(got["U"][sl].view(np.uint32), u.view(np.uint32))
    # the projection's own mask gives the projection back
    a = oracle.project(wl.table(), Wr, U)
    b = oracle.project_frozen(wl.table(), Wr, U, a["mask"])
    assert np.array_equal(a["Z"].view(np.uint32), b["Z"].view(np.uint32))
    assert np.array_equal(a["U"].view(np.uint32), b["U"].view(np.uint32))


def test_weighted_candidate_under_both_constraints():
    """Eq. (9) candidate followed by the composite projection: with a = 1, b = 0 it is the base path bit for
    bit; otherwise Z is the composite projection of the candidate, which the base path reproduces when that
    candidate is handed to it as the only replica with a zero dual."""
    rng = np.random.default_rng(44)
    wl = wk.custom_workload(random_table_with_both(rng, 7), R=2, seed=6, sigma_replica=0.03)
    W, U = wk.generate(wl)
    t = wl.table()
    L = len(wl.layers)
    Zg = (0.05 * rng.standard_normal(wl.n_arena)).astype(np.float32)
    Vd = (0.01 * rng.standard_normal(wl.n_arena)).astype(np.float32)
    one, zero = np.ones(L, np.float32), np.zeros(L, np.float32)
    a0 = oracle.project_weighted(t, W, U, Zg, Vd, one, zero, want_wbar=True)
    b0 = oracle.project(t, W, U, want_wbar=True)
    for name in ("Z", "U", "Wbar", "mask"):
        assert np.array_equal(a0[name], b0[name]), name
    a, b = oracle.node_coefficients(np.full(L, 1.5e-3), np.full(L, 1.5e-4), 1e-4, 16, 2)
    out = oracle.project_weighted(t, W, U, Zg, Vd, a, b, want_wbar=True)
    cand = np.zeros(wl.n_arena, np.float32)
    for li, l in enumerate(wl.layers):
        sl = slice(l.elem_off, l.elem_off + l.n)
        tt = (out["Wbar"][sl] + U[sl]).astype(np.float32)
        q = (Zg[sl] - Vd[sl]).astype(np.float32)
        cand[sl] = ((a[li] * tt).astype(np.float32) + (b[li] * q).astype(np.float32)).astype(np.float32)
    p = oracle.project(t, cand[None, :], np.zeros_like(U))
    assert np.array_equal(out["mask"], p["mask"])
    assert np.array_equal(out["Z"].view(np.uint32), p["Z"].view(np.uint32))
    u = (U + (out["Wbar"] - out["Z"]).astype(np.float32)).astype(np.float32)
    pad = np.ones(wl.n_arena, bool)
    for l in wl.layers:
        pad[l.elem_off:l.elem_off + l.n] = False
    assert np.array_equal(out["U"][~pad].view(np.uint32), u[~pad].view(np.uint32))


def test_union_of_composite_masks_packs_the_union_of_both_index_sets():
    """Eq. (14) on masks of composite layers: the byte-wise OR is the union of the filter sets and of the channel
    sets, which is what the any-reductions of Section 4.4.1 extract; the packed block is |K_out| x |K_in| x khw."""
    co, ci, khw = 6, 5, 4
    t = both_table(co, ci, khw, 2, 2)
    m1 = np.array([1, 0, 1, 0, 0, 0] + [1, 1, 0, 0, 0], np.uint8)
    m2 = np.array([0, 0, 1, 0, 0, 1] + [0, 1, 0, 0, 1], np.uint8)
    u = oracle.mask_or([m1, m2])
    assert u.tolist() == [1, 0, 1, 0, 0, 1, 1, 1, 0, 0, 1]
    src = np.arange(co * ci * khw, dtype=np.float32)
    c = oracle.compact(t, src, u)
    assert c["kept_idx"].tolist() == [0, 2, 5, 0, 1, 4]
    assert c["layer_off"].tolist() == [0, 3 * 3 * khw]
    assert np.array_equal(c["packed"], src.reshape(co, ci, khw)[np.ix_([0, 2, 5], [0, 1, 4])].reshape(-1))


def test_composite_rejects_bad_k():
    for k, k_in in ((0, 1), (1, 0), (5, 1), (1, 4)):
        with pytest.raises(ValueError):
            oracle.project(both_table(4, 3, 1, k, k_in), np.zeros((1, 12), np.float32), np.zeros(12, np.float32))
