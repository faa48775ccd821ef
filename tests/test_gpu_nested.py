"""GPU parity for the composite sets that put shape groups inside input channels (Section 2.1: S_c ^ S_s and
S_f ^ S_c ^ S_s; the projections one after the other, Section 3, paragraph after Eq. (10)).

The library takes such a layer through its [c_out][c_in*khw] GEMM view (a CHANNEL layer, or one under both
constraints, of c_in*khw channels with khw = 1) plus an hsadmm_nest_t entry: runs of khw channels, of which k_in may
hold kept channels.  The oracle computes modes 5 and 6 from their own definition on the layer as it is; its channel
entries have no counterpart in the view and are dropped before the comparison.  Everything else must agree as for any
other mode: masks, offsets, kept indices and packed layout bit-exact, fp32 outputs bit-identical, under every form
of the call (separate calls, cached mappings, fused, predicted, weighted candidate, frozen mask)."""
import numpy as np
import pytest

import oracle
import workloads as wk

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _view_workload(wl):
    """The workload as the library sees it: every layer through its GEMM view (same offsets, same elements)."""
    t = wl.gemm_view_table()
    shapes = [(int(t["c_out"][i]), int(t["c_in"][i]), int(t["khw"][i]), int(t["mode"][i]), int(t["k"][i]),
               int(t["k_in"][i])) for i in range(len(wl.layers))]
    v = wk.custom_workload(shapes, R=wl.R, seed=wl.seed, sigma_replica=wl.sigma_replica)
    assert [l.elem_off for l in v.layers] == [l.elem_off for l in wl.layers] and v.n_arena == wl.n_arena
    return v, t


def _reference(wl, W, U, pack_align, weighted=None):
    v, t = _view_workload(wl)
    if weighted is None:
        ref = oracle.project(wl.table(), W, U, want_wbar=True)
    else:
        Zg, Vd, a, b = weighted
        ref = oracle.project_weighted(wl.table(), W, U, Zg, Vd, a, b, want_wbar=True)
    ref = dict(ref, mask=wl.view_groups(ref["mask"]), key=wl.view_groups(ref["key"]))
    refc = oracle.compact(v.table(), ref["Z"], ref["mask"], pack_align=pack_align)
    return v, t, ref, refc


def _random_shapes(rng, n_layers=10):
    shapes = []
    for _ in range(n_layers):
        co, ci = int(rng.integers(1, 160)), int(rng.integers(1, 48))
        khw = int(rng.choice([1, 4, 9, 9, 25, 49]))
        mode = int(rng.choice([0, 1, 2, 3, 4, 5, 5, 5, 6, 6, 6]))
        k_in = int(rng.integers(1, ci + 1))
        if mode in (5, 6):
            shapes.append((co, ci, khw, mode, int(rng.integers(1, co + 1)) if mode == 6 else 0, k_in,
                           int(rng.integers(1, k_in * khw + 1))))
        elif mode == 3:
            shapes.append((co, ci, khw, mode, int(rng.integers(1, co + 1)), k_in))
        else:
            G = {0: co, 1: co, 2: ci, 4: ci * khw}[mode]
            shapes.append((co, ci, khw, mode, int(rng.integers(1, G + 1))))
    return shapes


def _check(v, got, ref, refc, pack_align, what=""):
    from tests.gpu_harness import check_against_oracle
    rep = check_against_oracle(v, got, ref, refc, pack_align=pack_align)
    assert all(c == 0 for c in rep.values()), (what, rep)


@pytest.mark.parametrize("R,pack_align,seed", [(1, 1, 0), (3, 4, 1), (4, 1, 2), (2, 7, 3), (4, 4, 4)])
def test_random_tables_in_every_form_of_the_call(R, pack_align, seed):
    from tests.gpu_harness import GpuRun
    rng = np.random.default_rng(5100 + seed)
    wl = wk.custom_workload(_random_shapes(rng), R=R, seed=seed, sigma_replica=0.03)
    W, U = wk.generate(wl)
    v, t, ref, refc = _reference(wl, W, U, pack_align)
    outs = []
    for form in (dict(), dict(cached=True), dict(fused=True)):
        run = GpuRun(v, W, U, pack_align=pack_align, table=t)
        run.step(**form)
        got = run.outputs()
        _check(v, got, ref, refc, pack_align, str(form))
        outs.append(got)
        run.close()
    for name in outs[0]:
        for other in outs[1:]:
            assert np.array_equal(outs[0][name].view(np.uint8), other[name].view(np.uint8)), name


def _resnet18_nested(mode, R=2, keep_in=0.5, keep_kern=0.5):
    base = wk.make_workload("resnet18")
    shapes = []
    for l in base.layers:
        if l.khw > 1:
            k_in = wk.keep_count(keep_in, l.c_in)
            shapes.append((l.c_out, l.c_in, l.khw, mode, wk.keep_count(0.6, l.c_out) if mode == 6 else 0, k_in,
                           wk.keep_count(keep_kern, k_in * l.khw)))
        else:
            shapes.append((l.c_out, l.c_in, l.khw, l.mode, l.k))
    return wk.custom_workload(shapes, R=R, seed=1, sigma_replica=0.03)


@pytest.mark.parametrize("mode", [5, 6])
def test_resnet18_shapes_base_step_frozen_mask_and_weighted_candidate(mode):
    """ResNet-18 with every 3x3 / 7x7 conv under channels-with-shapes (half the channels, then half of their
    positions) or all three constraints: up to 512 * 9 = 4608 view channels in 512 runs."""
    from tests.gpu_harness import GpuRun, bits
    import paper_2512_14628_amd as pkg
    wl = _resnet18_nested(mode)
    W, U = wk.generate(wl, threads=8)
    oracle.set_threads(8)
    v, t, ref, refc = _reference(wl, W, U, 1)
    run = GpuRun(v, W, U, table=t)
    run.step(fused=True)
    _check(v, run.outputs(), ref, refc, 1)
    # the frozen-mask step with the mask just selected reproduces the projection (and needs no nesting)
    run2 = GpuRun(v, W, U, table=t)
    pkg.hsadmm_project_frozen(run2.plan, run2.dW, run2.dU, run2.dZ, None, torch.from_numpy(ref["mask"]).to(run2.dev))
    got = run2.outputs()
    for l in v.layers:
        sl = slice(l.elem_off, l.elem_off + l.n)
        assert np.array_equal(bits(got["Z"][sl]), bits(ref["Z"][sl])) and np.array_equal(bits(got["U"][sl]), bits(ref["U"][sl]))
    # the weighted candidate of Eq. (9)
    rng = np.random.default_rng(7)
    L = len(wl.layers)
    Zg = (rng.standard_normal(wl.n_arena) * 0.05).astype(np.float32)
    Vd = (rng.standard_normal(wl.n_arena) * 0.01).astype(np.float32)
    a = rng.uniform(0.3, 0.9, L).astype(np.float32)
    b = rng.uniform(0.1, 0.7, L).astype(np.float32)
    v, t, wref, wrefc = _reference(wl, W, U, 1, weighted=(Zg, Vd, a, b))
    run3 = GpuRun(v, W, U, table=t)
    coef = torch.from_numpy(np.stack([a, b], axis=1).reshape(-1).copy()).to(run3.dev)
    pkg.hsadmm_step(run3.plan, run3.dW, U=run3.dU, Z=run3.dZ, Wbar=run3.dWbar, mask=run3.dmask, sqnorm=run3.dkey,
                    Zg=torch.from_numpy(Zg).to(run3.dev), Vd=torch.from_numpy(Vd).to(run3.dev), coef=coef,
                    workspace=run3.ws)
    got = run3.outputs()
    assert np.array_equal(got["mask"], wref["mask"])
    np.testing.assert_allclose(got["key"], wref["key"], rtol=1e-12, atol=0)
    for name in ("Z", "U", "Wbar"):
        for l in v.layers:
            sl = slice(l.elem_off, l.elem_off + l.n)
            assert np.array_equal(bits(got[name][sl]), bits(wref[name][sl])), (name, l.name)
    for r in (run, run2, run3):
        r.close()


def test_under_predictions_in_place_and_out_of_place():
    """The predicted step (hsadmm_step with sel_prev) on a table with nested layers: right, partly wrong and wrong
    records, dual in place and out of place; every output is the oracle's whatever the record says."""
    from tests.test_gpu_hinted import _Bufs, _hinted_step, record_of, degrade
    rng = np.random.default_rng(5200)
    shapes = _random_shapes(rng, 8) + [(96, 40, 9, 5, 0, 20, 70), (64, 24, 9, 6, 40, 12, 50), (128, 16, 49, 5, 0, 9, 200)]
    wl = wk.custom_workload(shapes, R=4, seed=9, sigma_replica=0.03)
    W, U = wk.generate(wl)
    for pack_align in (1, 4):
        v, t, ref, refc = _reference(wl, W, U, pack_align)
        want_sel = record_of(v, ref["mask"])
        b = _Bufs(v, W, U, pack_align, table=t)
        dev = b.U.device
        G = b.plan.groups_total
        records = {"all right": want_sel,
                   "a tenth wrong": record_of(v, degrade(v, ref["mask"], 0.1, rng)),
                   "all wrong": record_of(v, (ref["mask"] == 0).astype(np.uint8)),
                   "everything pruned": np.full(G, -1, np.int32),
                   None: None}
        for name, rec in records.items():
            for out_of_place in (False, True):
                b.reset()
                _hinted_step(b, None if rec is None else torch.from_numpy(rec).to(dev), out_of_place=out_of_place)
                got = b.outputs()
                _check(v, got, ref, refc, pack_align, (name, out_of_place))
                assert np.array_equal(got["sel"], want_sel), (name, out_of_place)
        b.plan.close()


def test_ties_zero_columns_and_more_columns_than_the_selection_holds_in_registers():
    """Identical channels and positions (every key ties: lower index first at both levels), columns of zeros (so
    that fewer nonzero candidates than k_kern remain: only positions of kept channels may fill up), and views of
    1100 * 9 = 9900 and 9000 * 2 = 18000 channels (the latter in 9000 runs), beyond what the selection ranks from
    registers."""
    from tests.gpu_harness import GpuRun
    shapes = [(6, 8, 4, 5, 0, 3, 7), (5, 6, 9, 6, 3, 2, 11), (4, 10, 4, 5, 0, 4, 16), (3, 1100, 9, 5, 0, 500, 2000),
              (9, 12, 9, 6, 9, 12, 108), (7, 5, 1, 5, 0, 3, 2),
              (2, 9000, 2, 5, 0, 4000, 5000)]      # more runs, too, than the selection holds in registers
    wl = wk.custom_workload(shapes, R=2, seed=3, sigma_replica=0.0)
    W, U = wk.generate(wl)
    U[:] = 0
    l0, l1, l2 = wl.layers[0], wl.layers[1], wl.layers[2]
    for l in (l0, l1):                                  # every position of the layer identical
        w = W[:, l.elem_off:l.elem_off + l.n].reshape(wl.R, l.c_out, l.c_in * l.khw)
        w[:] = w[:, :, :1]
    w = W[:, l2.elem_off:l2.elem_off + l2.n].reshape(wl.R, l2.c_out, l2.c_in, l2.khw)
    w[:, :, :, 1:] = 0                                  # one nonzero position per channel: 4 candidates for 16 places
    v, t, ref, refc = _reference(wl, W, U, 1)
    m0 = ref["mask"][v.layers[0].group_base:v.layers[0].group_base + v.layers[0].groups]
    assert m0.tolist() == [1] * 7 + [0] * 25
    m2 = ref["mask"][v.layers[2].group_base:v.layers[2].group_base + v.layers[2].groups].reshape(10, 4)
    assert int(m2.sum()) == 16 and set(np.flatnonzero(m2.sum(axis=1))) == set(np.flatnonzero(m2[:, 0]))
    from tests import gpu_harness
    run = GpuRun(v, W, U, table=t)
    run.step(fused=True)
    got = run.outputs()
    # ties everywhere: the near-tie guard of the general check does not apply; compare directly
    assert np.array_equal(got["mask"], ref["mask"])
    np.testing.assert_allclose(got["key"], ref["key"], rtol=1e-12, atol=0)
    for name in ("Z", "U", "Wbar"):
        for l in v.layers:
            sl = slice(l.elem_off, l.elem_off + l.n)
            assert np.array_equal(gpu_harness.bits(got[name][sl]), gpu_harness.bits(ref[name][sl])), (name, l.name)
    assert np.array_equal(got["layer_off"], refc["layer_off"])
    assert np.array_equal(got["kept_idx"][:refc["kept_idx"].size], refc["kept_idx"])
    n_used = int(refc["layer_off"][-1])
    assert np.array_equal(gpu_harness.bits(got["packed"][:n_used]), gpu_harness.bits(refc["packed"][:n_used]))
    run.close()


def test_bad_nest_entries_are_refused():
    import paper_2512_14628_amd as pkg

    def table(mode, ci, khw, k, k_in, span, k_coarse):
        return {"elem_off": np.array([0], np.int64), "c_out": np.array([8], np.int32), "c_in": np.array([ci], np.int32),
                "khw": np.array([khw], np.int32), "mode": np.array([mode], np.int32), "k": np.array([k], np.int32),
                "k_in": np.array([k_in], np.int32), "span": np.array([span], np.int32),
                "k_coarse": np.array([k_coarse], np.int32)}
    good = pkg.Plan(table(2, 36, 1, 10, 0, 9, 2))
    good.close()
    pkg.Plan(table(1, 36, 1, 4, 0, 0, 0)).close()            # span 0: no limit, any mode
    pkg.Plan(table(2, 36, 1, 10, 0, 1, 12)).close()          # runs of one channel
    for bad in (table(1, 36, 1, 4, 0, 9, 2),      # FILTER layers have no channels to nest
                table(2, 4, 9, 2, 0, 9, 2),       # not declared through the view (khw != 1)
                table(2, 35, 1, 10, 0, 9, 2),     # c_in not a multiple of span
                table(2, 36, 1, 10, 0, 9, 0),     # no run kept
                table(2, 36, 1, 10, 0, 9, 5),     # more runs than there are
                table(2, 36, 1, 19, 0, 9, 2),     # more columns than the kept runs hold
                table(3, 36, 1, 4, 19, 9, 2)):
        with pytest.raises(pkg.HsadmmError):
            pkg.Plan(bad)
