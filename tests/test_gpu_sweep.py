"""Randomised parity sweep: layer tables drawn at random over every mode, odd sizes, replica counts and packing
alignments, each run through project + compact + expand (with and without masks, as separate calls and through the *_compact
calls) and compared with the oracle on every element (tests/test_gpu_parity._run).  All sizes are within the documented limits of the library."""
import numpy as np
import pytest

import workloads as wk

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _random_shapes(rng, n_layers):
    shapes = []
    for _ in range(n_layers):
        kind = rng.integers(0, 6)
        if kind == 0:       # long rows, few of them
            co, ci, khw = int(rng.integers(1, 12)), int(rng.integers(300, 3000)), int(rng.choice([1, 9]))
        elif kind == 1:     # many short rows
            co, ci, khw = int(rng.integers(500, 5000)), int(rng.integers(1, 9)), int(rng.choice([1, 1, 4]))
        elif kind == 2:     # rows just around the wide-row threshold
            co, ci, khw = int(rng.integers(2, 40)), int(rng.choice([511, 512, 513, 2047, 2048, 2049])), int(rng.choice([1, 4]))
        else:
            co, ci, khw = int(rng.integers(1, 400)), int(rng.integers(1, 400)), int(rng.choice([1, 1, 4, 9, 25, 49]))
        mode = int(rng.choice([0, 1, 1, 2, 2, 3, 3]))
        if mode == wk.MODE_BOTH:
            shapes.append((co, ci, khw, mode, int(rng.integers(1, co + 1)), int(rng.integers(1, ci + 1))))
        else:
            G = ci if mode == wk.MODE_CHANNEL else co
            shapes.append((co, ci, khw, mode, int(rng.integers(1, G + 1))))
    return shapes


@pytest.mark.parametrize("seed", range(12))
def test_random_tables(seed):
    from tests.test_gpu_parity import _run
    rng = np.random.default_rng(9000 + seed)
    R = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 16]))
    wl = wk.custom_workload(_random_shapes(rng, int(rng.integers(1, 16))), R=R, seed=seed, sigma_replica=0.03)
    _run(wl, pack_align=int(rng.choice([1, 1, 2, 4, 5, 16])), want_wbar=bool(rng.integers(0, 2)),
         want_sqnorm=bool(rng.integers(0, 2)))


@pytest.mark.parametrize("seed", range(6))
def test_random_tables_weighted_and_frozen(seed):
    import oracle
    from tests.test_gpu_weighted import _phase4_chain
    from tests.test_gpu_frozen import _check_frozen
    rng = np.random.default_rng(9500 + seed)
    R = int(rng.choice([1, 2, 4, 6, 8]))
    wl = wk.custom_workload(_random_shapes(rng, int(rng.integers(2, 12))), R=R, seed=seed, sigma_replica=0.03)
    W, U = wk.generate(wl)
    L = len(wl.layers)
    a = rng.uniform(0.3, 1.0, L).astype(np.float32)
    b = rng.uniform(0.0, 0.7, L).astype(np.float32)
    _phase4_chain(wl, W, U, a, b, rng, want_wbar=bool(seed % 2), want_sqnorm=bool(seed % 3), fused_dual=bool(seed % 2))
    _phase4_chain(wl, W, U, a, b, rng, want_wbar=not bool(seed % 2), want_sqnorm=bool(seed % 3), fused_dual=True,
                  one_call=True)
    mask = (rng.random(wl.groups_total) < rng.uniform(0.1, 0.9)).astype(np.uint8) * 255
    _check_frozen(wl, W, U, mask, want_wbar=bool(seed % 2))
    _check_frozen(wl, W, U, oracle.project(wl.table(), W, U)["mask"], want_wbar=False)


@pytest.mark.parametrize("seed", range(8))
def test_random_tables_under_predictions(seed):
    """The step under a predicted selection (hsadmm_step with sel_prev) on random tables: the plain candidate with the
    dual in place and out of place, the weighted candidate out of place with and without the residual norms, each
    under the right record and under records degraded by a random fraction, against the oracle on every element."""
    import oracle
    import paper_2512_14628_amd as pkg
    from tests.gpu_harness import check_against_oracle, packed_segment_sizes
    from tests.test_gpu_hinted import _Bufs, _hinted_step, degrade, record_of
    rng = np.random.default_rng(9800 + seed)
    R = int(rng.choice([1, 2, 3, 4, 5, 8, 9]))
    pack_align = int(rng.choice([1, 1, 2, 4, 5, 16]))
    wl = wk.custom_workload(_random_shapes(rng, int(rng.integers(1, 14))), R=R, seed=seed, sigma_replica=0.03)
    W, U = wk.generate(wl)
    t = wl.table()
    L = len(wl.layers)
    ref = oracle.project(t, W, U, want_wbar=True)
    refc = oracle.compact(t, ref["Z"], ref["mask"], pack_align=pack_align)
    want_sel = record_of(wl, ref["mask"])
    b = _Bufs(wl, W, U, pack_align)
    dev = b.U.device
    recs = [want_sel] + [record_of(wl, degrade(wl, ref["mask"], float(f), rng)) for f in rng.uniform(0.02, 0.6, 2)]
    for rec in recs:
        for out_of_place in (False, True):
            b.reset()
            _hinted_step(b, torch.from_numpy(rec).to(dev), out_of_place=out_of_place)
            got = b.outputs()
            rep = check_against_oracle(wl, got, ref, refc, pack_align=pack_align)
            assert all(v == 0 for v in rep.values()), (out_of_place, rep)
            assert np.array_equal(got["sel"], want_sel)
    # the weighted candidate
    a, bb = oracle.node_coefficients(rng.uniform(1e-3, 2e-3, L), rng.uniform(1e-4, 3e-4, L), 1e-4, 16, R)
    Zg = rng.standard_normal(wl.n_arena).astype(np.float32) * 0.05
    Vd = rng.standard_normal(wl.n_arena).astype(np.float32) * 0.01
    Zp = rng.standard_normal(wl.n_arena).astype(np.float32) * 0.05
    wref = oracle.project_weighted(t, W, U, Zg, Vd, a, bb, want_wbar=True)
    wrefc = oracle.compact(t, oracle.add_arenas(t, wref["Z"], Vd), wref["mask"], pack_align=pack_align)
    sq = oracle.residuals(t, W, wref["Z"], Zp)
    sizes = packed_segment_sizes(wl, wref["mask"])
    wsel = record_of(wl, wref["mask"])
    dZg, dVd, dZp = torch.from_numpy(Zg).to(dev), torch.from_numpy(Vd).to(dev), torch.from_numpy(Zp).to(dev)
    coef = torch.from_numpy(np.stack([a, bb], axis=1).astype(np.float32).reshape(-1).copy()).to(dev)
    for rec in (wsel, record_of(wl, degrade(wl, wref["mask"], float(rng.uniform(0.02, 0.6)), rng))):
        for norms in (False, True):
            b.reset()
            b.out_of_place = True
            res = torch.full((4 * L,), -7.0, dtype=torch.float64, device=dev)
            extra = dict(residuals=res, Zi_prev=dZp) if norms else {}
            pkg.hsadmm_step(b.plan, b.W, U=b.U, U_out=b.Uout, Zg=dZg, Vd=dVd, coef=coef, Z=b.Z, Wbar=b.Wbar, mask=b.mask,
                            sqnorm=b.key, sel=b.sel, sel_prev=torch.from_numpy(rec).to(dev), packed=b.packed,
                            layer_off=b.off, kept_idx=b.kept, workspace=b.ws, **extra)
            got = b.outputs()
            assert np.array_equal(got["mask"], wref["mask"]) and np.array_equal(got["sel"], wsel)
            for key in ("Z", "U", "Wbar"):
                for l in wl.layers:
                    sl = slice(l.elem_off, l.elem_off + l.n)
                    assert np.array_equal(got[key][sl].view(np.uint32), wref[key][sl].view(np.uint32)), (key, l.name)
            assert np.array_equal(got["layer_off"], wrefc["layer_off"])
            for li in range(L):
                lo = int(wrefc["layer_off"][li])
                assert np.array_equal(got["packed"][lo:lo + sizes[li]].view(np.uint32),
                                      wrefc["packed"][lo:lo + sizes[li]].view(np.uint32)), li
            if norms:
                got_res = res.cpu().numpy().reshape(4, L)
                for li, l in enumerate(wl.layers):
                    tol = max(1e-12, l.n * R * 2.0 ** -53)
                    np.testing.assert_allclose(got_res[:2, li], sq[:2, li], rtol=tol, atol=0, err_msg=l.name)
    b.plan.close()
