"""GPU parity of the layer-wise residual norms (Algorithm 1 Phase 5) against the CPU oracle.

Both sides add the same non-negative fp64 terms in different (fixed) orders.  The oracle's sequential sum of N
terms carries a relative error of up to N * 2^-53 (about sqrt(N) * 2^-53 in practice), the GPU's tree far less;
with N up to 2.4e6 elements x 8 replicas the tolerance is N_l * R * 2^-53 per layer, at least 1e-12.  The GPU
result is bitwise reproducible run to run."""
import numpy as np
import pytest

import oracle
import workloads as wk

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _check(wl, seed, optional=(True, True, True)):
    import paper_2512_14628_amd as pkg
    rng = np.random.default_rng(seed)
    W, U = wk.generate(wl, threads=8)
    t = wl.table()
    Zi = oracle.project(t, W, U)["Z"]
    arrs = [rng.standard_normal(wl.n_arena).astype(np.float32) * 0.05 if on else None for on in optional]
    if arrs[1] is None:
        arrs[2] = None
    ref = oracle.residuals(t, W, Zi, *arrs)
    dev = torch.device("cuda:0")
    plan = pkg.Plan(t)
    dW = [torch.from_numpy(W[r]).to(dev) for r in range(wl.R)]
    dZ = torch.from_numpy(Zi).to(dev)
    d = [None if a is None else torch.from_numpy(a).to(dev) for a in arrs]
    ws = torch.zeros(plan.workspace_bytes, dtype=torch.uint8, device=dev)
    out = torch.full((4 * plan.n_layers,), float("nan"), dtype=torch.float64, device=dev)
    pkg.hsadmm_residuals(plan, dW, dZ, d[0], d[1], d[2], out, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(4, -1)
    for li, l in enumerate(wl.layers):
        tol = max(1e-12, l.n * wl.R * 2.0 ** -53)
        np.testing.assert_allclose(got[:, li], ref[:, li], rtol=tol, atol=0, err_msg=l.name)
    # tighter, against NumPy's pairwise float64 sums (error ~ log2(N) * 2^-53 on both sides)
    for li, l in enumerate(wl.layers):
        sl = slice(l.elem_off, l.elem_off + l.n)
        zi = Zi[sl].astype(np.float64)
        r_in = sum(float(np.sum((W[r][sl].astype(np.float64) - zi) ** 2)) for r in range(wl.R))
        np.testing.assert_allclose(got[0, li], r_in, rtol=1e-13, atol=0, err_msg=l.name)
    out2 = torch.full_like(out, float("nan"))
    pkg.hsadmm_residuals(plan, dW, dZ, d[0], d[1], d[2], out2, ws)
    torch.cuda.synchronize()
    assert np.array_equal(out2.cpu().numpy().view(np.uint64), out.cpu().numpy().view(np.uint64))
    plan.close()


@pytest.mark.parametrize("name", ["tiny", "resnet18", "resnet50", "resnet152"])
def test_residuals_named_workloads(name):
    oracle.set_threads(8)
    _check(wk.make_workload(name), 1)


@pytest.mark.parametrize("R", [1, 3, 4, 5, 8])
def test_residuals_ragged_shapes_and_optional_operands(R):
    from tests.test_gpu_parity import _odd_shapes
    rng = np.random.default_rng(700 + R)
    wl = wk.custom_workload(_odd_shapes(rng, 10), R=R, seed=R, sigma_replica=0.03)
    _check(wl, R, optional=(R % 2 == 1, R != 3, R != 4))
    _check(wl, R, optional=(False, False, False))


def test_residuals_error_codes():
    import paper_2512_14628_amd as pkg
    from tests.gpu_harness import GpuRun
    wl = wk.make_workload("tiny")
    W, U = wk.generate(wl)
    r = GpuRun(wl, W, U)
    out = torch.zeros(4 * r.plan.n_layers, dtype=torch.float64, device=r.dev)
    assert pkg.hsadmm_residuals(r.plan, r.dW, None, None, None, None, out, r.ws, check=False) == -1
    assert pkg.hsadmm_residuals(r.plan, r.dW, r.dZ, None, None, None, None, r.ws, check=False) == -1
    assert pkg.hsadmm_residuals(r.plan, r.dW, r.dZ, None, None, None, out, r.ws[:256], check=False) == -2
    assert pkg.hsadmm_residuals(r.plan, r.dW * 17, r.dZ, None, None, None, out, r.ws, check=False) == -4
    r.close()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_scale_layers_matches_the_oracle(seed):
    """hsadmm_scale_layers (a scaled dual follows its layer's penalty): one fp32 product per element, bit for bit;
    layers with factor 1 and the arena padding keep their bits."""
    import paper_2512_14628_amd as pkg
    from tests.test_gpu_composite import _shapes_with_both
    rng = np.random.default_rng(4100 + seed)
    wl = wk.custom_workload(_shapes_with_both(rng, 11), R=1, seed=seed)
    t = wl.table()
    L = len(wl.layers)
    X = rng.standard_normal(wl.n_arena).astype(np.float32)
    f = rng.choice(np.array([0.5, 2.0, 0.8, 1.0, 1.0, 1.25, 1.0 / 3.0], np.float32), L)
    ref = oracle.scale_layers(t, X, f)
    dev = torch.device("cuda:0")
    plan = pkg.Plan(t)
    dX = torch.from_numpy(X).to(dev)
    df = torch.from_numpy(f).to(dev)
    pkg.hsadmm_scale_layers(plan, dX, df)
    torch.cuda.synchronize()
    assert np.array_equal(dX.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    assert pkg.hsadmm_scale_layers(plan, None, df, check=False) == -1
    assert pkg.hsadmm_scale_layers(plan, dX, None, check=False) == -1
    assert pkg.hsadmm_scale_layers(plan, dX[1:], df, check=False) == -1
    plan.close()


def test_phase_5_on_the_device_residuals_then_penalties_then_rescaled_duals():
    """Algorithm 1, Phase 5 end to end: the residual sums of a retraining-phase iteration (formed by its two kernels),
    the residual-balancing rule on the host, the duals rescaled on the device and the node weights of Eq. (9)
    recomputed -- against the same chain made of oracle calls.  The GPU's residual sums differ from the oracle's in
    the last bits, which decides nothing here: no layer of this workload sits on a boundary of the rule."""
    import paper_2512_14628_amd as pkg
    from tests.gpu_harness import GpuRun, bits
    wl = wk.make_workload("resnet18")
    W, U = wk.generate(wl, threads=8)
    t = wl.table()
    L = len(wl.layers)
    rng = np.random.default_rng(12)
    rho1, rho2 = np.full(L, 1.5e-3), np.full(L, 1.5e-4)
    lam, M = 1e-4, 16
    a, b = oracle.node_coefficients(rho1, rho2, lam, M, wl.R)
    Zg = (rng.standard_normal(wl.n_arena) * 0.05).astype(np.float32)
    Vd = (rng.standard_normal(wl.n_arena) * 0.01).astype(np.float32)
    zi_prev = (rng.standard_normal(wl.n_arena) * 0.05).astype(np.float32)
    mask = oracle.project_weighted(t, W, U, Zg, Vd, a, b)["mask"]
    # oracle chain
    ref = oracle.project_weighted_frozen(t, W, U, Zg, Vd, a, b, mask)
    refc = oracle.compact(t, oracle.add_arenas(t, ref["Z"], Vd), mask)
    z_new = oracle.expand(t, refc["packed"], mask, wl.n_arena)
    v_new = oracle.dual_inter(t, ref["Z"], z_new, Vd)
    sq = oracle.residuals(t, W, ref["Z"], zi_prev, z_new, Zg)
    args = (wl.R, 1, 10.0, 2.0, 2.0, 10.0, 10.0)
    o1, o2, osu, osv = oracle.adapt_penalties(sq, rho1, rho2, *args)
    assert (o1 != rho1).any() or (o2 != rho2).any()                 # the rule does act on this workload
    oU = oracle.scale_layers(t, ref["U"], osu)
    oV = oracle.scale_layers(t, v_new, osv)
    oa, ob = oracle.node_coefficients(o1, o2, lam, M, wl.R)
    # device chain
    r = GpuRun(wl, W, U, want_wbar=False, want_sqnorm=False)
    dZg, dVd = torch.from_numpy(Zg).to(r.dev), torch.from_numpy(Vd).to(r.dev)
    dm = torch.from_numpy(mask).to(r.dev)
    r.dZ.copy_(torch.from_numpy(zi_prev))
    dres = torch.zeros(4 * L, dtype=torch.float64, device=r.dev)
    pkg.hsadmm_plan_set_node_weights(r.plan, a, b)
    pkg.hsadmm_retrain_project(r.plan, r.dW, r.dU, dZg, dVd, r.dZ, None, dm, False, r.dpacked, r.doff, r.dkept, dres,
                               r.ws)
    pkg.hsadmm_retrain_expand(r.plan, r.dpacked, None, r.ddst, r.dZ, dVd, dZg, dres, r.ws)
    g1, g2, gsu, gsv = pkg.hsadmm_adapt_penalties(dres.cpu().numpy().reshape(4, L), rho1, rho2, *args)
    assert np.array_equal(np.array(g1), o1) and np.array_equal(np.array(g2), o2)
    assert np.array_equal(np.array(gsu, np.float32), osu) and np.array_equal(np.array(gsv, np.float32), osv)
    pkg.hsadmm_scale_layers(r.plan, r.dU, torch.tensor(gsu, dtype=torch.float32, device=r.dev))
    pkg.hsadmm_scale_layers(r.plan, dVd, torch.tensor(gsv, dtype=torch.float32, device=r.dev))
    ga, gb = pkg.hsadmm_node_coefficients(g1, g2, lam, M, wl.R)
    assert np.array_equal(np.array(ga, np.float32), oa) and np.array_equal(np.array(gb, np.float32), ob)
    torch.cuda.synchronize()
    gU, gV = r.dU.cpu().numpy(), dVd.cpu().numpy()
    for l in wl.layers:
        sl = slice(l.elem_off, l.elem_off + l.n)
        assert np.array_equal(bits(gU[sl]), bits(oU[sl])), l.name
        assert np.array_equal(bits(gV[sl]), bits(oV[sl])), l.name
    r.close()


def _dynamic_with_norms(wl, seed):
    """A dynamic outer iteration that takes the intra-node residual norms on the way (hsadmm_step with Zg / Vd,
    `residuals` and `Zi_prev`) against the plain calls it extends and the oracle: every other output the bits of
    hsadmm_project_weighted_compact, rows 0 and 1 within the summation tolerance of oracle.residuals, rows 2 and 3
    untouched; then hsadmm_retrain_expand completes the four norms."""
    import paper_2512_14628_amd as pkg
    rng = np.random.default_rng(seed)
    W, U = wk.generate(wl, threads=8)
    t = wl.table()
    L = len(wl.layers)
    a, b = oracle.node_coefficients(rng.uniform(1e-3, 2e-3, L), rng.uniform(1e-4, 3e-4, L), 1e-4, 16, wl.R)
    Zg = rng.standard_normal(wl.n_arena).astype(np.float32) * 0.05
    Vd = rng.standard_normal(wl.n_arena).astype(np.float32) * 0.01
    Zp = rng.standard_normal(wl.n_arena).astype(np.float32) * 0.05
    Zp[rng.random(wl.n_arena) < 0.5] = 0.0                       # a previous z_i is sparse
    ref = oracle.project_weighted(t, W, U, Zg, Vd, a, b)
    refc = oracle.compact(t, oracle.add_arenas(t, ref["Z"], Vd), ref["mask"])
    z_new = oracle.expand(t, refc["packed"], ref["mask"], wl.n_arena)
    sq = oracle.residuals(t, W, ref["Z"], Zp, z_new, Zg)
    dev = torch.device("cuda:0")
    coef = torch.from_numpy(np.stack([a, b], axis=1).astype(np.float32).reshape(-1).copy()).to(dev)

    def bufs():
        plan = pkg.Plan(t)
        d = {"plan": plan, "W": [torch.from_numpy(W[r]).to(dev) for r in range(wl.R)],
             "U": torch.from_numpy(U).to(dev), "Zg": torch.from_numpy(Zg).to(dev), "Vd": torch.from_numpy(Vd).to(dev),
             "Z": torch.full((wl.n_arena,), float("nan"), dtype=torch.float32, device=dev),
             "mask": torch.full((plan.groups_total,), 7, dtype=torch.uint8, device=dev),
             "ws": torch.full((plan.workspace_bytes,), 0xCD, dtype=torch.uint8, device=dev),
             "packed": torch.full((plan.packed_capacity_elems,), float("nan"), dtype=torch.float32, device=dev),
             "off": torch.zeros(L + 1, dtype=torch.int64, device=dev),
             "kept": torch.full((plan.groups_total,), -1, dtype=torch.int32, device=dev)}
        return d

    x, y = bufs(), bufs()
    pkg.hsadmm_step(x["plan"], x["W"], U=x["U"], Zg=x["Zg"], Vd=x["Vd"], coef=coef, Z=x["Z"], mask=x["mask"],
                    packed=x["packed"], layer_off=x["off"], kept_idx=x["kept"], workspace=x["ws"])
    res = torch.full((4 * L,), -7.0, dtype=torch.float64, device=dev)
    dZp = torch.from_numpy(Zp).to(dev)
    pkg.hsadmm_step(y["plan"], y["W"], U=y["U"], Zg=y["Zg"], Vd=y["Vd"], coef=coef, Z=y["Z"], mask=y["mask"],
                    packed=y["packed"], layer_off=y["off"], kept_idx=y["kept"], workspace=y["ws"], residuals=res,
                    Zi_prev=dZp)
    torch.cuda.synchronize()
    assert np.array_equal(y["mask"].cpu().numpy(), ref["mask"])
    for k in ("U", "Z", "mask", "packed", "off", "kept"):
        assert np.array_equal(x[k].cpu().numpy().view(np.uint8), y[k].cpu().numpy().view(np.uint8)), k
    for l in wl.layers:
        sl = slice(l.elem_off, l.elem_off + l.n)
        assert np.array_equal(y["Z"].cpu().numpy()[sl].view(np.uint32), ref["Z"][sl].view(np.uint32)), l.name
    got = res.cpu().numpy().reshape(4, L)
    assert np.all(got[2:] == -7.0)
    for li, l in enumerate(wl.layers):
        tol = max(1e-12, l.n * wl.R * 2.0 ** -53)
        np.testing.assert_allclose(got[:2, li], sq[:2, li], rtol=tol, atol=0, err_msg=l.name)
    # a second run gives the same bits
    y2 = bufs()
    res2 = torch.full_like(res, -7.0)
    pkg.hsadmm_step(y2["plan"], y2["W"], U=y2["U"], Zg=y2["Zg"], Vd=y2["Vd"], coef=coef, Z=y2["Z"], mask=y2["mask"],
                    packed=y2["packed"], layer_off=y2["off"], kept_idx=y2["kept"], workspace=y2["ws"], residuals=res2,
                    Zi_prev=dZp)
    # the inter-node half on top: decompression + Eq. (13) with rows 2 and 3
    dz = torch.full((wl.n_arena,), float("nan"), dtype=torch.float32, device=dev)
    pkg.hsadmm_retrain_expand(y2["plan"], y2["packed"], None, dz, y2["Z"], y2["Vd"], y2["Zg"], res2, y2["ws"])
    torch.cuda.synchronize()
    got2 = res2.cpu().numpy().reshape(4, L)
    assert np.array_equal(got2[:2].view(np.uint64), got[:2].view(np.uint64))
    for li, l in enumerate(wl.layers):
        tol = max(1e-12, l.n * wl.R * 2.0 ** -53)
        np.testing.assert_allclose(got2[:, li], sq[:, li], rtol=tol, atol=0, err_msg=l.name)
    for d in (x, y, y2):
        d["plan"].close()


@pytest.mark.parametrize("R", [1, 2, 3, 4, 5, 8])
def test_dynamic_iteration_takes_its_intra_node_norms_on_the_way(R):
    shapes = [(96, 16, 1, wk.MODE_FILTER, 40), (80, 64, 9, wk.MODE_FILTER, 30), (24, 512, 9, wk.MODE_FILTER, 9),
              (64, 3, 49, wk.MODE_FILTER, 20), (37, 5, 7, wk.MODE_FILTER, 36), (300, 1, 1, wk.MODE_FILTER, 1),
              (96, 128, 1, wk.MODE_CHANNEL, 50), (48, 40, 9, wk.MODE_BOTH, 30, 21), (10, 128, 1, wk.MODE_NONE, 10),
              (33, 7, 1, wk.MODE_NONE, 33), (70, 2100, 1, wk.MODE_FILTER, 28), (50, 24, 9, wk.MODE_CHANNEL, 10)]
    _dynamic_with_norms(wk.custom_workload(shapes, R=R, seed=60 + R, sigma_replica=0.03), 70 + R)


def test_dynamic_iteration_with_norms_on_resnet50_shapes():
    oracle.set_threads(8)
    _dynamic_with_norms(wk.make_workload("resnet50"), 3)


def test_dynamic_norms_want_both_the_previous_consensus_and_a_place_for_the_norms():
    import paper_2512_14628_amd as pkg
    wl = wk.custom_workload([(16, 8, 1, wk.MODE_FILTER, 4)], R=2, seed=1, sigma_replica=0.03)
    W, U = wk.generate(wl)
    dev = torch.device("cuda:0")
    plan = pkg.Plan(wl.table())
    n = wl.n_arena
    f = lambda: torch.zeros(n, dtype=torch.float32, device=dev)        # noqa: E731
    dW, dU, dZ, dZg, dVd, dZp = [f(), f()], f(), f(), f(), f(), f()
    mask = torch.zeros(plan.groups_total, dtype=torch.uint8, device=dev)
    ws = torch.zeros(plan.workspace_bytes, dtype=torch.uint8, device=dev)
    res = torch.zeros(4, dtype=torch.float64, device=dev)
    common = dict(U=dU, Zg=dZg, Vd=dVd, Z=dZ, mask=mask, workspace=ws)
    assert pkg.hsadmm_step(plan, dW, residuals=res, check=False, **common) == -1          # no Zi_prev
    assert pkg.hsadmm_step(plan, dW, Zi_prev=dZp, check=False, **common) == -1            # no place for the norms
    assert pkg.hsadmm_step(plan, dW, residuals=res, Zi_prev=dZ, check=False, **common) == -1   # Zi_prev is Z
    assert pkg.hsadmm_step(plan, dW, U=dU, Z=dZ, mask=mask, workspace=ws, residuals=res, Zi_prev=dZp, check=False) == -4
    assert pkg.hsadmm_step(plan, dW, residuals=res, Zi_prev=dZp, **common) == 0
    plan.close()
