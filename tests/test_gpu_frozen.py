"""GPU parity of the frozen-mask projection (Algorithm 1 Phase 3, retraining branch) and of the mask union
(Eq. (14)) against the CPU oracle, through the C ABI.  Bit-exact on every output."""
import numpy as np
import pytest

import oracle
import workloads as wk

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _check_frozen(wl, W, U, mask_np, want_wbar=True):
    import paper_2512_14628_amd as pkg
    from tests.gpu_harness import GpuRun, bits
    run = GpuRun(wl, W, U, want_wbar=want_wbar)
    dmask = torch.from_numpy(mask_np).to(run.dev)
    pkg.hsadmm_project_frozen(run.plan, run.dW, run.dU, run.dZ, run.dWbar, dmask)
    pkg.hsadmm_compact(run.plan, run.dZ, dmask, run.dpacked, run.doff, run.dkept, run.ws)
    pkg.hsadmm_expand(run.plan, run.dpacked, None, run.ddst, run.ws)
    got = run.outputs()
    ref = oracle.project_frozen(wl.table(), W, U, mask_np, want_wbar=True)
    refc = oracle.compact(wl.table(), ref["Z"], (mask_np != 0).astype(np.uint8))
    for l in wl.layers:
        sl = slice(l.elem_off, l.elem_off + l.n)
        assert np.array_equal(bits(got["Z"][sl]), bits(ref["Z"][sl])), "Z " + l.name
        assert np.array_equal(bits(got["U"][sl]), bits(ref["U"][sl])), "U " + l.name
        if want_wbar:
            assert np.array_equal(bits(got["Wbar"][sl]), bits(ref["Wbar"][sl])), "Wbar " + l.name
        assert np.array_equal(bits(got["dst"][sl]), bits(ref["Z"][sl])), "expand " + l.name
    assert np.array_equal(got["layer_off"], refc["layer_off"])
    n = int(refc["layer_off"][-1])
    assert np.array_equal(bits(got["packed"][:n]), bits(refc["packed"]))
    run.close()
    # the call that projects and compacts in one go: every output, every bit, as the two calls; first deriving the
    # index mappings from the mask, then reusing the ones an earlier call left in the workspace
    for cached in (False, True):
        r2 = GpuRun(wl, W, U, want_wbar=want_wbar)
        dm2 = torch.from_numpy(mask_np).to(r2.dev)
        if cached:
            pkg.hsadmm_expand(r2.plan, r2.dpacked, dm2, r2.ddst, r2.ws)         # leaves this mask's mappings
            r2.ddst.fill_(float("nan"))
        pkg.hsadmm_project_frozen_compact(r2.plan, r2.dW, r2.dU, r2.dZ, r2.dWbar, dm2, cached, r2.dpacked, r2.doff,
                                          r2.dkept, r2.ws)
        pkg.hsadmm_expand(r2.plan, r2.dpacked, None, r2.ddst, r2.ws)
        got2 = r2.outputs()
        for name in got:
            if name == "mask":
                continue                                                         # the harness's own mask buffer: unused
            assert np.array_equal(got[name].view(np.uint8), got2[name].view(np.uint8)), \
                "one call (cached=%s): %s" % (cached, name)
        r2.close()


@pytest.mark.parametrize("name", ["tiny", "resnet18", "resnet50", "resnet152"])
def test_frozen_with_union_of_two_node_masks(name):
    """Two 'nodes' project different replicas, their masks are OR-ed on the device, and the union (which keeps
    more than k groups) is applied as a frozen mask, then compacted and expanded."""
    import paper_2512_14628_amd as pkg
    wl = wk.make_workload(name)
    W, U = wk.generate(wl, threads=8)
    wl_b = wk.make_workload(name, seed=7)
    Wb, Ub = wk.generate(wl_b, threads=8)
    oracle.set_threads(8)
    ma = oracle.project(wl.table(), W, U)["mask"]
    mb = oracle.project(wl.table(), Wb, Ub)["mask"]
    union_ref = oracle.mask_or([ma, mb])
    plan = pkg.Plan(wl.table())
    dev = torch.device("cuda:0")
    da, db = torch.from_numpy(ma).to(dev), torch.from_numpy(mb * 9).to(dev)     # any nonzero byte = kept
    dout = torch.full((plan.groups_total,), 77, dtype=torch.uint8, device=dev)
    pkg.hsadmm_mask_or(plan, [da, db], dout)
    torch.cuda.synchronize()
    assert np.array_equal(dout.cpu().numpy(), union_ref)
    pkg.hsadmm_mask_or(plan, [da, db], da)                                     # in place
    torch.cuda.synchronize()
    assert np.array_equal(da.cpu().numpy(), union_ref)
    plan.close()
    _check_frozen(wl, W, U, union_ref)


@pytest.mark.parametrize("R", [1, 2, 3, 4, 6, 8])
def test_frozen_ragged_shapes_random_masks(R):
    from tests.test_gpu_parity import _odd_shapes
    rng = np.random.default_rng(300 + R)
    wl = wk.custom_workload(_odd_shapes(rng, 12), R=R, seed=R, sigma_replica=0.03)
    W, U = wk.generate(wl)
    mask = (rng.random(wl.groups_total) < 0.45).astype(np.uint8) * 255
    _check_frozen(wl, W, U, mask, want_wbar=(R % 2 == 1))
    _check_frozen(wl, W, U, np.zeros(wl.groups_total, np.uint8), want_wbar=False)
    _check_frozen(wl, W, U, np.ones(wl.groups_total, np.uint8), want_wbar=False)


def test_frozen_with_own_mask_equals_dynamic_projection():
    import paper_2512_14628_amd as pkg
    from tests.gpu_harness import GpuRun, bits
    wl = wk.make_workload("resnet18")
    W, U = wk.generate(wl, threads=8)
    a = GpuRun(wl, W, U)
    a.project()
    b = GpuRun(wl, W, U)
    pkg.hsadmm_project_frozen(b.plan, b.dW, b.dU, b.dZ, b.dWbar, a.dmask)
    ga, gb = a.outputs(), b.outputs()
    for name in ("Z", "U", "Wbar"):
        assert np.array_equal(bits(ga[name]), bits(gb[name])), name
    a.close()
    b.close()


def test_frozen_error_codes():
    import paper_2512_14628_amd as pkg
    from tests.gpu_harness import GpuRun
    wl = wk.make_workload("tiny")
    W, U = wk.generate(wl)
    run = GpuRun(wl, W, U)
    assert pkg.hsadmm_project_frozen(run.plan, run.dW, run.dU, run.dZ, None, None, check=False) == -1
    assert pkg.hsadmm_project_frozen(run.plan, [], run.dU, run.dZ, None, run.dmask, check=False) == -1
    assert pkg.hsadmm_project_frozen(run.plan, run.dW * 17, run.dU, run.dZ, None, run.dmask, check=False) == -4
    pfc = pkg.hsadmm_project_frozen_compact
    assert pfc(run.plan, run.dW, run.dU, run.dZ, None, None, False, run.dpacked, run.doff, run.dkept, run.ws,
               check=False) == -1
    assert pfc(run.plan, run.dW, run.dU, run.dZ, None, run.dmask, False, None, run.doff, run.dkept, run.ws,
               check=False) == -1
    assert pfc(run.plan, run.dW, run.dU, run.dZ, None, run.dmask, False, run.dpacked, run.doff, run.dkept, None,
               workspace_bytes=1 << 30, check=False) == -1
    assert pfc(run.plan, run.dW, run.dU, run.dZ, None, run.dmask, False, run.dpacked, run.doff, run.dkept,
               run.ws[:256], check=False) == -2
    assert pfc(run.plan, run.dW * 17, run.dU, run.dZ, None, run.dmask, False, run.dpacked, run.doff, run.dkept,
               run.ws, check=False) == -4
    assert pkg.hsadmm_mask_or(run.plan, [], run.dmask, check=False) == -1
    assert pkg.hsadmm_mask_or(run.plan, [run.dmask] * 65, run.dmask, check=False) == -4
    assert pkg.hsadmm_mask_or(run.plan, [run.dmask, None], run.dmask, check=False) == -1
    run.close()


def test_mask_drift_between_two_iterations():
    """Section 4.5: per-layer count of groups whose kept flag changed; zero drift is the freezing signal."""
    import paper_2512_14628_amd as pkg
    from tests.gpu_harness import GpuRun
    from tests.test_gpu_composite import _shapes_with_both
    rng = np.random.default_rng(8)
    wl = wk.custom_workload(_shapes_with_both(rng, 14), R=2, seed=3, sigma_replica=0.03)
    W, U = wk.generate(wl)
    run = GpuRun(wl, W, U)
    run.project()
    m1 = run.dmask.clone()
    run.project()                                   # second iteration: U has moved on
    drift = torch.full((len(wl.layers),), -7, dtype=torch.int32, device=run.dev)
    pkg.hsadmm_mask_drift(run.plan, m1, run.dmask, drift)
    torch.cuda.synchronize()
    ref = oracle.mask_drift(wl.table(), m1.cpu().numpy(), run.dmask.cpu().numpy())
    assert np.array_equal(drift.cpu().numpy(), ref)
    pkg.hsadmm_mask_drift(run.plan, m1, m1 * 5, drift)
    torch.cuda.synchronize()
    assert not drift.cpu().numpy().any()
    x = torch.from_numpy((rng.random(wl.groups_total) < 0.5).astype(np.uint8)).to(run.dev)
    y = torch.from_numpy(((rng.random(wl.groups_total) < 0.5) * 255).astype(np.uint8)).to(run.dev)
    pkg.hsadmm_mask_drift(run.plan, x, y, drift)
    torch.cuda.synchronize()
    assert np.array_equal(drift.cpu().numpy(), oracle.mask_drift(wl.table(), x.cpu().numpy(), y.cpu().numpy()))
    assert pkg.hsadmm_mask_drift(run.plan, x, None, drift, check=False) == -1
    run.close()


def test_rows_longer_than_four_million_columns():
    """A CHANNEL layer whose rows hold more than 2^22 columns (c_in * khw = 5.4 M): the column -> channel division
    leaves its fast path.  Frozen-mask projection, compaction and expansion (no selection: the oracle's rank count is
    quadratic in the number of groups)."""
    wl = wk.custom_workload([(2, 600_000, 9, wk.MODE_CHANNEL, 1000), (3, 5, 1, wk.MODE_FILTER, 2)], R=2, seed=1,
                            sigma_replica=0.03)
    W, U = wk.generate(wl)
    rng = np.random.default_rng(4)
    mask = (rng.random(wl.groups_total) < 0.4).astype(np.uint8)
    _check_frozen(wl, W, U, mask, want_wbar=False)
