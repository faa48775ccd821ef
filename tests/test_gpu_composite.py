"""GPU parity of layers under both constraints (S = S_f ^ S_c, Section 2.1; the two projections applied one
after the other, Section 3, paragraph after Eq. (10); K_out x K_in packing, Eq. (15)) against the CPU oracle,
through the C ABI: the base step, the frozen-mask path, the full node update and the mask union.

Bar: masks, offsets, kept indices and packed layout bit-exact; fp32 outputs bit-identical; keys rtol 1e-12."""
import numpy as np
import pytest

import oracle
import workloads as wk

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

BOTH = wk.MODE_BOTH


def _shapes_with_both(rng, n_layers):
    shapes = []
    for _ in range(n_layers):
        co = int(rng.integers(1, 300))
        ci = int(rng.integers(1, 300))
        khw = int(rng.choice([1, 1, 1, 4, 9, 9, 25, 49]))
        mode = int(rng.choice([0, 1, 2, 3, 3, 3]))
        if mode == BOTH:
            shapes.append((co, ci, khw, mode, int(rng.integers(1, co + 1)), int(rng.integers(1, ci + 1))))
        else:
            G = ci if mode == wk.MODE_CHANNEL else co
            shapes.append((co, ci, khw, mode, int(rng.integers(1, G + 1))))
    return shapes


@pytest.mark.parametrize("R", [1, 2, 3, 4, 5, 8])
def test_composite_ragged_shapes(R):
    from tests.test_gpu_parity import _run
    rng = np.random.default_rng(2000 + R)
    wl = wk.custom_workload(_shapes_with_both(rng, 12), R=R, seed=R, sigma_replica=0.03)
    _run(wl, pack_align=(1, 4, 7)[R % 3], want_wbar=(R % 2 == 0), want_sqnorm=(R % 3 != 0))


@pytest.mark.parametrize("pack_align", [1, 5])
def test_composite_and_filter_layers_without_channel_layers(pack_align):
    """No CHANNEL layer: hsadmm_project_compact then runs the FILTER fix-up and the gather (also of the BOTH layers'
    rows, repaired by the launch before) in one launch; _run compares it with the two calls and with the oracle."""
    from tests.test_gpu_parity import _run
    shapes = [(70, 33, 9, wk.MODE_FILTER, 21), (40, 30, 4, BOTH, 13, 11), (10, 5, 1, wk.MODE_NONE, 10),
              (300, 7, 1, wk.MODE_FILTER, 299), (129, 130, 1, BOTH, 64, 100), (3, 5000, 1, wk.MODE_FILTER, 1),
              (64, 64, 9, BOTH, 1, 64), (17, 3, 25, wk.MODE_FILTER, 17), (256, 96, 1, BOTH, 200, 1)]
    wl = wk.custom_workload(shapes, R=3, seed=21, sigma_replica=0.03)
    _run(wl, pack_align=pack_align)


def test_composite_degenerate_layers():
    """1 x 1 layers, everything kept, one filter / one channel kept, a single column, a single row, rows longer than
    a workgroup's span, more groups than one scan block, a 3-channel stem."""
    shapes = [(1, 1, 1, BOTH, 1, 1), (5, 7, 9, BOTH, 5, 7), (40, 33, 1, BOTH, 1, 1), (300, 1, 9, BOTH, 120, 1),
              (1, 300, 4, BOTH, 1, 77), (6, 4100, 1, BOTH, 3, 2000), (3000, 5, 1, BOTH, 1500, 2),
              (64, 3, 49, BOTH, 38, 2), (2, 1500, 9, BOTH, 1, 600), (33, 31, 25, BOTH, 32, 30),
              (8, 8, 1, wk.MODE_NONE, 8), (17, 19, 1, BOTH, 17, 1)]
    from tests.test_gpu_parity import _run
    wl = wk.custom_workload(shapes, R=3, seed=13, sigma_replica=0.03)
    _run(wl)


def test_composite_resnet50_full_size():
    """ResNet-50 shapes, every conv under both constraints (keep 0.6 of the filters, then 0.6 of the channels),
    R = 4: every element against the oracle, in the launch configuration the benchmark times."""
    from tests.test_gpu_parity import _run
    _run(wk.make_workload("resnet50_both"), threads=16)


def test_composite_ties_lower_index_wins_in_both_selections():
    from tests.gpu_harness import GpuRun
    wl = wk.custom_workload([(120, 90, 4, BOTH, 50, 40), (30, 20, 1, BOTH, 10, 5)], R=2, seed=4, sigma_replica=0.0)
    W, U = wk.generate(wl)
    l0, l1 = wl.layers
    for arr in (W[0], W[1], U):
        a = arr[l0.elem_off:l0.elem_off + l0.n].reshape(120, 90, 4)
        a[:] = a[np.arange(120) % 13][:, np.arange(90) % 7]      # 13 distinct filters, 7 distinct channels
        arr[l1.elem_off:l1.elem_off + l1.n] = 0                  # all keys zero: the first indices win
    t = wl.table()
    ref = oracle.project(t, W, U)
    run = GpuRun(wl, W, U)
    run.step()
    got = run.outputs()
    assert np.array_equal(got["mask"], ref["mask"])
    assert got["mask"][l1.group_base:l1.group_base + 50].tolist() == [1] * 10 + [0] * 20 + [1] * 5 + [0] * 15
    # identical groups have identical keys on the GPU too (the order of additions does not depend on the position)
    k0 = got["key"][l0.group_base:l0.group_base + l0.groups]
    for g in range(13, 120):
        assert k0[g] == k0[g % 13]
    for c in range(7, 90):
        assert k0[120 + c] == k0[120 + c % 7]
    for l in wl.layers:
        sl = slice(l.elem_off, l.elem_off + l.n)
        assert np.array_equal(got["Z"][sl].view(np.uint32), ref["Z"][sl].view(np.uint32))
        assert np.array_equal(got["U"][sl].view(np.uint32), ref["U"][sl].view(np.uint32))
    refc = oracle.compact(t, ref["Z"], ref["mask"])
    assert np.array_equal(got["layer_off"], refc["layer_off"])
    assert np.array_equal(got["kept_idx"][:refc["kept_idx"].size], refc["kept_idx"])
    run.close()


@pytest.mark.parametrize("R", [1, 4, 8])
def test_composite_frozen_masks(R):
    from tests.test_gpu_frozen import _check_frozen
    rng = np.random.default_rng(2300 + R)
    wl = wk.custom_workload(_shapes_with_both(rng, 12), R=R, seed=R, sigma_replica=0.03)
    W, U = wk.generate(wl)
    mask = (rng.random(wl.groups_total) < 0.55).astype(np.uint8) * 255
    _check_frozen(wl, W, U, mask, want_wbar=(R != 4))
    _check_frozen(wl, W, U, np.zeros(wl.groups_total, np.uint8), want_wbar=False)
    _check_frozen(wl, W, U, np.ones(wl.groups_total, np.uint8), want_wbar=False)
    _check_frozen(wl, W, U, oracle.project(wl.table(), W, U)["mask"], want_wbar=False)


def test_composite_union_of_two_node_masks_full_size():
    """Eq. (14) on masks of composite layers, then the frozen path, compaction and expansion under the union."""
    import paper_2512_14628_amd as pkg
    from tests.test_gpu_frozen import _check_frozen
    wl = wk.make_workload("resnet50_both")
    W, U = wk.generate(wl, threads=16)
    Wb, Ub = wk.generate(wk.make_workload("resnet50_both", seed=7), threads=16)
    oracle.set_threads(16)
    ma = oracle.project(wl.table(), W, U)["mask"]
    mb = oracle.project(wl.table(), Wb, Ub)["mask"]
    union_ref = oracle.mask_or([ma, mb])
    plan = pkg.Plan(wl.table())
    dev = torch.device("cuda:0")
    dout = torch.full((plan.groups_total,), 77, dtype=torch.uint8, device=dev)
    pkg.hsadmm_mask_or(plan, [torch.from_numpy(ma).to(dev), torch.from_numpy(mb * 3).to(dev)], dout)
    torch.cuda.synchronize()
    assert np.array_equal(dout.cpu().numpy(), union_ref)
    plan.close()
    _check_frozen(wl, W, U, union_ref, want_wbar=False)


@pytest.mark.parametrize("R", [1, 2, 4, 7])
def test_composite_weighted_step(R):
    from tests.test_gpu_weighted import _phase4_chain
    rng = np.random.default_rng(2500 + R)
    wl = wk.custom_workload(_shapes_with_both(rng, 12), R=R, seed=R, sigma_replica=0.03)
    W, U = wk.generate(wl)
    L = len(wl.layers)
    a = rng.uniform(0.3, 1.0, L).astype(np.float32)
    b = rng.uniform(0.0, 0.7, L).astype(np.float32)
    _phase4_chain(wl, W, U, a, b, rng, want_wbar=(R % 2 == 0), want_sqnorm=(R != 4), fused_dual=(R in (2, 7)))
    _phase4_chain(wl, W, U, a, b, rng, want_wbar=(R % 2 == 1), want_sqnorm=(R != 4), fused_dual=True, one_call=True)


def test_composite_arbitrary_source_and_mask_and_cached_expand():
    from tests.gpu_harness import GpuRun, bits
    rng = np.random.default_rng(91)
    wl = wk.custom_workload(_shapes_with_both(rng, 10), R=1, seed=2)
    W, U = wk.generate(wl)
    for align in (1, 8):
        run = GpuRun(wl, W, U, pack_align=align)
        src = rng.standard_normal(wl.n_arena).astype(np.float32)
        mask = (rng.random(wl.groups_total) < 0.5).astype(np.uint8) * 17
        dsrc, dm = torch.from_numpy(src).to(run.dev), torch.from_numpy(mask).to(run.dev)
        run.compact(src=dsrc, mask=dm)
        run.expand(cached=True)
        got = run.outputs()
        refc = oracle.compact(wl.table(), src, mask, pack_align=align)
        back = oracle.expand(wl.table(), refc["packed"], mask, wl.n_arena, pack_align=align)
        assert np.array_equal(got["layer_off"], refc["layer_off"])
        assert np.array_equal(got["kept_idx"][:refc["kept_idx"].size], refc["kept_idx"])
        for li, l in enumerate(wl.layers):
            m = mask[l.group_base:l.group_base + l.groups] != 0
            if l.mode == BOTH:
                used = int(m[:l.c_out].sum()) * int(m[l.c_out:].sum()) * l.khw
            elif l.mode == wk.MODE_NONE:
                used = l.n
            else:
                used = int(m.sum()) * l.group_size
            a0 = int(refc["layer_off"][li])
            assert np.array_equal(bits(got["packed"][a0:a0 + used]), bits(refc["packed"][a0:a0 + used])), li
            sl = slice(l.elem_off, l.elem_off + l.n)
            assert np.array_equal(bits(got["dst"][sl]), bits(back[sl])), li
        # the same through a fresh scan of the mask
        run.ddst.fill_(float("nan"))
        run.expand(mask=dm)
        got2 = run.outputs()
        for l in wl.layers:
            sl = slice(l.elem_off, l.elem_off + l.n)
            assert np.array_equal(bits(got2["dst"][sl]), bits(back[sl]))
        run.close()


def test_composite_plan_rejects_bad_counts():
    import paper_2512_14628_amd as pkg
    for k, k_in in ((0, 1), (1, 0), (5, 1), (1, 4)):
        wl = wk.custom_workload([(4, 3, 1, BOTH, k, k_in)], R=1)
        with pytest.raises(pkg.HsadmmError):
            pkg.Plan(wl.table())
