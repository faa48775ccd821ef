"""GPU parity for shape sparsity (Section 2.1: groups W[:, b, u, v]).  The library has no mode of its own for it: such
a group is a column of the layer's [c_out][c_in*khw] GEMM view, so the layer is handed over as a CHANNEL layer of
c_in*khw channels with khw = 1.  The oracle computes the shape mode from its own literal definition; every output must
agree as for any other mode (masks, offsets, kept indices, packed layout bit-exact, fp32 outputs bit-identical)."""
import numpy as np
import pytest

import oracle
import workloads as wk

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.mark.parametrize("R", [1, 3, 4])
def test_shape_sparsity_through_the_gemm_view(R):
    from tests.test_gpu_parity import _run
    rng = np.random.default_rng(3100 + R)
    shapes = []
    for _ in range(10):
        co, ci = int(rng.integers(1, 200)), int(rng.integers(1, 80))
        khw = int(rng.choice([1, 4, 9, 9, 25, 49]))
        mode = int(rng.choice([1, 2, 4, 4, 4]))
        G = {1: co, 2: ci, 4: ci * khw}[mode]
        shapes.append((co, ci, khw, mode, int(rng.integers(1, G + 1))))
    wl = wk.custom_workload(shapes, R=R, seed=R, sigma_replica=0.03)
    _run(wl, pack_align=(1, 4)[R % 2], gpu_table=wl.gemm_view_table())


def test_shape_sparsity_resnet18_shapes_base_and_frozen():
    """ResNet-18 shapes with every 3x3 / 7x7 conv under shape sparsity (keep 0.5 of the (channel, position) groups):
    base step and frozen-mask step against the oracle's literal shape mode."""
    from tests.test_gpu_parity import _run
    from tests.gpu_harness import GpuRun, bits
    import paper_2512_14628_amd as pkg
    base = wk.make_workload("resnet18")
    shapes = []
    for l in base.layers:
        if l.khw > 1:
            shapes.append((l.c_out, l.c_in, l.khw, wk.MODE_SHAPE, wk.keep_count(0.5, l.c_in * l.khw)))
        else:
            shapes.append((l.c_out, l.c_in, l.khw, l.mode, l.k))
    wl = wk.custom_workload(shapes, R=2, seed=0, sigma_replica=0.03)
    gt = wl.gemm_view_table()
    _run(wl, gpu_table=gt, determinism=False)
    W, U = wk.generate(wl, threads=8)
    mask = oracle.project(wl.table(), W, U)["mask"]
    ref = oracle.project_frozen(wl.table(), W, U, mask)
    run = GpuRun(wl, W, U, table=gt)
    pkg.hsadmm_project_frozen(run.plan, run.dW, run.dU, run.dZ, None, torch.from_numpy(mask).to(run.dev))
    got = run.outputs()
    for l in wl.layers:
        sl = slice(l.elem_off, l.elem_off + l.n)
        assert np.array_equal(bits(got["Z"][sl]), bits(ref["Z"][sl])) and np.array_equal(bits(got["U"][sl]), bits(ref["U"][sl]))
    run.close()
