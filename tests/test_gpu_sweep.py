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
