"""GPU parity of the top-k selection (Eq. (10): the k groups of largest norm, lower index first among equals) on
key distributions chosen to take each route through the selection kernel: keys that agree in their upper 32 bits,
many groups tied at the threshold (so that no short list of candidates ever forms and the last, partly repeated
digit is reached), tie classes in layers too wide for the in-register path, and the same for channel keys.

Every key is exact in fp64 whatever the order of its additions (squares of small dyadic numbers), so the oracle
and the GPU see the same bit patterns and the masks must agree bit for bit."""
import numpy as np
import pytest

import oracle
import workloads as wk

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _fill(wl, W, U, li, first_column):
    """Layer li becomes zero except for element 0 of every group, taken from first_column (FILTER: one per row;
    CHANNEL: row 0, one per column); 1.0 goes into a second element so that no key is zero."""
    l = wl.layers[li]
    U[l.elem_off:l.elem_off + l.n] = 0
    for w in W:
        a = w[l.elem_off:l.elem_off + l.n].reshape(l.c_out, l.c_in * l.khw)
        a[:] = 0
        if l.mode == wk.MODE_CHANNEL:
            a[0, :] = first_column
            a[1, :] = 1.0
        else:
            a[:, 0] = first_column
            a[:, 1] = 1.0


def test_selection_routes():
    rng = np.random.default_rng(5)
    shapes = [
        (1000, 2, 1, wk.MODE_FILTER, 400),      # 0: keys equal in the upper word, all distinct
        (3000, 2, 1, wk.MODE_FILTER, 1500),     # 1: three values, 1000 groups each: threshold inside a class
        (2000, 2, 1, wk.MODE_FILTER, 975),      # 2: 40 values x 50: more ties than the short list holds
        (9000, 2, 1, wk.MODE_FILTER, 4550),     # 3: wider than the in-register path, 90 values x 100
        (2, 2000, 1, wk.MODE_CHANNEL, 975),     # 4: as 2, channel keys
        (2, 1000, 1, wk.MODE_CHANNEL, 400),     # 5: as 0, channel keys
        (2, 9000, 1, wk.MODE_CHANNEL, 4550),    # 6: as 3, channel keys
        (700, 2, 1, wk.MODE_FILTER, 300),       # 7: two values only, one of them once
        (500, 2, 1, wk.MODE_FILTER, 33),        # 8: 33 wanted of 34 tied at the top
    ]
    wl = wk.custom_workload(shapes, R=2, seed=3, sigma_replica=0.0)
    W, U = wk.generate(wl)
    distinct = rng.permutation(1000).astype(np.float32) * np.float32(2.0 ** -20)      # key = 1 + g^2 2^-40
    classes40 = (1.0 + rng.permutation(2000) % 40 * 2.0 ** -10).astype(np.float32)
    classes90 = (1.0 + rng.permutation(9000) % 90 * 2.0 ** -10).astype(np.float32)
    _fill(wl, W, U, 0, distinct)
    _fill(wl, W, U, 1, (1 + rng.permutation(3000) % 3).astype(np.float32))
    _fill(wl, W, U, 2, classes40)
    _fill(wl, W, U, 3, classes90)
    _fill(wl, W, U, 4, classes40)
    _fill(wl, W, U, 5, distinct)
    _fill(wl, W, U, 6, classes90)
    two = np.full(700, 3.0, np.float32)
    two[412] = 5.0
    _fill(wl, W, U, 7, two)
    top = np.full(500, 1.0, np.float32)
    top[rng.permutation(500)[:34]] = 2.0
    _fill(wl, W, U, 8, top)

    t = wl.table()
    ref = oracle.project(t, W, U)
    # what the construction promises
    k0 = ref["key"][wl.layers[0].group_base:wl.layers[0].group_base + 1000].view(np.uint64)
    assert len(set((k0 >> np.uint64(32)).tolist())) == 1 and len(set(k0.tolist())) == 1000
    k2 = ref["key"][wl.layers[2].group_base:wl.layers[2].group_base + 2000]
    assert len(set(k2.tolist())) == 40

    from tests.gpu_harness import GpuRun, bits
    run = GpuRun(wl, W, U)
    run.step()
    got = run.outputs()
    for li, l in enumerate(wl.layers):
        g = slice(l.group_base, l.group_base + l.groups)
        assert np.array_equal(got["key"][g].view(np.uint64), ref["key"][g].view(np.uint64)), li
        assert np.array_equal(got["mask"][g], ref["mask"][g]), li
        assert int(np.count_nonzero(got["mask"][g])) == l.k
        sl = slice(l.elem_off, l.elem_off + l.n)
        assert np.array_equal(bits(got["Z"][sl]), bits(ref["Z"][sl])), li
        assert np.array_equal(bits(got["U"][sl]), bits(ref["U"][sl])), li
    refc = oracle.compact(t, ref["Z"], ref["mask"])
    assert np.array_equal(got["layer_off"], refc["layer_off"])
    assert np.array_equal(got["kept_idx"][:refc["kept_idx"].size], refc["kept_idx"])
    assert np.array_equal(bits(got["packed"][:refc["packed"].size]), bits(refc["packed"]))
    # lower index first among equals, spelled out for layer 8: the 33 lowest of the 34 tied groups
    l8 = wl.layers[8]
    tied = np.flatnonzero(top == 2.0)
    assert np.flatnonzero(got["mask"][l8.group_base:l8.group_base + 500]).tolist() == tied[:33].tolist()
    run.close()
