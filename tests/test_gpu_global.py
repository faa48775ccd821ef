"""GPU parity of the global consensus of Eq. (11) and of the whole consensus side of one outer iteration for several
nodes whose buffers live on one device (Algorithm 1, Phases 3-4): per node the weighted projection, the mask union
(Eq. (14)), the compaction of c_i = z_i + v_i under the union, the mean of the compact buffers (Eq. (11)), the expansion
to the global z, and per node the inter-node dual update (Eq. (13)).  Everything through the C ABI, against the same
chain built from oracle calls.  Bit-exact."""
import numpy as np
import pytest

import oracle
import workloads as wk

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.mark.parametrize("M,n", [(1, 4096), (2, 1_000_003), (3, 17), (5, 2_097_152), (16, 65_537), (64, 4099)])
def test_average_of_node_buffers(M, n):
    import paper_2512_14628_amd as pkg
    rng = np.random.default_rng(M * 1000 + n % 97)
    bufs = [rng.standard_normal(n).astype(np.float32) for _ in range(M)]
    ref = oracle.average(bufs)
    wl = wk.make_workload("tiny")
    plan = pkg.Plan(wl.table())
    dev = torch.device("cuda:0")
    d = [torch.from_numpy(b).to(dev) for b in bufs]
    out = torch.full((n + 8,), float("nan"), dtype=torch.float32, device=dev)
    pkg.hsadmm_average(plan, d, n, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got[:n].view(np.uint32), ref.view(np.uint32))
    assert np.all(np.isnan(got[n:]))                                     # nothing written past the end
    pkg.hsadmm_average(plan, d, n, d[0])                                 # in place
    torch.cuda.synchronize()
    assert np.array_equal(d[0].cpu().numpy().view(np.uint32), ref.view(np.uint32))
    assert pkg.hsadmm_average(plan, [], n, out, check=False) == -1
    assert pkg.hsadmm_average(plan, d * 65, n, out, check=False) == -4
    assert pkg.hsadmm_average(plan, [d[0][1:]], n - 1, out, check=False) == -1   # misaligned
    plan.close()


def _chain_on_gpu(wl, table, nodes, a, b, Zg, pack_align):
    import paper_2512_14628_amd as pkg
    dev = torch.device("cuda:0")
    plan = pkg.Plan(table, pack_align_elems=pack_align)
    pkg.hsadmm_plan_set_node_weights(plan, a, b)
    n = wl.n_arena
    dZg = torch.from_numpy(Zg).to(dev)
    st = []
    for nd in nodes:
        s = {"W": [torch.from_numpy(np.ascontiguousarray(w)).to(dev) for w in nd["W"]],
             "U": torch.from_numpy(nd["U"].copy()).to(dev), "V": torch.from_numpy(nd["Vd"].copy()).to(dev),
             "Z": torch.full((n,), float("nan"), dtype=torch.float32, device=dev),
             "mask": torch.zeros(plan.groups_total, dtype=torch.uint8, device=dev),
             "ws": torch.zeros(plan.workspace_bytes, dtype=torch.uint8, device=dev),
             "packed": torch.full((plan.packed_capacity_elems,), float("nan"), dtype=torch.float32, device=dev),
             "off": torch.zeros(plan.n_layers + 1, dtype=torch.int64, device=dev),
             "kept": torch.zeros(plan.groups_total, dtype=torch.int32, device=dev)}
        st.append(s)
    for s in st:                                                             # Phase 3 on every node
        pkg.hsadmm_project_weighted(plan, s["W"], s["U"], dZg, s["V"], s["Z"], None, s["mask"], None, s["ws"])
    m = torch.zeros(plan.groups_total, dtype=torch.uint8, device=dev)
    pkg.hsadmm_mask_or(plan, [s["mask"] for s in st], m)                     # Eq. (14)
    for s in st:                                                             # shrink c_i = z_i + v_i under the union
        pkg.hsadmm_compact_sum(plan, s["Z"], s["V"], m, s["packed"], s["off"], s["kept"], s["ws"])
    torch.cuda.synchronize()
    n_packed = int(st[0]["off"][-1].item())
    zp = torch.full((plan.packed_capacity_elems,), float("nan"), dtype=torch.float32, device=dev)
    pkg.hsadmm_average(plan, [s["packed"] for s in st], n_packed, zp)        # Eq. (11)
    z = torch.full((n,), float("nan"), dtype=torch.float32, device=dev)
    pkg.hsadmm_expand(plan, zp, None, z, st[0]["ws"])                        # node 0's workspace holds the union's maps
    for s in st:
        pkg.hsadmm_dual_inter(plan, s["Z"], z, s["V"])                       # Eq. (13)
    torch.cuda.synchronize()
    out = {"Z": [s["Z"].cpu().numpy() for s in st], "U": [s["U"].cpu().numpy() for s in st],
           "V": [s["V"].cpu().numpy() for s in st], "mask_i": [s["mask"].cpu().numpy() for s in st],
           "mask": m.cpu().numpy(), "z": z.cpu().numpy(), "packed_mean": zp.cpu().numpy()[:n_packed],
           "layer_off": st[0]["off"].cpu().numpy()}
    plan.close()
    return out


@pytest.mark.parametrize("M,R,pack_align", [(2, 1, 1), (3, 2, 4), (4, 4, 1)])
def test_consensus_side_of_an_outer_iteration_for_several_nodes(M, R, pack_align):
    from tests.test_oracle_global import node_chain
    from tests.test_gpu_composite import _shapes_with_both
    from tests.gpu_harness import bits
    rng = np.random.default_rng(4000 + M)
    shapes = _shapes_with_both(rng, 9)
    wl = wk.custom_workload(shapes, R=R, seed=1, sigma_replica=0.03)
    t = wl.table()
    L = len(wl.layers)
    a, b = oracle.node_coefficients(rng.uniform(1e-3, 2e-3, L), rng.uniform(1e-4, 3e-4, L), 1e-4, M, R)
    Zg = (0.05 * rng.standard_normal(wl.n_arena)).astype(np.float32)
    nodes = []
    for i in range(M):
        W, U = wk.generate(wk.custom_workload(shapes, R=R, seed=50 + i, sigma_replica=0.03))
        nodes.append({"W": W, "U": U, "Vd": (0.01 * rng.standard_normal(wl.n_arena)).astype(np.float32)})
    ref = node_chain(t, wl.n_arena, nodes, a, b, Zg, pack_align=pack_align)
    got = _chain_on_gpu(wl, t, nodes, a, b, Zg, pack_align)
    assert np.array_equal(got["mask"], ref["mask"])
    assert np.array_equal(got["layer_off"], ref["layer_off"])
    for i in range(M):
        assert np.array_equal(got["mask_i"][i], ref["mask_i"][i]), i
    pad = np.ones(wl.n_arena, bool)
    for l in wl.layers:
        sl = slice(l.elem_off, l.elem_off + l.n)
        pad[sl] = False
        assert np.array_equal(bits(got["z"][sl]), bits(ref["z"][sl])), l.name
        for i in range(M):
            for name in ("Z", "U", "V"):
                assert np.array_equal(bits(got[name][i][sl]), bits(ref[name][i][sl])), (name, i, l.name)
    # compact mean: compare the layers' used parts (alignment padding is unspecified)
    for li, l in enumerate(wl.layers):
        m = ref["mask"][l.group_base:l.group_base + l.groups] != 0
        if l.mode == wk.MODE_BOTH:
            used = int(m[:l.c_out].sum()) * int(m[l.c_out:].sum()) * l.khw
        elif l.mode == wk.MODE_NONE:
            used = l.n
        else:
            used = int(m.sum()) * l.group_size
        a0 = int(ref["layer_off"][li])
        assert np.array_equal(bits(got["packed_mean"][a0:a0 + used]), bits(ref["packed_mean"][a0:a0 + used])), li
