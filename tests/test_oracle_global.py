"""Pins of the oracle's global consensus step, Eq. (11): z = (1/M) sum_i (z_i + v_i), and of the chain that leads to it
on one device (Algorithm 1, Phases 3-4: node projections, mask union, compaction of c_i = z_i + v_i under the union,
mean of the compact buffers, expansion, inter-node dual update).  CPU only."""
import numpy as np
import pytest

import oracle
import workloads as wk
from tests.test_oracle_pins import one_layer_table, random_table


def test_handworked_mean_of_node_buffers():
    # three nodes, c_i = z_i + v_i given; mean exact in fp32
    c = [np.array([3, 0, -6, 1.5], np.float32), np.array([0, 3, 0, 1.5], np.float32), np.array([3, 3, 0, 0], np.float32)]
    assert oracle.average(c).tolist() == [(np.float32(6) * (np.float32(1) / np.float32(3))).item(),
                                          (np.float32(6) * (np.float32(1) / np.float32(3))).item(), -2.0, 1.0]
    assert oracle.average(c[:1]).tolist() == c[0].tolist()                      # M = 1: z = z_1 + v_1
    assert oracle.average([c[0], c[0]]).tolist() == c[0].tolist()
    # left-to-right in node order, then times fl32(1/M) (the convention of the replica mean)
    big = np.float32(2 ** 24)
    assert oracle.average([np.array([big]), np.array([1.0]), np.array([1.0]), np.array([0.0])])[0] == np.float32(2 ** 22)
    assert oracle.average([np.array([1.0]), np.array([1.0]), np.array([big]), np.array([0.0])])[0] == np.float32((2 ** 24 + 2) / 4)
    five_thirds = oracle.average([np.array([1.0]), np.array([2.0]), np.array([2.0])])[0]
    assert five_thirds == np.float32(5) * (np.float32(1) / np.float32(3)) and five_thirds != np.float32(5) / np.float32(3)


@pytest.mark.parametrize("seed", range(3))
def test_mean_equals_the_pinned_replica_mean_and_numpy(seed):
    """The same arithmetic as the consensus average of step (a): the buffers handed to oracle_project as the
    replicas of an unconstrained layer give the same bits; and it is the float64 mean within fp32 rounding."""
    rng = np.random.default_rng(900 + seed)
    M, n = int(rng.integers(1, 9)), 4 * int(rng.integers(1, 200))
    bufs = [rng.standard_normal(n).astype(np.float32) for _ in range(M)]
    got = oracle.average(bufs)
    t = one_layer_table(n // 4, 4, 1, wk.MODE_NONE, 1)
    ref = oracle.project(t, np.stack(bufs), np.zeros(n, np.float32), want_wbar=True)["Wbar"]
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    exact = np.mean(np.stack(bufs).astype(np.float64), axis=0)
    assert np.all(np.abs(got - exact) <= 2.0 ** -22 * np.maximum(np.max(np.abs(np.stack(bufs)), axis=0) * M, 1e-30))


def node_chain(table, n_arena, nodes, a, b, Zg, pack_align=1):
    """One outer iteration's consensus side for M nodes on one device, from oracle calls only.
    nodes: list of dict(W, U, Vd).  Returns dict with per-node Z, U, V and the global mask, z, packed mean."""
    out = {"Z": [], "U": [], "mask_i": []}
    for nd in nodes:
        r = oracle.project_weighted(table, nd["W"], nd["U"], Zg, nd["Vd"], a, b)
        out["Z"].append(r["Z"]); out["U"].append(r["U"]); out["mask_i"].append(r["mask"])
    m = oracle.mask_or(out["mask_i"])                                        # Eq. (14)
    packed = [oracle.compact(table, oracle.add_arenas(table, z, nd["Vd"]), m, pack_align=pack_align)
              for z, nd in zip(out["Z"], nodes)]                             # c_i = z_i + v_i, shrunk under m
    zp = oracle.average([p["packed"] for p in packed])                       # Eq. (11) on the compact buffers
    z = oracle.expand(table, zp, m, n_arena, pack_align=pack_align)
    out.update(mask=m, packed_mean=zp, layer_off=packed[0]["layer_off"], z=z,
               V=[oracle.dual_inter(table, zi, z, nd["Vd"]) for zi, nd in zip(out["Z"], nodes)])   # Eq. (13)
    return out


def test_global_consensus_chain_invariants():
    """z computed through shrink -> mean -> expand equals the plain mean of the c_i masked by the union (nothing the
    union mask drops is nonzero in any z_i; v_i entries outside the union are dropped by the shrinkage, as in the
    paper's pipeline), and with M = 1, v = 0 the chain returns z = z_1 and leaves v at zero."""
    rng = np.random.default_rng(5)
    wl = wk.custom_workload(random_table(rng, 6), R=2, seed=3, sigma_replica=0.03)
    t = wl.table()
    L = len(wl.layers)
    a, b = oracle.node_coefficients(np.full(L, 1.5e-3), np.full(L, 1.5e-4), 1e-4, 3, 2)
    Zg = (0.05 * rng.standard_normal(wl.n_arena)).astype(np.float32)
    nodes = []
    for i in range(3):
        W, U = wk.generate(wk.custom_workload([(l.c_out, l.c_in, l.khw, l.mode, l.k) for l in wl.layers], R=2,
                                              seed=10 + i, sigma_replica=0.03))
        nodes.append({"W": W, "U": U, "Vd": (0.01 * rng.standard_normal(wl.n_arena)).astype(np.float32)})
    ch = node_chain(t, wl.n_arena, nodes, a, b, Zg)
    # reference: mean of full-layout c_i, then the union mask applied element-wise
    c_full = [oracle.add_arenas(t, z, nd["Vd"]) for z, nd in zip(ch["Z"], nodes)]
    mean_full = oracle.average(c_full)
    keep = np.zeros(wl.n_arena, bool)
    for l in wl.layers:
        m = ch["mask"][l.group_base:l.group_base + l.groups].astype(bool)
        m3 = np.broadcast_to(m[None, :, None] if l.mode == wk.MODE_CHANNEL else m[:, None, None],
                             (l.c_out, l.c_in, l.khw))
        keep[l.elem_off:l.elem_off + l.n] = m3.reshape(-1)
    assert np.array_equal(ch["z"][keep].view(np.uint32), mean_full[keep].view(np.uint32))
    assert not ch["z"][~keep].any()
    for zi in ch["Z"]:
        assert not zi[~keep].any()                      # the union contains every node's support
    for v_new, zi, nd in zip(ch["V"], ch["Z"], nodes):
        assert np.array_equal(v_new, (nd["Vd"] + (zi - ch["z"]).astype(np.float32)).astype(np.float32))
    # one node, zero duals: z = z_1, v stays zero
    one = [{"W": nodes[0]["W"], "U": nodes[0]["U"], "Vd": np.zeros(wl.n_arena, np.float32)}]
    c1 = node_chain(t, wl.n_arena, one, a, b, Zg)
    assert np.array_equal(c1["z"].view(np.uint32), c1["Z"][0].view(np.uint32)) and not c1["V"][0].any()
