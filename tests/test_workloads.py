"""The seeded input module: table sizes of the named configurations (the figures the byte accounting rests on),
reproducibility of the draws, and that it holds none of the method's arithmetic.  CPU only."""
import ast
import os

import numpy as np
import pytest

import workloads as wk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("name,layers,n_total,groups,n_kept", [
    ("tiny", 5, 33_328, 154, 16_664),
    ("resnet18", 21, 11_678_912, 4_800 + 1000, 4_978_926),
    ("resnet50", 54, 25_502_912, 26_560 + 1000, 11_426_030),
    ("resnet152", 156, 60_040_384, 71_683 + 1000, 19_470_400),
    ("wrn50_2", 54, 68_814_016, None, None),
])
def test_named_configurations_have_the_published_sizes(name, layers, n_total, groups, n_kept):
    """Layer counts and parameter counts of the conv / fc weights of the models the paper trains (Section 5.1), and
    the kept-parameter counts that follow from the keep ratios (fc kept whole: its 1000 groups are counted)."""
    wl = wk.make_workload(name)
    assert len(wl.layers) == layers and wl.n_total == n_total
    if groups is not None:
        expect = groups if name != "tiny" else 154
        assert wl.groups_total == expect
    if n_kept is not None:
        assert wl.n_kept == n_kept
    offs = [l.elem_off for l in wl.layers]
    assert all(o % 4 == 0 for o in offs) and all(b >= a + l.n for a, b, l in zip(offs, offs[1:], wl.layers))
    b = wl.algorithmic_bytes()
    assert b["project"] == 4 * wl.n_total * (wl.R + 3) and b["step"] == 4 * wl.n_total * (wl.R + 4) + 12 * wl.n_kept


def test_resnet50_step_moves_953_MB():
    assert wk.make_workload("resnet50").algorithmic_bytes()["step"] == 953_205_544


def test_draws_are_reproducible_and_per_layer():
    wl = wk.make_workload("tiny", seed=3)
    W1, U1 = wk.generate(wl)
    W2, U2 = wk.generate(wk.make_workload("tiny", seed=3), threads=4)
    assert np.array_equal(W1, W2) and np.array_equal(U1, U2)
    W3, _ = wk.generate(wk.make_workload("tiny", seed=4))
    assert not np.array_equal(W1, W3)
    reps, u = wk.generate_layer(wl, 2)                       # any layer alone gives the same values
    l = wl.layers[2]
    assert np.array_equal(reps[0], W1[0, l.elem_off:l.elem_off + l.n]) and np.array_equal(u, U1[l.elem_off:l.elem_off + l.n])
    # the value recipe: He-normal weights, duals of variance 1e-4, replica noise of variance 1e-3
    big = wk.make_workload("resnet18")
    Wb, Ub = wk.generate(big, threads=4)
    l = big.layers[5]
    w = Wb[0, l.elem_off:l.elem_off + l.n]
    assert abs(float(np.var(w)) / (2.0 / l.fan_in) - 1.0) < 0.05
    assert abs(float(np.var(Ub[l.elem_off:l.elem_off + l.n])) / 1e-4 - 1.0) < 0.05
    r50 = wk.make_workload("resnet50")
    reps, _ = wk.generate_layer(r50, 10)
    assert abs(float(np.var(reps[1] - reps[0])) / 2e-3 - 1.0) < 0.1


def test_keep_count_rounds_half_up_and_clamps():
    assert [wk.keep_count(0.4, g) for g in (64, 3, 1, 5)] == [26, 1, 1, 2]
    assert wk.keep_count(0.5, 5) == 3 and wk.keep_count(0.0, 7) == 1 and wk.keep_count(1.5, 7) == 7


def test_the_shared_module_holds_none_of_the_methods_arithmetic():
    """workloads.py is the only module both sides import: it may draw numbers and build tables, nothing else."""
    src = open(os.path.join(ROOT, "workloads.py")).read()
    tree = ast.parse(src)
    imported = {n.names[0].name.split(".")[0] for n in ast.walk(tree) if isinstance(n, ast.Import)}
    imported |= {n.module.split(".")[0] for n in ast.walk(tree) if isinstance(n, ast.ImportFrom) and n.module}
    assert imported <= {"__future__", "dataclasses", "typing", "numpy", "concurrent"}
    used = {n.id for n in ast.walk(tree) if isinstance(n, ast.Name)}
    used |= {n.attr for n in ast.walk(tree) if isinstance(n, ast.Attribute)}
    assert not used & {"argsort", "argpartition", "partition", "sort", "cumsum", "linalg", "norm", "mean", "average",
                       "topk", "oracle", "paper_2512_14628_amd"}
