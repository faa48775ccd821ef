"""The C ABI from a process that holds neither Python nor PyTorch: tests/c_client/step_client.c (plain C99, device
memory from hipMalloc; built by __graft_entry__.build()) reads a layer table and inputs from a file, runs one step
through the named calls and a second one through hsadmm_step with a prediction and the dual out of place, and writes
the outputs, which are compared here with the oracle's on every element."""
import os
import struct
import subprocess

import numpy as np
import pytest

import oracle
import workloads as wk

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLIENT = os.path.join(ROOT, "tests", "c_client", "step_client")


@pytest.mark.parametrize("pack_align", [1, 4])
def test_a_plain_c_program_runs_two_steps(tmp_path, pack_align):
    if not os.path.exists(CLIENT):      # normally built by __graft_entry__.build(); host code only, a second with gcc
        import __graft_entry__ as entry
        import paper_2512_14628_amd as pkg
        entry.build_c_client(pkg.LIB_PATH)
    from tests.test_gpu_hinted import SHAPES
    wl = wk.custom_workload(SHAPES, R=3, seed=9, sigma_replica=0.03)
    W, U = wk.generate(wl)
    t = wl.table()
    L = len(wl.layers)
    inp, outp = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(inp, "wb") as f:
        f.write(struct.pack("=iii", L, wl.R, pack_align))
        for l in wl.layers:
            f.write(struct.pack("=qiiiiii", l.elem_off, l.c_out, l.c_in, l.khw, l.mode, l.k, getattr(l, "k_in", 0) or 0))
        f.write(struct.pack("=q", wl.n_arena))
        for r in range(wl.R):
            f.write(np.ascontiguousarray(W[r], dtype=np.float32).tobytes())
        f.write(np.ascontiguousarray(U, dtype=np.float32).tobytes())
    env = dict(os.environ)
    env.pop("PYTHONPATH", None)
    done = subprocess.run([CLIENT, str(inp), str(outp)], capture_output=True, text=True, timeout=100, env=env)
    assert done.returncode == 0, (done.returncode, done.stdout[-500:], done.stderr[-2000:])
    raw = np.fromfile(outp, dtype=np.uint8)
    n, G = wl.n_arena, wl.groups_total
    pos = 0

    def take(count, dtype):
        nonlocal pos
        nbytes = count * np.dtype(dtype).itemsize
        a = raw[pos:pos + nbytes].view(dtype)
        pos += nbytes
        return a

    u_in = U
    for step in range(2):
        ref = oracle.project(t, W, u_in)
        refc = oracle.compact(t, ref["Z"], ref["mask"], pack_align=pack_align)
        Z, Unew, dst = take(n, np.float32), take(n, np.float32), take(n, np.float32)
        mask, off = take(G, np.uint8), take(L + 1, np.int64)
        packed = take(int(off[-1]), np.float32)
        assert np.array_equal(mask, ref["mask"]), step
        assert np.array_equal(off, refc["layer_off"]), step
        for l in wl.layers:
            sl = slice(l.elem_off, l.elem_off + l.n)
            for got, want, name in ((Z, ref["Z"], "Z"), (Unew, ref["U"], "U"), (dst, ref["Z"], "dst")):
                assert np.array_equal(got[sl].view(np.uint32), want[sl].view(np.uint32)), (step, name, l.name)
        from tests.gpu_harness import packed_segment_sizes
        sizes = packed_segment_sizes(wl, ref["mask"])
        for li in range(L):
            lo = int(off[li])
            assert np.array_equal(packed[lo:lo + sizes[li]].view(np.uint32),
                                  refc["packed"][lo:lo + sizes[li]].view(np.uint32)), (step, li)
        u_in = ref["U"]
    assert pos == raw.size
