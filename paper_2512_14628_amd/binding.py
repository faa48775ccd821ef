"""ctypes binding of the C ABI declared in include/hsadmm.h (argument marshalling only).

Device buffers are torch tensors (or raw integer device addresses); torch is used for device memory
and streams and for nothing else.  torch is imported before the library is loaded so that the HIP
runtime the library links against is the one already in the process.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
SRC_PATH = os.path.join(_HERE, "csrc", "hsadmm.hip")
INCLUDE_DIR = os.path.join(_ROOT, "include")
# HSADMM_LIB: load this build of the library instead of the in-tree one (e.g. one whose host code carries sanitizers)
LIB_PATH = os.environ.get("HSADMM_LIB") or os.path.join(_HERE, "libhsadmm.so")

MODE_NONE, MODE_FILTER, MODE_CHANNEL, MODE_BOTH = 0, 1, 2, 3
MAX_REPLICAS = 16

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fPIC", "-shared",
]

EXPORTS = ("hsadmm_plan_create", "hsadmm_plan_destroy", "hsadmm_plan_sizes", "hsadmm_project",
           "hsadmm_compact", "hsadmm_expand", "hsadmm_strerror", "hsadmm_version",
           "hsadmm_kernel_timing_enable", "hsadmm_kernel_timing_read", "hsadmm_kernel_name",
           "hsadmm_project_frozen", "hsadmm_mask_or", "hsadmm_compact_sum", "hsadmm_node_coefficients",
           "hsadmm_plan_set_node_weights", "hsadmm_project_weighted", "hsadmm_dual_inter", "hsadmm_residuals",
           "hsadmm_average", "hsadmm_mask_drift", "hsadmm_expand_dual", "hsadmm_project_compact",
           "hsadmm_project_weighted_compact", "hsadmm_project_frozen_compact",
           "hsadmm_project_weighted_frozen", "hsadmm_project_weighted_frozen_compact",
           "hsadmm_retrain_project", "hsadmm_retrain_expand",
           "hsadmm_adapt_penalties", "hsadmm_scale_layers", "hsadmm_project_compact_static",
           "hsadmm_step", "hsadmm_selection_from_mask", "hsadmm_kernel_grid", "hsadmm_plan_estimates",
           "hsadmm_layer_sqnorms", "hsadmm_stopping_test", "hsadmm_plan_create_nested")
KERNEL_COUNT = 29


class HsadmmError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__("%s failed: %s (code %d)" % (what, hsadmm_strerror(code), code))
        self.code = code


class _Layer(ctypes.Structure):
    _fields_ = [("elem_off", ctypes.c_int64), ("c_out", ctypes.c_int32), ("c_in", ctypes.c_int32),
                ("khw", ctypes.c_int32), ("mode", ctypes.c_int32), ("k", ctypes.c_int32),
                ("k_in", ctypes.c_int32)]


class _Nest(ctypes.Structure):
    _fields_ = [("span", ctypes.c_int32), ("k_coarse", ctypes.c_int32)]


# hsadmm_step_args_t, field by field, in declaration order: (name, C type, how the binding fills it).
#   "dev": device buffer (torch tensor, integer address or None)
_vp = ctypes.c_void_p
_STEP_FIELDS = (
    ("struct_bytes", ctypes.c_size_t, "sizeof"),
    ("W_replicas", ctypes.POINTER(_vp), "replicas"),
    ("R", ctypes.c_int32, "replica_count"),
    ("mappings_cached", ctypes.c_int32, "flag"),
    ("U", _vp, "dev"), ("U_out", _vp, "dev"), ("Zg", _vp, "dev"), ("Vd", _vp, "dev"), ("coef", _vp, "dev"),
    ("Zi_prev", _vp, "dev"), ("mask_frozen", _vp, "dev"), ("sel_prev", _vp, "dev"),
    ("Z", _vp, "dev"), ("Wbar", _vp, "dev"), ("mask", _vp, "dev"), ("sqnorm", _vp, "dev"), ("sel", _vp, "dev"),
    ("packed", _vp, "dev"), ("layer_off", _vp, "dev"), ("kept_idx", _vp, "dev"), ("residuals", _vp, "dev"),
    ("workspace", _vp, "dev"),
    ("workspace_bytes", ctypes.c_size_t, "workspace_size"),
    ("hip_stream", _vp, "stream"),
)


class _StepArgs(ctypes.Structure):
    _fields_ = [(name, ctype) for name, ctype, _ in _STEP_FIELDS]


_lib = None


def build_library(verbose: bool = False) -> str:
    """Compile csrc/hsadmm.hip for gfx950 with hipcc into libhsadmm.so (in-tree)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    cmd = [hipcc, *HIPCC_FLAGS, "-I", INCLUDE_DIR, "-I", os.path.dirname(SRC_PATH), "-o", tmp, SRC_PATH]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed (%d): %s" % (res.returncode, " ".join(cmd)))
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


def load_library():
    """Load libhsadmm.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libhsadmm.so is missing at %s: build it first "
                           "(python -c 'import __graft_entry__ as g; g.build()')" % LIB_PATH)
    import torch  # noqa: F401  (brings the HIP runtime into the process first)
    lib = ctypes.CDLL(LIB_PATH)
    vp = ctypes.c_void_p
    lib.hsadmm_plan_create.argtypes = [ctypes.POINTER(_Layer), ctypes.c_int32, ctypes.c_int32,
                                       ctypes.POINTER(vp)]
    lib.hsadmm_plan_create.restype = ctypes.c_int
    lib.hsadmm_plan_create_nested.argtypes = [ctypes.POINTER(_Layer), ctypes.POINTER(_Nest), ctypes.c_int32,
                                              ctypes.c_int32, ctypes.POINTER(vp)]
    lib.hsadmm_plan_create_nested.restype = ctypes.c_int
    lib.hsadmm_plan_destroy.argtypes = [vp]
    lib.hsadmm_plan_destroy.restype = None
    lib.hsadmm_plan_sizes.argtypes = [vp, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64),
                                      ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_size_t)]
    lib.hsadmm_plan_sizes.restype = ctypes.c_int
    lib.hsadmm_project.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, vp, vp, vp, vp, vp, vp,
                                   ctypes.c_size_t, vp]
    lib.hsadmm_project.restype = ctypes.c_int
    lib.hsadmm_project_compact.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                           ctypes.c_size_t, vp]
    lib.hsadmm_project_compact.restype = ctypes.c_int
    lib.hsadmm_project_compact_static.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp,
                                                  vp, vp]
    lib.hsadmm_project_compact_static.restype = ctypes.c_int
    lib.hsadmm_step.argtypes = [vp, ctypes.POINTER(_StepArgs)]
    lib.hsadmm_step.restype = ctypes.c_int
    lib.hsadmm_selection_from_mask.argtypes = [vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hsadmm_selection_from_mask.restype = ctypes.c_int
    lib.hsadmm_project_frozen.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, vp, vp, vp, vp, vp]
    lib.hsadmm_project_frozen.restype = ctypes.c_int
    lib.hsadmm_project_frozen_compact.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, vp, vp, vp, vp,
                                                  ctypes.c_int32, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hsadmm_project_frozen_compact.restype = ctypes.c_int
    lib.hsadmm_mask_or.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, vp, vp]
    lib.hsadmm_mask_or.restype = ctypes.c_int
    lib.hsadmm_expand_dual.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hsadmm_expand_dual.restype = ctypes.c_int
    lib.hsadmm_mask_drift.argtypes = [vp, vp, vp, vp, vp]
    lib.hsadmm_mask_drift.restype = ctypes.c_int
    lib.hsadmm_average.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, ctypes.c_int64, vp, vp]
    lib.hsadmm_average.restype = ctypes.c_int
    lib.hsadmm_compact_sum.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hsadmm_compact_sum.restype = ctypes.c_int
    f64p = ctypes.POINTER(ctypes.c_double)
    f32p = ctypes.POINTER(ctypes.c_float)
    lib.hsadmm_node_coefficients.argtypes = [f64p, f64p, ctypes.c_int32, ctypes.c_double, ctypes.c_int32,
                                             ctypes.c_int32, f32p, f32p]
    lib.hsadmm_node_coefficients.restype = ctypes.c_int
    lib.hsadmm_plan_set_node_weights.argtypes = [vp, f32p, f32p]
    lib.hsadmm_plan_set_node_weights.restype = ctypes.c_int
    lib.hsadmm_project_weighted.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp, vp,
                                            ctypes.c_size_t, vp]
    lib.hsadmm_project_weighted.restype = ctypes.c_int
    lib.hsadmm_project_weighted_compact.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp,
                                                    vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hsadmm_project_weighted_compact.restype = ctypes.c_int
    lib.hsadmm_project_weighted_frozen.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp]
    lib.hsadmm_project_weighted_frozen.restype = ctypes.c_int
    lib.hsadmm_project_weighted_frozen_compact.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, vp, vp, vp, vp, vp,
                                                           vp, ctypes.c_int32, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hsadmm_project_weighted_frozen_compact.restype = ctypes.c_int
    lib.hsadmm_retrain_project.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, vp, vp, vp, vp, vp, vp,
                                           ctypes.c_int32, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hsadmm_retrain_project.restype = ctypes.c_int
    lib.hsadmm_retrain_expand.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hsadmm_retrain_expand.restype = ctypes.c_int
    dp, fp = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_float)
    lib.hsadmm_adapt_penalties.argtypes = [dp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                           ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                           dp, dp, fp, fp]
    lib.hsadmm_adapt_penalties.restype = ctypes.c_int
    lib.hsadmm_scale_layers.argtypes = [vp, vp, vp, vp]
    lib.hsadmm_scale_layers.restype = ctypes.c_int
    lib.hsadmm_residuals.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hsadmm_residuals.restype = ctypes.c_int
    lib.hsadmm_dual_inter.argtypes = [vp, vp, vp, vp, vp]
    lib.hsadmm_dual_inter.restype = ctypes.c_int
    lib.hsadmm_compact.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hsadmm_compact.restype = ctypes.c_int
    lib.hsadmm_expand.argtypes = [vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hsadmm_expand.restype = ctypes.c_int
    lib.hsadmm_strerror.argtypes = [ctypes.c_int]
    lib.hsadmm_strerror.restype = ctypes.c_char_p
    lib.hsadmm_version.argtypes = []
    lib.hsadmm_version.restype = ctypes.c_int
    lib.hsadmm_kernel_timing_enable.argtypes = [vp, ctypes.c_int]
    lib.hsadmm_kernel_timing_enable.restype = ctypes.c_int
    lib.hsadmm_kernel_timing_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.hsadmm_kernel_timing_read.restype = ctypes.c_int
    lib.hsadmm_layer_sqnorms.argtypes = [vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hsadmm_layer_sqnorms.restype = ctypes.c_int
    lib.hsadmm_stopping_test.argtypes = [ctypes.POINTER(ctypes.c_int64), ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                         dp, dp, dp, dp, ctypes.c_double,
                                         ctypes.c_double, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
    lib.hsadmm_stopping_test.restype = ctypes.c_int
    lib.hsadmm_kernel_grid.argtypes = [vp, ctypes.c_int]
    lib.hsadmm_kernel_grid.restype = ctypes.c_int
    lib.hsadmm_plan_estimates.argtypes = [vp]
    lib.hsadmm_plan_estimates.restype = ctypes.c_int
    lib.hsadmm_kernel_name.argtypes = [ctypes.c_int]
    lib.hsadmm_kernel_name.restype = ctypes.c_char_p
    _lib = lib
    return lib


def exported_symbols():
    """Names include/hsadmm.h declares, each resolved in the loaded library."""
    lib = load_library()
    return {name: getattr(lib, name) for name in EXPORTS}


def hsadmm_strerror(code: int) -> str:
    return load_library().hsadmm_strerror(int(code)).decode()


def hsadmm_version() -> int:
    return int(load_library().hsadmm_version())


def _ptr(x) -> Optional[int]:
    """Device address of a torch tensor, or an integer address passed through; None -> NULL."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _nbytes(x) -> int:
    return int(x.numel() * x.element_size())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


class Plan:
    """Owner of an hsadmm_plan_t*.  `table` has the columns elem_off, c_out, c_in, khw, mode, k and, when it
    holds layers under both constraints (mode 3), k_in.  With the columns span and k_coarse (runs of channels,
    hsadmm_nest_t) the plan is made by hsadmm_plan_create_nested."""

    def __init__(self, table, pack_align_elems: int = 1):
        lib = load_library()
        L = len(table["c_out"])
        arr = (_Layer * max(L, 1))()
        for i in range(L):
            arr[i].elem_off = int(table["elem_off"][i])
            arr[i].c_out = int(table["c_out"][i])
            arr[i].c_in = int(table["c_in"][i])
            arr[i].khw = int(table["khw"][i])
            arr[i].mode = int(table["mode"][i])
            arr[i].k = int(table["k"][i])
            arr[i].k_in = int(table["k_in"][i]) if "k_in" in table else 0
        handle = ctypes.c_void_p()
        self.handle = None
        if "span" in table:
            nest = (_Nest * max(L, 1))()
            for i in range(L):
                nest[i].span = int(table["span"][i])
                nest[i].k_coarse = int(table["k_coarse"][i])
            rc = lib.hsadmm_plan_create_nested(arr, nest, L, int(pack_align_elems), ctypes.byref(handle))
            if rc != 0:
                raise HsadmmError(rc, "hsadmm_plan_create_nested")
        else:
            rc = lib.hsadmm_plan_create(arr, L, int(pack_align_elems), ctypes.byref(handle))
            if rc != 0:
                raise HsadmmError(rc, "hsadmm_plan_create")
        self.handle = handle
        self.n_layers = L
        self.pack_align_elems = int(pack_align_elems)
        a, g, c, w = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_size_t()
        rc = lib.hsadmm_plan_sizes(self.handle, ctypes.byref(a), ctypes.byref(g), ctypes.byref(c),
                                   ctypes.byref(w))
        if rc != 0:
            raise HsadmmError(rc, "hsadmm_plan_sizes")
        self.arena_elems, self.groups_total = a.value, g.value
        self.packed_capacity_elems, self.workspace_bytes = c.value, w.value

    def close(self):
        if getattr(self, "handle", None):
            load_library().hsadmm_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def hsadmm_kernel_timing_enable(plan: Plan, enable: bool) -> None:
    rc = load_library().hsadmm_kernel_timing_enable(plan.handle, 1 if enable else 0)
    if rc != 0:
        raise HsadmmError(rc, "hsadmm_kernel_timing_enable")


def hsadmm_kernel_timing_read(plan: Plan):
    """{kernel name: (total milliseconds, launches)} since the last read."""
    lib = load_library()
    ms = (ctypes.c_double * KERNEL_COUNT)()
    cnt = (ctypes.c_int64 * KERNEL_COUNT)()
    rc = lib.hsadmm_kernel_timing_read(plan.handle, ms, cnt)
    if rc != 0:
        raise HsadmmError(rc, "hsadmm_kernel_timing_read")
    return {lib.hsadmm_kernel_name(i).decode(): (float(ms[i]), int(cnt[i])) for i in range(KERNEL_COUNT)}


def hsadmm_plan_estimates(plan: Plan) -> bool:
    """Whether this plan's un-predicted projection forms a prediction inside pass 1 (see include/hsadmm.h)."""
    return bool(load_library().hsadmm_plan_estimates(plan.handle))


def hsadmm_kernel_grids(plan: Plan):
    """{kernel name: workgroups of its latest timed launch on this plan} (0: not launched with timing on)."""
    lib = load_library()
    return {lib.hsadmm_kernel_name(i).decode(): int(lib.hsadmm_kernel_grid(plan.handle, i)) for i in range(KERNEL_COUNT)}


def hsadmm_project(plan: Plan, W_replicas: Sequence, U, Z, Wbar, mask, sqnorm, workspace,
                   stream=None, workspace_bytes: Optional[int] = None, check: bool = True) -> int:
    lib = load_library()
    R = len(W_replicas)
    ptrs = (ctypes.c_void_p * max(R, 1))(*[_ptr(w) for w in W_replicas])
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_project(plan.handle, ptrs, R, _ptr(U), _ptr(Z), _ptr(Wbar), _ptr(mask), _ptr(sqnorm),
                            _ptr(workspace), wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_project")
    return rc


def hsadmm_project_compact(plan: Plan, W_replicas: Sequence, U, Z, Wbar, mask, sqnorm, packed, layer_off, kept_idx,
                           workspace, stream=None, workspace_bytes: Optional[int] = None, check: bool = True) -> int:
    lib = load_library()
    R = len(W_replicas)
    ptrs = (ctypes.c_void_p * max(R, 1))(*[_ptr(w) for w in W_replicas])
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_project_compact(plan.handle, ptrs, R, _ptr(U), _ptr(Z), _ptr(Wbar), _ptr(mask), _ptr(sqnorm),
                                    _ptr(packed), _ptr(layer_off), _ptr(kept_idx), _ptr(workspace), wb,
                                    _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_project_compact")
    return rc


def hsadmm_project_compact_static(plan: Plan, W_replicas: Sequence, U, Z, Wbar, mask, sqnorm, packed, layer_off,
                                  kept_idx, stream=None, check: bool = True) -> int:
    """hsadmm_project_compact on the library's static scratch array (no workspace argument, no allocation)."""
    lib = load_library()
    R = len(W_replicas)
    ptrs = (ctypes.c_void_p * max(R, 1))(*[_ptr(w) for w in W_replicas])
    rc = lib.hsadmm_project_compact_static(plan.handle, ptrs, R, _ptr(U), _ptr(Z), _ptr(Wbar), _ptr(mask),
                                           _ptr(sqnorm), _ptr(packed), _ptr(layer_off), _ptr(kept_idx),
                                           _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_project_compact_static")
    return rc


def hsadmm_step(plan: Plan, W_replicas: Sequence, stream=None, workspace_bytes: Optional[int] = None,
                check: bool = True, **fields) -> int:
    """hsadmm_step: every form of the projection step through one argument structure.  Keyword arguments are the
    device-buffer fields of hsadmm_step_args_t (U, Z, mask, packed, sel_prev, ...) and the flag mappings_cached;
    fields that are not given stay NULL."""
    lib = load_library()
    R = len(W_replicas)
    ptrs = (ctypes.c_void_p * max(R, 1))(*[_ptr(w) for w in W_replicas])
    args = _StepArgs()
    known = {name for name, _, how in _STEP_FIELDS if how in ("dev", "flag")}
    unknown = set(fields) - known
    if unknown:
        raise TypeError("hsadmm_step has no field(s) %s" % ", ".join(sorted(unknown)))
    for name, _, how in _STEP_FIELDS:
        if how == "sizeof":
            value = ctypes.sizeof(_StepArgs)
        elif how == "replicas":
            value = ptrs
        elif how == "replica_count":
            value = R
        elif how == "flag":
            value = 1 if fields.get(name) else 0
        elif how == "dev":
            value = _ptr(fields.get(name))
        elif how == "workspace_size":
            ws = fields.get("workspace")
            value = int(workspace_bytes) if workspace_bytes is not None else (0 if ws is None or isinstance(ws, int)
                                                                             else _nbytes(ws))
        else:
            value = _stream(stream)
        setattr(args, name, value)
    rc = lib.hsadmm_step(plan.handle, ctypes.byref(args))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_step")
    return rc


def hsadmm_selection_from_mask(plan: Plan, mask, sel, workspace, stream=None, workspace_bytes: Optional[int] = None,
                               check: bool = True) -> int:
    """sel[g] = rank of group g among its layer's groups kept by `mask`, -1 if not kept."""
    lib = load_library()
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_selection_from_mask(plan.handle, _ptr(mask), _ptr(sel), _ptr(workspace), wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_selection_from_mask")
    return rc


def hsadmm_project_frozen(plan: Plan, W_replicas: Sequence, U, Z, Wbar, mask, stream=None, check: bool = True) -> int:
    lib = load_library()
    R = len(W_replicas)
    ptrs = (ctypes.c_void_p * max(R, 1))(*[_ptr(w) for w in W_replicas])
    rc = lib.hsadmm_project_frozen(plan.handle, ptrs, R, _ptr(U), _ptr(Z), _ptr(Wbar), _ptr(mask), _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_project_frozen")
    return rc


def hsadmm_project_frozen_compact(plan: Plan, W_replicas: Sequence, U, Z, Wbar, mask, mappings_cached: bool, packed,
                                  layer_off, kept_idx, workspace, stream=None, workspace_bytes: Optional[int] = None,
                                  check: bool = True) -> int:
    lib = load_library()
    R = len(W_replicas)
    ptrs = (ctypes.c_void_p * max(R, 1))(*[_ptr(w) for w in W_replicas])
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_project_frozen_compact(plan.handle, ptrs, R, _ptr(U), _ptr(Z), _ptr(Wbar), _ptr(mask),
                                           1 if mappings_cached else 0, _ptr(packed), _ptr(layer_off),
                                           _ptr(kept_idx), _ptr(workspace), wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_project_frozen_compact")
    return rc


def hsadmm_mask_or(plan: Plan, masks: Sequence, out, stream=None, check: bool = True) -> int:
    lib = load_library()
    M = len(masks)
    ptrs = (ctypes.c_void_p * max(M, 1))(*[_ptr(m) for m in masks])
    rc = lib.hsadmm_mask_or(plan.handle, ptrs, M, _ptr(out), _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_mask_or")
    return rc


def hsadmm_mask_drift(plan: Plan, mask_a, mask_b, drift, stream=None, check: bool = True) -> int:
    """Section 4.5: drift[l] = groups of layer l whose kept flag differs between the two masks."""
    rc = load_library().hsadmm_mask_drift(plan.handle, _ptr(mask_a), _ptr(mask_b), _ptr(drift), _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_mask_drift")
    return rc


def hsadmm_average(plan: Plan, bufs: Sequence, n_elems: int, out, stream=None, check: bool = True) -> int:
    """Eq. (11): out = mean of the M buffers (each n_elems floats)."""
    lib = load_library()
    M = len(bufs)
    ptrs = (ctypes.c_void_p * max(M, 1))(*[_ptr(b) for b in bufs])
    rc = lib.hsadmm_average(plan.handle, ptrs, M, int(n_elems), _ptr(out), _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_average")
    return rc


def hsadmm_node_coefficients(rho1, rho2, lam: float, M: int, P: int):
    """Eq. (9) weights as two lists of L floats (host computation inside the library)."""
    lib = load_library()
    L = len(rho1)
    r1 = (ctypes.c_double * L)(*[float(x) for x in rho1])
    r2 = (ctypes.c_double * L)(*[float(x) for x in rho2])
    a = (ctypes.c_float * L)()
    b = (ctypes.c_float * L)()
    rc = lib.hsadmm_node_coefficients(r1, r2, L, float(lam), int(M), int(P), a, b)
    if rc != 0:
        raise HsadmmError(rc, "hsadmm_node_coefficients")
    return list(a), list(b)


def hsadmm_adapt_penalties(residuals, rho1, rho2, P: int, n_out: int, mu: float, tau_incr: float, tau_decr: float,
                           rho1_max: float, rho2_max: float):
    """Residual balancing per layer and level (host computation inside the library).  residuals: 4*L floats on the
    host, rows as hsadmm_residuals writes them.  Returns (rho1, rho2, scale_u, scale_v) as lists of L numbers."""
    lib = load_library()
    L = len(rho1)
    flat = [float(x) for row in residuals for x in (row if hasattr(row, "__len__") else [row])]
    if len(flat) != 4 * L or len(rho2) != L:
        raise ValueError("residuals need 4 entries per layer, rho1 and rho2 one")
    sq = (ctypes.c_double * (4 * L))(*flat)
    r1 = (ctypes.c_double * L)(*[float(x) for x in rho1])
    r2 = (ctypes.c_double * L)(*[float(x) for x in rho2])
    su = (ctypes.c_float * L)()
    sv = (ctypes.c_float * L)()
    rc = lib.hsadmm_adapt_penalties(sq, L, int(P), int(n_out), float(mu), float(tau_incr), float(tau_decr),
                                    float(rho1_max), float(rho2_max), r1, r2, su, sv)
    if rc != 0:
        raise HsadmmError(rc, "hsadmm_adapt_penalties")
    return list(r1), list(r2), list(su), list(sv)


def hsadmm_layer_sqnorms(plan: Plan, X, out, workspace, stream=None, workspace_bytes: Optional[int] = None,
                         check: bool = True) -> int:
    """out[l] = squared Frobenius norm of layer l of the arena X (fp64, on the device)."""
    lib = load_library()
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_layer_sqnorms(plan.handle, _ptr(X), _ptr(out), _ptr(workspace), wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_layer_sqnorms")
    return rc


def hsadmm_stopping_test(n_elems, P: int, n_out: int, rho1, rho2, residuals, magnitudes, eps_abs: float,
                         eps_rel: float):
    """Section 3.4's stopping test on the host.  n_elems: elements per layer; residuals: 4*L numbers, magnitudes:
    5*L numbers (rows as in the header).  Returns (list of L flags, all_done)."""
    lib = load_library()
    L = len(n_elems)
    ne = (ctypes.c_int64 * L)(*[int(x) for x in n_elems])

    def flat(x, rows):
        v = [float(y) for r in x for y in (r if hasattr(r, "__len__") else [r])]
        if len(v) != rows * L:
            raise ValueError("%d numbers per layer expected" % rows)
        return (ctypes.c_double * len(v))(*v)
    if len(rho1) != L or len(rho2) != L:
        raise ValueError("one penalty per layer and level")
    r1 = (ctypes.c_double * L)(*[float(x) for x in rho1])
    r2 = (ctypes.c_double * L)(*[float(x) for x in rho2])
    done = (ctypes.c_int32 * L)()
    every = ctypes.c_int32(-1)
    rc = lib.hsadmm_stopping_test(ne, L, int(P), int(n_out), r1, r2, flat(residuals, 4), flat(magnitudes, 5),
                                  float(eps_abs), float(eps_rel), done, ctypes.byref(every))
    if rc != 0:
        raise HsadmmError(rc, "hsadmm_stopping_test")
    return list(done), bool(every.value)


def hsadmm_scale_layers(plan: Plan, X, factor, stream=None, check: bool = True) -> int:
    """X *= factor[layer] on the device (factor: L floats on the device)."""
    lib = load_library()
    rc = lib.hsadmm_scale_layers(plan.handle, _ptr(X), _ptr(factor), _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_scale_layers")
    return rc


def hsadmm_plan_set_node_weights(plan: Plan, a, b) -> None:
    lib = load_library()
    L = plan.n_layers
    if len(a) != L or len(b) != L:
        raise ValueError("a and b need one entry per layer")
    fa = (ctypes.c_float * L)(*[float(x) for x in a])
    fb = (ctypes.c_float * L)(*[float(x) for x in b])
    rc = lib.hsadmm_plan_set_node_weights(plan.handle, fa, fb)
    if rc != 0:
        raise HsadmmError(rc, "hsadmm_plan_set_node_weights")


def hsadmm_project_weighted(plan: Plan, W_replicas: Sequence, U, Zg, Vd, Z, Wbar, mask, sqnorm, workspace,
                            stream=None, workspace_bytes: Optional[int] = None, check: bool = True) -> int:
    lib = load_library()
    R = len(W_replicas)
    ptrs = (ctypes.c_void_p * max(R, 1))(*[_ptr(w) for w in W_replicas])
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_project_weighted(plan.handle, ptrs, R, _ptr(U), _ptr(Zg), _ptr(Vd), _ptr(Z), _ptr(Wbar),
                                     _ptr(mask), _ptr(sqnorm), _ptr(workspace), wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_project_weighted")
    return rc


def hsadmm_project_weighted_compact(plan: Plan, W_replicas: Sequence, U, Zg, Vd, Z, Wbar, mask, sqnorm, packed,
                                    layer_off, kept_idx, workspace, stream=None,
                                    workspace_bytes: Optional[int] = None, check: bool = True) -> int:
    lib = load_library()
    R = len(W_replicas)
    ptrs = (ctypes.c_void_p * max(R, 1))(*[_ptr(w) for w in W_replicas])
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_project_weighted_compact(plan.handle, ptrs, R, _ptr(U), _ptr(Zg), _ptr(Vd), _ptr(Z), _ptr(Wbar),
                                             _ptr(mask), _ptr(sqnorm), _ptr(packed), _ptr(layer_off),
                                             _ptr(kept_idx), _ptr(workspace), wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_project_weighted_compact")
    return rc


def hsadmm_project_weighted_frozen(plan: Plan, W_replicas: Sequence, U, Zg, Vd, Z, Wbar, mask, stream=None,
                                   check: bool = True) -> int:
    lib = load_library()
    R = len(W_replicas)
    ptrs = (ctypes.c_void_p * max(R, 1))(*[_ptr(w) for w in W_replicas])
    rc = lib.hsadmm_project_weighted_frozen(plan.handle, ptrs, R, _ptr(U), _ptr(Zg), _ptr(Vd), _ptr(Z), _ptr(Wbar),
                                            _ptr(mask), _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_project_weighted_frozen")
    return rc


def hsadmm_project_weighted_frozen_compact(plan: Plan, W_replicas: Sequence, U, Zg, Vd, Z, Wbar, mask,
                                           mappings_cached: bool, packed, layer_off, kept_idx, workspace, stream=None,
                                           workspace_bytes: Optional[int] = None, check: bool = True) -> int:
    lib = load_library()
    R = len(W_replicas)
    ptrs = (ctypes.c_void_p * max(R, 1))(*[_ptr(w) for w in W_replicas])
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_project_weighted_frozen_compact(plan.handle, ptrs, R, _ptr(U), _ptr(Zg), _ptr(Vd), _ptr(Z),
                                                    _ptr(Wbar), _ptr(mask), 1 if mappings_cached else 0,
                                                    _ptr(packed), _ptr(layer_off), _ptr(kept_idx), _ptr(workspace),
                                                    wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_project_weighted_frozen_compact")
    return rc


def hsadmm_retrain_project(plan: Plan, W_replicas: Sequence, U, Zg, Vd, Z, Wbar, mask, mappings_cached: bool,
                           packed, layer_off, kept_idx, residuals, workspace, stream=None,
                           workspace_bytes: Optional[int] = None, check: bool = True) -> int:
    """hsadmm_project_weighted_frozen_compact that also writes rows 0 and 1 of `residuals` (Z in: previous z_i)."""
    lib = load_library()
    R = len(W_replicas)
    ptrs = (ctypes.c_void_p * max(R, 1))(*[_ptr(w) for w in W_replicas])
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_retrain_project(plan.handle, ptrs, R, _ptr(U), _ptr(Zg), _ptr(Vd), _ptr(Z), _ptr(Wbar),
                                    _ptr(mask), 1 if mappings_cached else 0, _ptr(packed), _ptr(layer_off),
                                    _ptr(kept_idx), _ptr(residuals), _ptr(workspace), wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_retrain_project")
    return rc


def hsadmm_retrain_expand(plan: Plan, packed, mask, dst, Zi, Vd, z_prev, residuals, workspace, stream=None,
                          workspace_bytes: Optional[int] = None, check: bool = True) -> int:
    """hsadmm_expand_dual that also writes rows 2 and 3 of `residuals` (z_prev: the previous global consensus)."""
    lib = load_library()
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_retrain_expand(plan.handle, _ptr(packed), _ptr(mask), _ptr(dst), _ptr(Zi), _ptr(Vd), _ptr(z_prev),
                                   _ptr(residuals), _ptr(workspace), wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_retrain_expand")
    return rc


def hsadmm_residuals(plan: Plan, W_replicas: Sequence, Zi, Zi_prev, Zg, Zg_prev, out, workspace, stream=None,
                     workspace_bytes: Optional[int] = None, check: bool = True) -> int:
    lib = load_library()
    R = len(W_replicas)
    ptrs = (ctypes.c_void_p * max(R, 1))(*[_ptr(w) for w in W_replicas])
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_residuals(plan.handle, ptrs, R, _ptr(Zi), _ptr(Zi_prev), _ptr(Zg), _ptr(Zg_prev), _ptr(out),
                              _ptr(workspace), wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_residuals")
    return rc


def hsadmm_dual_inter(plan: Plan, Zi, Zg, Vd, stream=None, check: bool = True) -> int:
    rc = load_library().hsadmm_dual_inter(plan.handle, _ptr(Zi), _ptr(Zg), _ptr(Vd), _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_dual_inter")
    return rc


def hsadmm_compact_sum(plan: Plan, src0, src1, mask, packed, layer_off, kept_idx, workspace, stream=None,
                       workspace_bytes: Optional[int] = None, check: bool = True) -> int:
    lib = load_library()
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_compact_sum(plan.handle, _ptr(src0), _ptr(src1), _ptr(mask), _ptr(packed), _ptr(layer_off),
                                _ptr(kept_idx), _ptr(workspace), wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_compact_sum")
    return rc


def hsadmm_compact(plan: Plan, src, mask, packed, layer_off, kept_idx, workspace, stream=None,
                   workspace_bytes: Optional[int] = None, check: bool = True) -> int:
    lib = load_library()
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_compact(plan.handle, _ptr(src), _ptr(mask), _ptr(packed), _ptr(layer_off), _ptr(kept_idx),
                            _ptr(workspace), wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_compact")
    return rc


def hsadmm_expand(plan: Plan, packed, mask, dst, workspace, stream=None,
                  workspace_bytes: Optional[int] = None, check: bool = True) -> int:
    lib = load_library()
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_expand(plan.handle, _ptr(packed), _ptr(mask), _ptr(dst), _ptr(workspace), wb,
                           _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_expand")
    return rc


def hsadmm_expand_dual(plan: Plan, packed, mask, dst, Zi, Vd, workspace, stream=None,
                       workspace_bytes: Optional[int] = None, check: bool = True) -> int:
    """hsadmm_expand with Vd <- Vd + (Zi - dst) (Eq. (13)) applied in the same pass."""
    lib = load_library()
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    rc = lib.hsadmm_expand_dual(plan.handle, _ptr(packed), _ptr(mask), _ptr(dst), _ptr(Zi), _ptr(Vd), _ptr(workspace),
                                wb, _stream(stream))
    if check and rc != 0:
        raise HsadmmError(rc, "hsadmm_expand_dual")
    return rc
