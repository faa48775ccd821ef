"""Seeded synthetic workloads for the H-SADMM structured-sparsity step.

This module builds layer tables (shapes, group mode, number of groups kept) and
draws the input tensors.  It is the only module shared by the CPU oracle's
tests and the HIP path's tests / benchmark, and it holds none of the method's
arithmetic: no averaging, norms, selection, dual update or packing happens
here.

Shapes follow the torchvision-style ResNets the paper trains (Section 5.1,
Table 2): weights of every conv layer W[C_out, C_in, K_H, K_W] and of the final
linear layer W[d_out, d_in] (Section 2, first paragraph), row-major fp32.  The
values are synthetic: He-normal weights, small Gaussian duals, replicas equal
to the base weight plus Gaussian noise.

Random draws use one Philox stream per (layer, tensor, replica), so any layer
can be generated alone and in any order.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

MODE_NONE = 0      # no constraint on this layer: every filter is kept
MODE_FILTER = 1    # groups are output filters  W[g, :, :, :]
MODE_CHANNEL = 2   # groups are input channels  W[:, g, :, :]
MODE_BOTH = 3      # both constraints: c_out filter groups followed by c_in channel groups
MODE_SHAPE = 4     # groups are the spatial positions of the input channels  W[:, b, u, v]  (c_in * khw groups)
MODE_CHANNEL_SHAPE = 5   # channels and shape groups: c_in channel groups followed by c_in * khw shape groups
MODE_ALL = 6       # filters, channels and shape groups: c_out + c_in + c_in * khw groups

_TENSOR_W = 0
_TENSOR_U = 1
_TENSOR_REPLICA0 = 2      # + r
_TENSOR_SCALE = 100
_TENSOR_KEEP = 101


@dataclass
class Layer:
    name: str
    c_out: int
    c_in: int
    khw: int
    mode: int = MODE_NONE
    k: int = 0
    k_in: int = 0              # MODE_BOTH, MODE_CHANNEL_SHAPE, MODE_ALL: channels kept (k is the number of filters kept)
    k_kern: int = 0            # MODE_CHANNEL_SHAPE, MODE_ALL: shape groups kept, all of them inside kept channels
    elem_off: int = 0          # offset, in elements, inside every full-layout arena
    group_base: int = 0        # offset of this layer's groups in mask / sqnorm

    @property
    def n(self) -> int:
        return self.c_out * self.c_in * self.khw

    @property
    def groups(self) -> int:
        if self.mode == MODE_BOTH:
            return self.c_out + self.c_in
        if self.mode == MODE_SHAPE:
            return self.c_in * self.khw
        if self.mode == MODE_CHANNEL_SHAPE:
            return self.c_in + self.c_in * self.khw
        if self.mode == MODE_ALL:
            return self.c_out + self.c_in + self.c_in * self.khw
        return self.c_in if self.mode == MODE_CHANNEL else self.c_out

    @property
    def group_size(self) -> int:
        """Elements per group (MODE_BOTH: of a filter group)."""
        if self.mode == MODE_SHAPE:
            return self.c_out
        return (self.c_out if self.mode == MODE_CHANNEL else self.c_in) * self.khw

    @property
    def fan_in(self) -> int:
        return self.c_in * self.khw

    @property
    def kept_elems(self) -> int:
        if self.mode == MODE_NONE:
            return self.n
        if self.mode == MODE_BOTH:
            return self.k * self.k_in * self.khw
        if self.mode == MODE_CHANNEL_SHAPE:
            return self.c_out * self.k_kern
        if self.mode == MODE_ALL:
            return self.k * self.k_kern
        return self.k * self.group_size


@dataclass
class Workload:
    name: str
    layers: List[Layer]
    R: int
    seed: int = 0
    sigma_u: float = 1e-2            # U ~ N(0, var 1e-4)
    sigma_replica: float = 0.0       # replica_r = W + N(0, var sigma^2); 0: replicas equal W
    filter_scale_log10: Optional[Tuple[float, float]] = None   # per-filter scale 10^U(a,b)
    description: str = ""
    n_arena: int = field(default=0)
    groups_total: int = field(default=0)

    @property
    def n_total(self) -> int:
        return sum(l.n for l in self.layers)

    @property
    def n_kept(self) -> int:
        return sum(l.kept_elems for l in self.layers)

    def table(self):
        """Plain integer columns of the layer table (what both implementations take)."""
        cols = {
            "elem_off": np.array([l.elem_off for l in self.layers], dtype=np.int64),
            "c_out": np.array([l.c_out for l in self.layers], dtype=np.int32),
            "c_in": np.array([l.c_in for l in self.layers], dtype=np.int32),
            "khw": np.array([l.khw for l in self.layers], dtype=np.int32),
            "mode": np.array([l.mode for l in self.layers], dtype=np.int32),
            "k": np.array([l.k for l in self.layers], dtype=np.int32),
            "k_in": np.array([l.k_in for l in self.layers], dtype=np.int32),
            "k_kern": np.array([l.k_kern for l in self.layers], dtype=np.int32),
        }
        return cols

    def gemm_view_table(self):
        """The same layers with every MODE_SHAPE layer declared as what it is in the [c_out][c_in*khw] GEMM view:
        a MODE_CHANNEL layer of c_in*khw channels with khw = 1 (its groups are that view's columns).  Element
        offsets, group order and k do not change."""
        cols = self.table()
        mode = cols["mode"]
        cs, al = mode == MODE_CHANNEL_SHAPE, mode == MODE_ALL
        shape = (mode == MODE_SHAPE) | cs | al
        # a layer that also limits its channels: the view's columns come in runs of khw per channel, of which
        # k_in runs may hold kept columns (columns "span" and "k_coarse" of the table)
        cols["span"] = np.where(cs | al, cols["khw"], 0).astype(np.int32)
        cols["k_coarse"] = np.where(cs | al, cols["k_in"], 0).astype(np.int32)
        cols["k"] = np.where(cs, cols["k_kern"], cols["k"]).astype(np.int32)
        cols["k_in"] = np.where(al, cols["k_kern"], cols["k_in"]).astype(np.int32)
        cols["c_in"] = np.where(shape, cols["c_in"] * cols["khw"], cols["c_in"]).astype(np.int32)
        cols["khw"] = np.where(shape, 1, cols["khw"]).astype(np.int32)
        cols["mode"] = np.where(al, MODE_BOTH, np.where(shape, MODE_CHANNEL, mode)).astype(np.int32)
        del cols["k_kern"]
        return cols

    def view_groups(self, per_group):
        """An array over the groups of table() as an array over the groups of gemm_view_table(): the channel
        entries of the layers of MODE_CHANNEL_SHAPE and MODE_ALL are dropped (the view has no groups for them)."""
        parts = []
        for l in self.layers:
            g = per_group[l.group_base:l.group_base + l.groups]
            if l.mode == MODE_CHANNEL_SHAPE:
                g = g[l.c_in:]
            elif l.mode == MODE_ALL:
                g = np.concatenate([g[:l.c_out], g[l.c_out + l.c_in:]])
            parts.append(g)
        return np.concatenate(parts)

    def algorithmic_bytes(self):
        """Bytes the method must move: each unique input read once, each output written once."""
        n, nk, R = self.n_total, self.n_kept, self.R
        project = 4 * n * (R + 3)
        compact = 8 * nk
        expand = 4 * nk + 4 * n
        return {"project": project, "compact": compact, "expand": expand,
                "step": project + compact + expand}


def keep_count(keep: float, groups: int) -> int:
    """Number of groups kept for a keep ratio: round half up, at least 1, at most all."""
    k = int(np.floor(float(keep) * groups + 0.5))
    return max(1, min(groups, k))


def finalize(layers: List[Layer], align_elems: int = 4):
    """Assign arena offsets (each layer starts on a multiple of align_elems) and group bases."""
    off = 0
    gb = 0
    for l in layers:
        off = (off + align_elems - 1) // align_elems * align_elems
        l.elem_off = off
        l.group_base = gb
        off += l.n
        gb += l.groups
    return off, gb


# ----------------------------------------------------------------------------- shapes

def _tiny_shapes():
    return [("conv1", 16, 3, 9), ("conv2", 32, 16, 9), ("conv3", 32, 32, 9),
            ("conv4", 64, 32, 9), ("fc", 10, 64, 1)]


def _resnet_basic_shapes(blocks=(2, 2, 2, 2), mult=1, n_classes=1000):
    s = [("conv1", 64 * mult, 3, 49)]
    inp = 64 * mult
    for si, nb in enumerate(blocks):
        w = 64 * mult * (2 ** si)
        for b in range(nb):
            pre = "layer%d.%d." % (si + 1, b)
            s.append((pre + "conv1", w, inp, 9))
            s.append((pre + "conv2", w, w, 9))
            if b == 0 and inp != w:
                s.append((pre + "downsample", w, inp, 1))
            inp = w
    s.append(("fc", n_classes, inp, 1))
    return s


def _resnet_bottleneck_shapes(blocks, mult=1, n_classes=1000, inner_mult=1):
    """inner_mult widens only the two inner convs of every bottleneck (the wide-ResNet construction: the block's
    output width stays 4 * w)."""
    s = [("conv1", 64 * mult, 3, 49)]
    inp = 64 * mult
    for si, nb in enumerate(blocks):
        w = 64 * mult * (2 ** si)
        wi = w * inner_mult
        for b in range(nb):
            pre = "layer%d.%d." % (si + 1, b)
            s.append((pre + "conv1", wi, inp, 1))
            s.append((pre + "conv2", wi, wi, 9))
            s.append((pre + "conv3", 4 * w, wi, 1))
            if b == 0:
                s.append((pre + "downsample", 4 * w, inp, 1))
            inp = 4 * w
    s.append(("fc", n_classes, inp, 1))
    return s


def _apply_policy(shapes, mode, keep, prune_fc, keep_in=None):
    """keep_in: MODE_BOTH only, keep ratio of the input channels (keep is then that of the filters)."""
    layers = []
    for (name, co, ci, khw) in shapes:
        l = Layer(name, co, ci, khw)
        if name == "fc" and not prune_fc:
            l.mode, l.k = MODE_NONE, co
        elif mode == MODE_BOTH:
            l.mode = mode
            l.k = keep_count(keep, co)
            l.k_in = keep_count(keep_in, ci)
        else:
            l.mode = mode
            l.k = keep_count(keep, l.groups)
        layers.append(l)
    return layers


def _philox(seed: int, layer: int, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), (int(layer) << 16) | int(tensor)]))


WORKLOAD_NAMES = ("tiny", "resnet18", "resnet50", "resnet152", "wide", "resnet50_both", "wrn50_2", "resnet152_filter")


def make_workload(name: str, seed: int = 0, prune_fc: Optional[bool] = None) -> Workload:
    """Layer table and generation recipe of one named configuration (no data is drawn)."""
    if name == "tiny":
        layers = _apply_policy(_tiny_shapes(), MODE_FILTER, 0.5,
                               True if prune_fc is None else prune_fc)
        wl = Workload(name, layers, R=1, seed=seed,
                      description="Tiny CNN, 4 conv + linear, output-filter groups, keep 0.5, R=1")
    elif name == "resnet18":
        layers = _apply_policy(_resnet_basic_shapes(), MODE_FILTER, 0.4, bool(prune_fc))
        wl = Workload(name, layers, R=1, seed=seed,
                      description="ResNet-18 conv/fc weights, output-filter groups, keep 0.4, R=1")
    elif name == "resnet50":
        layers = _apply_policy(_resnet_bottleneck_shapes((3, 4, 6, 3)), MODE_FILTER, 0.4,
                               bool(prune_fc))
        wl = Workload(name, layers, R=4, seed=seed, sigma_replica=float(np.sqrt(1e-3)),
                      description="ResNet-50 conv/fc weights, output-filter groups, keep 0.4, R=4")
    elif name == "resnet152":
        layers = _apply_policy(_resnet_bottleneck_shapes((3, 8, 36, 3)), MODE_CHANNEL, 0.3,
                               bool(prune_fc))
        wl = Workload(name, layers, R=4, seed=seed, sigma_replica=float(np.sqrt(1e-3)),
                      description="ResNet-152 conv/fc weights, input-channel groups, keep 0.3, R=4")
    elif name == "wide":
        shapes = _resnet_bottleneck_shapes((3, 4, 6, 3), mult=4)
        layers = _apply_policy(shapes, MODE_FILTER, 0.5, bool(prune_fc))
        keeps = _philox(seed, 0xFFFF, _TENSOR_KEEP).uniform(0.2, 0.8, size=len(layers))
        for l, kr in zip(layers, keeps):
            if l.mode != MODE_NONE:
                l.k = keep_count(kr, l.groups)
        wl = Workload(name, layers, R=8, seed=seed, sigma_replica=float(np.sqrt(1e-3)),
                      filter_scale_log10=(-3.0, 1.0),
                      description="ResNet-50 shapes with every width x4, output-filter groups, "
                                  "keep ~ U(0.2,0.8) per layer, per-filter scales 1e-3..1e1, R=8")
    elif name == "wrn50_2":
        shapes = _resnet_bottleneck_shapes((3, 4, 6, 3), inner_mult=2)
        layers = _apply_policy(shapes, MODE_FILTER, 0.4, bool(prune_fc))
        wl = Workload(name, layers, R=4, seed=seed, sigma_replica=float(np.sqrt(1e-3)),
                      description="WideResNet-50-2 conv/fc weights (inner bottleneck widths x2, ~69 M parameters), "
                                  "output-filter groups, keep 0.4, R=4")
    elif name == "resnet152_filter":
        layers = _apply_policy(_resnet_bottleneck_shapes((3, 8, 36, 3)), MODE_FILTER, 0.4, bool(prune_fc))
        wl = Workload(name, layers, R=4, seed=seed, sigma_replica=float(np.sqrt(1e-3)),
                      description="ResNet-152 conv/fc weights, output-filter groups, keep 0.4, R=4")
    elif name == "resnet50_both":
        layers = _apply_policy(_resnet_bottleneck_shapes((3, 4, 6, 3)), MODE_BOTH, 0.6, bool(prune_fc),
                               keep_in=0.6)
        wl = Workload(name, layers, R=4, seed=seed, sigma_replica=float(np.sqrt(1e-3)),
                      description="ResNet-50 conv/fc weights, filter and channel constraints together "
                                  "(keep 0.6 of the filters, then 0.6 of the channels), R=4")
    else:
        raise ValueError("unknown workload %r (have %s)" % (name, ", ".join(WORKLOAD_NAMES)))
    wl.n_arena, wl.groups_total = finalize(wl.layers)
    return wl


def custom_workload(shapes, R=1, seed=0, sigma_replica=0.0, name="custom") -> Workload:
    """shapes: list of (c_out, c_in, khw, mode, k) or, for MODE_BOTH, (c_out, c_in, khw, mode, k, k_in), or, for
    MODE_CHANNEL_SHAPE and MODE_ALL, (c_out, c_in, khw, mode, k, k_in, k_kern).
    For tests of odd shapes and edge cases."""
    layers = [Layer("l%d" % i, *sh) for i, sh in enumerate(shapes)]
    for l in layers:
        if l.mode == MODE_NONE:
            l.k = l.c_out
    wl = Workload(name, layers, R=R, seed=seed, sigma_replica=sigma_replica)
    wl.n_arena, wl.groups_total = finalize(wl.layers)
    return wl


# ----------------------------------------------------------------------------- values

def generate_layer(wl: Workload, li: int):
    """Draw the inputs of layer li: (replicas [R, n_l] float32, U [n_l] float32)."""
    l = wl.layers[li]
    n = l.n
    base = _philox(wl.seed, li, _TENSOR_W).standard_normal(n, dtype=np.float32)
    base *= np.float32(np.sqrt(2.0 / l.fan_in))
    if wl.filter_scale_log10 is not None:
        lo, hi = wl.filter_scale_log10
        ex = _philox(wl.seed, li, _TENSOR_SCALE).uniform(lo, hi, size=l.c_out)
        scale = np.power(10.0, ex).astype(np.float32)
        base = (base.reshape(l.c_out, -1) * scale[:, None]).reshape(-1)
    reps = np.empty((wl.R, n), dtype=np.float32)
    if wl.sigma_replica == 0.0:
        reps[:] = base[None, :]
    else:
        s = np.float32(wl.sigma_replica)
        for r in range(wl.R):
            noise = _philox(wl.seed, li, _TENSOR_REPLICA0 + r).standard_normal(n, dtype=np.float32)
            noise *= s
            np.add(base, noise, out=reps[r])
    U = _philox(wl.seed, li, _TENSOR_U).standard_normal(n, dtype=np.float32)
    U *= np.float32(wl.sigma_u)
    return reps, U


def generate(wl: Workload, threads: int = 1):
    """Full-layout arenas: (W [R, n_arena] float32, U [n_arena] float32). Padding is zero."""
    W = np.zeros((wl.R, wl.n_arena), dtype=np.float32)
    U = np.zeros(wl.n_arena, dtype=np.float32)

    def one(li):
        l = wl.layers[li]
        reps, u = generate_layer(wl, li)
        W[:, l.elem_off:l.elem_off + l.n] = reps
        U[l.elem_off:l.elem_off + l.n] = u

    if threads <= 1:
        for li in range(len(wl.layers)):
            one(li)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(one, range(len(wl.layers))))
    return W, U
