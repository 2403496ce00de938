"""Seeded synthetic workloads: layer graphs, fusion groups and tensors.

This module holds DATA only: which layers a workload has, how they are wired,
which fusion block (paper section 3.1: straight / split / merge) each belongs
to, and the seeded random tensors that feed them.  It contains none of the
method's arithmetic (no convolution, pooling, activation or tiling code), so
the CPU oracle and the HIP path can both be fed from it without sharing any
computation.

Graph vocabulary (paper section 3.1, Fig. 5: boxes = layers, arrows = data
flow, dotted box = fusion block with its mode letter):

  Layer.op      "conv" | "maxpool" | "gap" | "add" | "concat"
  Layer.inputs  tensor ids read (1 or 2)
  Layer.out     tensor id written
  Group.mode    "straight" | "split" | "merge" | "single"

Tensor shapes are NCHW, fp32, dense.  Filters are [Cout, Cin/groups, kh, kw]
(paper section 4.1 notation [O, I, KH, KW]/pad, stride, group).

Value recipes (one `numpy.random.default_rng(seed)` stream per workload, draws
in this fixed order: the input tensor, then per conv layer in graph order its
filter, then bias  -- or scale then shift when the layer has a folded BN):
  filter  ~ N(0, std = sqrt(2 / fan_in)), fan_in = (Cin/groups)*kh*kw
  bias    ~ N(0, std = 0.01)
  scale   ~ N(1, std = 0.1),  shift ~ N(0, std = 0.1)
All draws are made in float64 and rounded once to float32.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np


@dataclass
class Layer:
    op: str
    inputs: Tuple[int, ...]
    out: int
    cin: int = 0
    cout: int = 0
    k: int = 1
    stride: int = 1
    pad: int = 0
    groups: int = 1
    bias: bool = False          # epilogue adds a per-channel bias (held in "shift")
    bn: bool = False            # epilogue is a folded BN: y*scale + shift
    relu: bool = False
    name: str = ""


@dataclass
class Group:
    mode: str                   # straight | split | merge | single
    layers: Tuple[int, ...]     # indices into Workload.layers, topological order


@dataclass
class Workload:
    name: str
    shapes: List[Tuple[int, int, int, int]]      # NCHW per tensor id
    layers: List[Layer]
    groups: List[Group]
    input_id: int
    output_id: int
    input_dist: str                              # "uniform01" | "normal" | "relu_normal"
    seed: int
    notes: str = ""

    @property
    def batch(self) -> int:
        return self.shapes[self.input_id][0]


def _out_hw(h: int, w: int, k: int, s: int, p: int) -> Tuple[int, int]:
    return (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1


class _Builder:
    """Tiny helper that assigns tensor ids and infers output shapes."""

    def __init__(self, name: str, n: int, c: int, h: int, w: int):
        self.name = name
        self.shapes: List[Tuple[int, int, int, int]] = [(n, c, h, w)]
        self.layers: List[Layer] = []
        self.groups: List[Group] = []

    def _new(self, shape) -> int:
        self.shapes.append(tuple(int(v) for v in shape))
        return len(self.shapes) - 1

    def conv(self, x: int, cout: int, k: int, stride: int = 1, pad: int = 0, groups: int = 1,
             bias: bool = False, bn: bool = False, relu: bool = False, name: str = "") -> int:
        n, c, h, w = self.shapes[x]
        ho, wo = _out_hw(h, w, k, stride, pad)
        y = self._new((n, cout, ho, wo))
        self.layers.append(Layer("conv", (x,), y, cin=c, cout=cout, k=k, stride=stride, pad=pad,
                                 groups=groups, bias=bias, bn=bn, relu=relu, name=name))
        return y

    def maxpool(self, x: int, k: int, stride: int, pad: int = 0, name: str = "") -> int:
        n, c, h, w = self.shapes[x]
        ho, wo = _out_hw(h, w, k, stride, pad)
        y = self._new((n, c, ho, wo))
        self.layers.append(Layer("maxpool", (x,), y, cin=c, cout=c, k=k, stride=stride, pad=pad, name=name))
        return y

    def gap(self, x: int, name: str = "") -> int:
        n, c, h, w = self.shapes[x]
        y = self._new((n, c, 1, 1))
        self.layers.append(Layer("gap", (x,), y, cin=c, cout=c, name=name))
        return y

    def add(self, a: int, b: int, relu: bool = False, name: str = "") -> int:
        assert self.shapes[a] == self.shapes[b]
        y = self._new(self.shapes[a])
        c = self.shapes[a][1]
        self.layers.append(Layer("add", (a, b), y, cin=c, cout=c, relu=relu, name=name))
        return y

    def concat(self, a: int, b: int, name: str = "") -> int:
        na, ca, ha, wa = self.shapes[a]
        nb, cb, hb, wb = self.shapes[b]
        assert (na, ha, wa) == (nb, hb, wb)
        y = self._new((na, ca + cb, ha, wa))
        self.layers.append(Layer("concat", (a, b), y, cin=ca + cb, cout=ca + cb, name=name))
        return y

    def group(self, mode: str, first_layer: int) -> None:
        """Close a fusion block made of layers[first_layer:]."""
        self.groups.append(Group(mode, tuple(range(first_layer, len(self.layers)))))

    def fire(self, x: int, s: int, e: int, name: str, pool=None) -> int:
        """SqueezeNet fire module = one split-mode block (paper section 4.2: 8 mode-b blocks).
        pool = (k, stride, name): a max pooling of the module's output joins the block."""
        first = len(self.layers)
        sq = self.conv(x, s, 1, bias=True, relu=True, name=name + ".squeeze")
        e1 = self.conv(sq, e, 1, bias=True, relu=True, name=name + ".expand1x1")
        e3 = self.conv(sq, e, 3, pad=1, bias=True, relu=True, name=name + ".expand3x3")
        y = self.concat(e1, e3, name=name + ".concat")
        if pool is not None:
            y = self.maxpool(y, pool[0], pool[1], pool[3] if len(pool) > 3 else 0, name=pool[2])
        self.group("split", first)
        return y

    def done(self, out: int, input_dist: str, seed: int, notes: str = "") -> Workload:
        covered = {i for g in self.groups for i in g.layers}
        for i in range(len(self.layers)):
            if i not in covered:
                self.groups.append(Group("single", (i,)))
        self.groups.sort(key=lambda g: g.layers[0])
        return Workload(self.name, self.shapes, self.layers, self.groups, 0, out, input_dist, seed, notes)


def straight_tiny(n: int = 1, c: int = 16, hw: int = 16) -> Workload:
    """Config 1: conv3x3+bias+ReLU twice, 16 channels, 16x16, batch 1 (straight mode)."""
    b = _Builder("cfg1_straight_tiny", n, c, hw, hw)
    t = b.conv(0, c, 3, pad=1, bias=True, relu=True, name="conv1")
    t = b.conv(t, c, 3, pad=1, bias=True, relu=True, name="conv2")
    b.group("straight", 0)
    return b.done(t, "uniform01", 1001)


def straight_pool(n: int = 8, c: int = 64, hw: int = 56) -> Workload:
    """Config 2: conv1x1 + folded BN + ReLU, then maxpool 3x3 s2 p1 (straight mode)."""
    b = _Builder("cfg2_straight_pool", n, c, hw, hw)
    t = b.conv(0, c, 1, bn=True, relu=True, name="conv")
    t = b.maxpool(t, 3, 2, 1, name="pool")
    b.group("straight", 0)
    return b.done(t, "uniform01", 1002)


def split_fire(n: int = 16, cin: int = 96, hw: int = 55, s: int = 16, e: int = 64) -> Workload:
    """Config 3: SqueezeNet fire module (split mode; family of the paper's case b.1)."""
    b = _Builder("cfg3_split_fire", n, cin, hw, hw)
    t = b.fire(0, s, e, "fire")
    return b.done(t, "relu_normal", 1003)


def split_fire_pool(n: int = 2, cin: int = 32, hw: int = 27, s: int = 16, e: int = 32, pk: int = 3, ps: int = 2,
                    seed: int = 12, pp: int = 0) -> Workload:
    """A fire module whose concatenated output is max-pooled inside the block (straight after split)."""
    b = _Builder(f"firepool_{cin}x{hw}_{s}_{e}_p{pk}s{ps}", n, cin, hw, hw)
    t = b.fire(0, s, e, "fire", pool=(pk, ps, "pool", pp))
    return b.done(t, "relu_normal", seed)


def merge_residual(n: int = 32, c: int = 64, hw: int = 56) -> Workload:
    """Config 4: residual basic block, identity shortcut (merge mode)."""
    b = _Builder("cfg4_merge_residual", n, c, hw, hw)
    t = b.conv(0, c, 3, pad=1, bn=True, relu=True, name="conv1")
    t = b.conv(t, c, 3, pad=1, bn=True, relu=False, name="conv2")
    t = b.add(t, 0, relu=True, name="add")
    b.group("merge", 0)
    return b.done(t, "relu_normal", 1004)


def merge_residual_projection(n: int = 2, cin: int = 32, c: int = 64, hw: int = 28, shortcut_first: bool = True) -> Workload:
    """Residual block whose shortcut is a 1x1 projection of the block input (channel counts differ).
    The projection is a layer outside the merge block; listed before the block (shortcut_first) the
    block can read it, listed between the block's layers it is produced too late for a fused block."""
    b = _Builder(f"merge_proj_{cin}_{c}x{hw}", n, cin, hw, hw)
    if shortcut_first:
        sc = b.conv(0, c, 1, bn=True, relu=False, name="projection")
        first = len(b.layers)
        t = b.conv(0, c, 3, pad=1, bn=True, relu=True, name="conv1")
        t = b.conv(t, c, 3, pad=1, bn=True, relu=False, name="conv2")
        t = b.add(t, sc, relu=True, name="add")
        b.group("merge", first)
    else:
        t = b.conv(0, c, 3, pad=1, bn=True, relu=True, name="conv1")
        t = b.conv(t, c, 3, pad=1, bn=True, relu=False, name="conv2")
        sc = b.conv(0, c, 1, bn=True, relu=False, name="projection")
        t = b.add(t, sc, relu=True, name="add")
        b.groups.append(Group("merge", (0, 1, 3)))
    return b.done(t, "relu_normal", 1014)


def squeezenet11(n: int = 64, hw: int = 224, classes: int = 1000, fuse_stem: bool = True,
                 fuse_head: bool = True, fuse_pools: bool = True) -> Workload:
    """Config 5: SqueezeNet-v1.1-shaped network; 8 split-mode fire blocks (paper section 4.2).
    fuse_pools: the two max poolings between fire modules join the fire block before them."""
    b = _Builder("cfg5_squeezenet11", n, 3, hw, hw)
    first = len(b.layers)
    t = b.conv(0, 64, 3, stride=2, pad=0, bias=True, relu=True, name="conv1")
    t = b.maxpool(t, 3, 2, 0, name="pool1")
    if fuse_stem:
        b.group("straight", first)
    t = b.fire(t, 16, 64, "fire2")
    if fuse_pools:
        t = b.fire(t, 16, 64, "fire3", pool=(3, 2, "pool2"))
    else:
        t = b.fire(t, 16, 64, "fire3")
        t = b.maxpool(t, 3, 2, 0, name="pool2")
    t = b.fire(t, 32, 128, "fire4")
    if fuse_pools:
        t = b.fire(t, 32, 128, "fire5", pool=(3, 2, "pool3"))
    else:
        t = b.fire(t, 32, 128, "fire5")
        t = b.maxpool(t, 3, 2, 0, name="pool3")
    t = b.fire(t, 48, 192, "fire6")
    t = b.fire(t, 48, 192, "fire7")
    t = b.fire(t, 64, 256, "fire8")
    t = b.fire(t, 64, 256, "fire9")
    first = len(b.layers)
    t = b.conv(t, classes, 1, bias=True, relu=True, name="conv10")
    t = b.gap(t, name="gap")
    if fuse_head:
        b.group("straight", first)
    return b.done(t, "normal", 1005)


CONFIGS = {
    1: straight_tiny,
    2: straight_pool,
    3: split_fire,
    4: merge_residual,
    5: squeezenet11,
}


def config(i: int, **kw) -> Workload:
    return CONFIGS[i](**kw)


# ---------------------------------------------------------------------------
# Extra shapes used by tests (paper Table 1 and small ragged cases).
# ---------------------------------------------------------------------------

def straight_generic(n, cin, h, w, c1, k1, p1, s1, c2, k2, p2, s2, bn1=False, bn2=False,
                     relu1=True, relu2=True, seed=7, dist="normal") -> Workload:
    b = _Builder(f"straight_{cin}x{h}x{w}_{c1}k{k1}_{c2}k{k2}", n, cin, h, w)
    t = b.conv(0, c1, k1, stride=s1, pad=p1, bias=not bn1, bn=bn1, relu=relu1, name="conv1")
    t = b.conv(t, c2, k2, stride=s2, pad=p2, bias=not bn2, bn=bn2, relu=relu2, name="conv2")
    b.group("straight", 0)
    return b.done(t, dist, seed)


def conv_pool_generic(n, cin, h, w, c1, k1, p1, s1, pk, ps, pp, bn=False, relu=True, seed=8,
                      dist="normal") -> Workload:
    b = _Builder(f"convpool_{cin}x{h}x{w}_{c1}k{k1}_p{pk}", n, cin, h, w)
    t = b.conv(0, c1, k1, stride=s1, pad=p1, bias=not bn, bn=bn, relu=relu, name="conv")
    t = b.maxpool(t, pk, ps, pp, name="pool")
    b.group("straight", 0)
    return b.done(t, dist, seed)


def depthwise_pointwise(n, c, h, w, c2, k1=3, p1=1, s1=1, k2=1, p2=0, bn1=False, bn2=False, relu1=True, relu2=True,
                        seed=10, dist="normal") -> Workload:
    """Depthwise k1 x k1 convolution (one filter per channel) -> convolution, one straight block
    (paper Table 1, case a.2: [16,80,80], 3x3 depthwise pad 1, then 1x1 16 -> 16)."""
    b = _Builder(f"dwpw_{c}x{h}x{w}_k{k1}s{s1}_{c2}k{k2}", n, c, h, w)
    t = b.conv(0, c, k1, stride=s1, pad=p1, groups=c, bias=not bn1, bn=bn1, relu=relu1, name="depthwise")
    t = b.conv(t, c2, k2, stride=1, pad=p2, bias=not bn2, bn=bn2, relu=relu2, name="pointwise")
    b.group("straight", 0)
    return b.done(t, dist, seed)


def merge_two_producers(n=1, c=64, h=56, w=56, cmid=256, cout=64, bn=True, relu_a=False, relu_b=False,
                        relu_sum=True, seed=11, dist="relu_normal") -> Workload:
    """Merge mode with two producer layers (paper Fig. 4c; Table 1, case c.1: two 1x1 convolutions
    64 -> 256 of the same input, added, feeding a 1x1 convolution 256 -> 64)."""
    b = _Builder(f"merge2_{c}x{h}x{w}_{cmid}_{cout}", n, c, h, w)
    a = b.conv(0, cmid, 1, bias=not bn, bn=bn, relu=relu_a, name="producer_a")
    bb = b.conv(0, cmid, 1, bias=not bn, bn=bn, relu=relu_b, name="producer_b")
    t = b.add(a, bb, relu=relu_sum, name="add")
    t = b.conv(t, cout, 1, bias=not bn, bn=bn, relu=True, name="consumer")
    b.group("merge", 0)
    return b.done(t, dist, seed)


def conv_gap_generic(n, cin, h, w, c1, k1, p1, s1, bn=False, relu=True, seed=9, dist="relu_normal") -> Workload:
    """Convolution -> global average pooling as one straight block (the head of config 5)."""
    b = _Builder(f"convgap_{cin}x{h}x{w}_{c1}k{k1}", n, cin, h, w)
    t = b.conv(0, c1, k1, stride=s1, pad=p1, bias=not bn, bn=bn, relu=relu, name="conv")
    t = b.gap(t, name="gap")
    b.group("straight", 0)
    return b.done(t, dist, seed)


def single_conv(n, cin, h, w, cout, k, stride=1, pad=0, bias=True, bn=False, relu=True, seed=9,
                dist="normal") -> Workload:
    b = _Builder(f"conv_{cin}x{h}x{w}_{cout}k{k}s{stride}p{pad}", n, cin, h, w)
    t = b.conv(0, cout, k, stride=stride, pad=pad, bias=bias, bn=bn, relu=relu, name="conv")
    return b.done(t, dist, seed)


# ---------------------------------------------------------------------------
# Seeded tensors
# ---------------------------------------------------------------------------

def make_tensors(wl: Workload, seed: Optional[int] = None):
    """Return (input, params): input is the NCHW float32 array; params maps a
    layer index to {"w": filter, "scale": array|None, "shift": array|None}."""
    rng = np.random.default_rng(wl.seed if seed is None else seed)
    shape = wl.shapes[wl.input_id]
    if wl.input_dist == "uniform01":
        x = rng.random(shape)
    elif wl.input_dist == "normal":
        x = rng.standard_normal(shape)
    elif wl.input_dist == "relu_normal":
        x = np.maximum(rng.standard_normal(shape), 0.0)
    else:
        raise ValueError(wl.input_dist)
    x = np.ascontiguousarray(x, dtype=np.float32)
    params: Dict[int, dict] = {}
    for li, L in enumerate(wl.layers):
        if L.op != "conv":
            continue
        cin_g = L.cin // L.groups
        fan_in = cin_g * L.k * L.k
        w = rng.standard_normal((L.cout, cin_g, L.k, L.k)) * np.sqrt(2.0 / fan_in)
        scale = shift = None
        if L.bn:
            scale = 1.0 + 0.1 * rng.standard_normal(L.cout)
            shift = 0.1 * rng.standard_normal(L.cout)
        elif L.bias:
            shift = 0.01 * rng.standard_normal(L.cout)
        params[li] = {
            "w": np.ascontiguousarray(w, dtype=np.float32),
            "scale": None if scale is None else np.ascontiguousarray(scale, dtype=np.float32),
            "shift": None if shift is None else np.ascontiguousarray(shift, dtype=np.float32),
        }
    return x, params


def count_params(wl: Workload) -> int:
    """Learnable parameters (filters + bias, or filters + scale + shift)."""
    total = 0
    for L in wl.layers:
        if L.op == "conv":
            total += L.cout * (L.cin // L.groups) * L.k * L.k
            if L.bn:
                total += 2 * L.cout
            elif L.bias:
                total += L.cout
    return total


def count_flops(wl: Workload) -> int:
    """2*MAC over all convolutions, whole batch, no halo recompute."""
    total = 0
    for L in wl.layers:
        if L.op == "conv":
            n, c, h, w = wl.shapes[L.out]
            total += 2 * n * c * h * w * (L.cin // L.groups) * L.k * L.k
    return total


def subgraph(wl: Workload, group_index: int) -> Workload:
    """The layers of one fusion block as a workload of their own (same shapes,
    tensor ids renumbered).  Its input stands for the activations that reach the
    block inside the network: post-ReLU, so non-negative N(0,1) draws, unless the
    block starts at the network input."""
    g = wl.groups[group_index]
    ids = list(g.layers)
    produced = {wl.layers[i].out for i in ids}
    ext_in = []
    for i in ids:
        for t in wl.layers[i].inputs:
            if t not in produced and t not in ext_in:
                ext_in.append(t)
    assert len(ext_in) == 1, "a block has one external input"
    consumed = {t for i in ids for t in wl.layers[i].inputs}
    outs = [wl.layers[i].out for i in ids if wl.layers[i].out not in consumed]
    assert len(outs) == 1, "a block has one external output"
    remap = {ext_in[0]: 0}
    shapes = [wl.shapes[ext_in[0]]]
    layers = []
    for i in ids:
        L = wl.layers[i]
        remap[L.out] = len(shapes)
        shapes.append(wl.shapes[L.out])
        layers.append(Layer(L.op, tuple(remap[t] for t in L.inputs), remap[L.out], cin=L.cin, cout=L.cout, k=L.k,
                            stride=L.stride, pad=L.pad, groups=L.groups, bias=L.bias, bn=L.bn, relu=L.relu,
                            name=L.name))
    dist = wl.input_dist if ext_in[0] == wl.input_id else "relu_normal"
    name = f"{wl.name}.block{group_index}.{wl.layers[ids[0]].name}"
    return Workload(name, shapes, layers, [Group(g.mode, tuple(range(len(ids))))], 0, remap[outs[0]], dist,
                    wl.seed + 100 + group_index)
