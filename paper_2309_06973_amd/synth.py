"""Seeded synthetic networks: shapes, channel groups and weights.

This module only *describes and fills* inputs.  It holds none of the pruning
method's arithmetic (no ranking, masking, scanning, planning or gathering); both
the GPU library's tests and the CPU oracle take their inputs from here.

A network is a flat fp32 *weight arena* holding every conv / linear weight tensor
(OIHW, row-major, in descriptor order), a flat fp32 *vector arena* holding every
per-channel vector (BatchNorm gamma, beta, running mean, running variance, and the
classifier bias), and three descriptor tables:

* ``TensorDesc``  - where a weight tensor sits, its shape, and the channel groups
  of its output filters and of its input channels;
* ``VecDesc``     - where a per-channel vector sits and the group it belongs to;
* ``GroupDesc``   - a channel space shared by producers (tensors whose filters
  write it), vectors, and consumers (tensors whose input channels read it).  The
  network input and the logits are *pinned* groups: never shrunk.

The five shapes follow the workloads of the paper's evaluation (Table II: VGG-16 on
CIFAR-10, ResNet-50 on an ImageNet-style input) plus a tiny net, a ResNet-56 and a
4x-wide VGG-19 used for stress.  Trained checkpoints are not available, so weights
are drawn as Kaiming-normal values times a heavy-tailed per-filter scale, which
makes whole filters fall under a global magnitude threshold the way trained sparse
models do (Sec. III-A.1 of the paper motivates exactly this structure).

``ops`` is a small op list describing how the tensors are wired (strides, pooling,
residual adds); only the forward-equivalence test executes it.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

SEED_BASE = 2309069730


@dataclass
class TensorDesc:
    offset: int          # fp32 element offset into the weight arena
    out_ch: int          # O
    in_ch: int           # I  (input *features*: group width * in_mult)
    kh: int
    kw: int
    in_mult: int         # input features per input channel (flatten -> linear), else 1
    out_group: int
    in_group: int
    prunable: int        # 1: takes part in the global magnitude ranking

    @property
    def numel(self) -> int:
        return self.out_ch * self.in_ch * self.kh * self.kw


@dataclass
class VecDesc:
    offset: int          # fp32 element offset into the vector arena
    length: int
    group: int


@dataclass
class GroupDesc:
    width: int
    pinned: int


@dataclass
class NetSpec:
    name: str
    tensors: List[TensorDesc] = field(default_factory=list)
    vecs: List[VecDesc] = field(default_factory=list)
    groups: List[GroupDesc] = field(default_factory=list)
    ops: List[tuple] = field(default_factory=list)
    input_hw: int = 32
    lognormal_sigma: float = 1.5
    kill_prob: float = 0.0
    w_elems: int = 0
    v_elems: int = 0

    @property
    def n_prunable(self) -> int:
        return sum(t.numel for t in self.tensors if t.prunable)

    @property
    def n_param_total(self) -> int:
        """Trainable parameters: weights + BN gamma/beta + bias (not running stats)."""
        n = sum(t.numel for t in self.tensors)
        for op in self.ops:
            if op[0] == "bn":
                n += 2 * self.vecs[op[1][0]].length
            elif op[0] == "linear" and op[2] is not None:
                n += self.vecs[op[2]].length
        return n


class _Builder:
    def __init__(self, name: str, in_ch: int, n_cls: int, input_hw: int,
                 sigma: float, kill_prob: float):
        self.s = NetSpec(name=name, input_hw=input_hw, lognormal_sigma=sigma,
                         kill_prob=kill_prob)
        self.g_in = self.group(in_ch, pinned=1)
        self.n_cls = n_cls

    def group(self, width: int, pinned: int = 0) -> int:
        self.s.groups.append(GroupDesc(width, pinned))
        return len(self.s.groups) - 1

    def tensor(self, out_ch, in_ch, k, out_group, in_group, in_mult=1) -> int:
        t = TensorDesc(self.s.w_elems, out_ch, in_ch, k, k, in_mult, out_group,
                       in_group, 1)
        self.s.tensors.append(t)
        self.s.w_elems += t.numel
        return len(self.s.tensors) - 1

    def vec(self, length, group) -> int:
        self.s.vecs.append(VecDesc(self.s.v_elems, length, group))
        self.s.v_elems += length
        return len(self.s.vecs) - 1

    # ops work on named activation slots
    def conv_bn(self, src: str, dst: str, in_group: int, out_group: int, k: int,
                stride: int = 1, relu: bool = True) -> None:
        gi, go = self.s.groups[in_group], self.s.groups[out_group]
        t = self.tensor(go.width, gi.width, k, out_group, in_group)
        self.s.ops.append(("conv", t, stride, k // 2, src, dst))
        v = [self.vec(go.width, out_group) for _ in range(4)]
        self.s.ops.append(("bn", v, dst))
        if relu:
            self.s.ops.append(("relu", dst))

    def classifier(self, src: str, in_group: int) -> None:
        g_out = self.group(self.n_cls, pinned=1)
        gi = self.s.groups[in_group]
        t = self.tensor(self.n_cls, gi.width, 1, g_out, in_group)
        b = self.vec(self.n_cls, g_out)
        self.s.ops.append(("gap", src))
        self.s.ops.append(("linear", t, b, src, "logits"))


def tiny_cnn() -> NetSpec:
    b = _Builder("tiny_cnn", 3, 10, 32, 1.5, 0.25)
    g_prev, src = b.g_in, "x"
    for i, w in enumerate((16, 32, 64)):
        g = b.group(w)
        b.conv_bn(src, f"a{i}", g_prev, g, 3)
        g_prev, src = g, f"a{i}"
    b.classifier(src, g_prev)
    return b.s


def _vgg(name, widths_with_pool, n_cls, sigma, kill_prob, input_hw=32) -> NetSpec:
    b = _Builder(name, 3, n_cls, input_hw, sigma, kill_prob)
    g_prev, src, i = b.g_in, "x", 0
    for w in widths_with_pool:
        if w == "M":
            b.s.ops.append(("maxpool", 2, 2, 0, src))
            continue
        g = b.group(w)
        b.conv_bn(src, f"a{i}", g_prev, g, 3)
        g_prev, src, i = g, f"a{i}", i + 1
    b.classifier(src, g_prev)
    return b.s


def vgg16_cifar() -> NetSpec:
    cfg = [64, 64, "M", 128, 128, "M", 256, 256, 256, "M", 512, 512, 512, "M",
           512, 512, 512, "M"]
    return _vgg("vgg16_cifar", cfg, 10, 1.5, 0.0)


def wide_vgg19(width_mult: int = 4, n_cls: int = 1000) -> NetSpec:
    base = [64, 64, "M", 128, 128, "M", 256, 256, 256, 256, "M", 512, 512, 512, 512,
            "M", 512, 512, 512, 512, "M"]
    cfg = [c if c == "M" else c * width_mult for c in base]
    return _vgg(f"wide_vgg19_x{width_mult}", cfg, n_cls, 2.0, 0.30)


def resnet56_cifar() -> NetSpec:
    b = _Builder("resnet56_cifar", 3, 10, 32, 1.5, 0.0)
    stream = b.group(16)
    b.conv_bn("x", "s", b.g_in, stream, 3)
    for stage, width in enumerate((16, 32, 64)):
        for blk in range(9):
            stride = 2 if (stage > 0 and blk == 0) else 1
            if stride == 2:
                new_stream = b.group(width)
                b.conv_bn("s", "sc", stream, new_stream, 1, stride=2, relu=False)
            else:
                new_stream = stream
            mid = b.group(width)
            b.conv_bn("s", "h", stream, mid, 3, stride=stride)
            b.conv_bn("h", "h", mid, new_stream, 3, relu=False)
            b.s.ops.append(("add", "h", "sc" if stride == 2 else "s", "s"))
            b.s.ops.append(("relu", "s"))
            stream = new_stream
    b.classifier("s", stream)
    return b.s


def resnet50_imagenet(input_hw: int = 224) -> NetSpec:
    b = _Builder("resnet50_imagenet", 3, 1000, input_hw, 2.0, 0.0)
    stem = b.group(64)
    b.conv_bn("x", "s", b.g_in, stem, 7, stride=2)
    b.s.ops.append(("maxpool", 3, 2, 1, "s"))
    stream = stem
    for stage, (width, n_blk) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for blk in range(n_blk):
            stride = 2 if (stage > 0 and blk == 0) else 1
            if blk == 0:
                new_stream = b.group(width * 4)
                b.conv_bn("s", "sc", stream, new_stream, 1, stride=stride, relu=False)
            else:
                new_stream = stream
            m1, m2 = b.group(width), b.group(width)
            b.conv_bn("s", "h", stream, m1, 1)
            b.conv_bn("h", "h", m1, m2, 3, stride=stride)
            b.conv_bn("h", "h", m2, new_stream, 1, relu=False)
            b.s.ops.append(("add", "h", "sc" if blk == 0 else "s", "s"))
            b.s.ops.append(("relu", "s"))
            stream = new_stream
    b.classifier("s", stream)
    return b.s


CONFIGS = {
    1: ("C1 tiny CNN", tiny_cnn),
    2: ("C2 VGG-16-shaped (CIFAR)", vgg16_cifar),
    3: ("C3 ResNet-56-shaped (CIFAR)", resnet56_cifar),
    4: ("C4 ResNet-50-shaped (ImageNet)", resnet50_imagenet),
    5: ("C5 wide VGG-19 x4", wide_vgg19),
}


def build_config(c: int) -> NetSpec:
    return CONFIGS[c][1]()


def config_sparsities(c: int) -> List[float]:
    """Cumulative sparsity schedule of each workload: s_k = 1 - 0.8**k."""
    if c == 1:
        return [0.9]
    k = {2: 10, 3: 15, 4: 20, 5: 10}[c]
    return [1.0 - 0.8 ** j for j in range(1, k + 1)]


def prune_count(n: int, s: float) -> int:
    """Integer number of weights to remove at sparsity ``s``: n - round((1-s) n).

    Round-half-up in IEEE double, done once here so that the same integer is handed
    to every implementation (a sparse model of compression ratio C keeps 1 of every C
    weights, Sec. IV-B.1 of the paper: s = 1 - 1/C)."""
    keep = int(math.floor((1.0 - s) * float(n) + 0.5))
    keep = min(max(keep, 0), n)
    return n - keep


def generate_weights(spec: NetSpec, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Fill the weight and vector arenas of ``spec`` from a counter-based generator.

    w[o,i,y,x] = z * sqrt(2/fan_in) * scale_o * kill_o with z ~ N(0,1),
    scale_o ~ LogNormal(0, sigma) per output filter and kill_o = 1e-4 with
    probability ``kill_prob`` (else 1).  BatchNorm: gamma ~ U(0.5,1.5),
    beta ~ N(0,0.1); the running mean and variance follow the filter's scale
    (mean ~ N(0,0.1) * f, var ~ U(0.5,1.5) * f^2 with f = scale_o * kill_o) as a
    trained BatchNorm's statistics would, which keeps activations O(1) through
    the depth of the net.  Classifier bias ~ N(0, 0.01).
    """
    rng = np.random.Generator(np.random.Philox(seed))
    w = np.empty(spec.w_elems, dtype=np.float32)
    v = np.zeros(spec.v_elems, dtype=np.float32)
    filt_scale = {}
    for ti, t in enumerate(spec.tensors):
        fan_in = t.in_ch * t.kh * t.kw
        scale = np.exp(rng.normal(0.0, spec.lognormal_sigma, size=t.out_ch))
        if spec.kill_prob > 0.0:
            kill = np.where(rng.random(t.out_ch) < spec.kill_prob, 1e-4, 1.0)
        else:
            kill = np.ones(t.out_ch)
        f = scale * kill
        filt_scale[ti] = f
        per_filter = (math.sqrt(2.0 / fan_in) * f).astype(np.float32)
        z = rng.standard_normal(t.numel, dtype=np.float32).reshape(t.out_ch, -1)
        z *= per_filter[:, None]
        w[t.offset:t.offset + t.numel] = z.reshape(-1)
    last_conv = None
    for op in spec.ops:
        if op[0] == "conv":
            last_conv = op[1]
        elif op[0] == "bn":
            g, b_, m, var = (spec.vecs[i] for i in op[1])
            f = filt_scale[last_conv]
            n = g.length
            v[g.offset:g.offset + n] = rng.uniform(0.5, 1.5, n)
            v[b_.offset:b_.offset + n] = rng.normal(0.0, 0.1, n)
            v[m.offset:m.offset + n] = rng.normal(0.0, 0.1, n) * f
            v[var.offset:var.offset + n] = rng.uniform(0.5, 1.5, n) * f * f
        elif op[0] == "linear" and op[2] is not None:
            b_ = spec.vecs[op[2]]
            v[b_.offset:b_.offset + b_.length] = rng.normal(0.0, 0.01, b_.length)
    return w, v


def generate_config(c: int) -> Tuple[NetSpec, np.ndarray, np.ndarray]:
    spec = build_config(c)
    w, v = generate_weights(spec, SEED_BASE + c)
    return spec, w, v


# ---------------------------------------------------------------------------
# Hand-sized adversarial arenas for tie / edge-case parity (not timed).
# ---------------------------------------------------------------------------

def chain_spec(widths: List[int], k: int = 3, in_ch: int = 3, n_cls: int = 4,
               name: str = "chain") -> NetSpec:
    """A plain conv chain (the setting of the paper's Algorithms 1 and 2)."""
    b = _Builder(name, in_ch, n_cls, 8, 1.0, 0.0)
    g_prev, src = b.g_in, "x"
    for i, wd in enumerate(widths):
        g = b.group(wd)
        b.conv_bn(src, f"a{i}", g_prev, g, k)
        g_prev, src = g, f"a{i}"
    b.classifier(src, g_prev)
    return b.s


def residual_toy_spec(width: int = 6, mid: int = 5, n_blocks: int = 2) -> NetSpec:
    """Stem + ``n_blocks`` basic residual blocks on one stream + classifier."""
    b = _Builder("residual_toy", 3, 4, 8, 1.0, 0.0)
    stream = b.group(width)
    b.conv_bn("x", "s", b.g_in, stream, 3)
    for _ in range(n_blocks):
        m = b.group(mid)
        b.conv_bn("s", "h", stream, m, 3)
        b.conv_bn("h", "h", m, stream, 3, relu=False)
        b.s.ops.append(("add", "h", "s", "s"))
        b.s.ops.append(("relu", "s"))
    b.classifier("s", stream)
    return b.s


@dataclass
class FoldDesc:
    """One layer of the conv + BatchNorm fold (Sec. III-D, Module 1): which vectors of the
    unfused network normalise the filters of ``tensor`` and where the layer's bias goes in
    the vector arena of the fused network.  -1 marks a vector the layer does not have; a
    layer with a bias and no BatchNorm (the classifier) passes its bias through."""
    tensor: int
    gamma: int
    beta: int
    mean: int
    var: int
    bias: int
    out_offset: int


def fused_spec(spec: NetSpec) -> Tuple[NetSpec, List[FoldDesc]]:
    """The network of ``spec`` after Module 1: same tensors and groups (same weight-arena
    layout), every conv + BatchNorm pair replaced by a conv with a bias, so the vector
    arena holds one bias per layer and nothing else.  Structure only: the arithmetic of
    the fold is the library's (and, separately, the oracle's)."""
    f = NetSpec(name=spec.name + "_fused", input_hw=spec.input_hw,
                lognormal_sigma=spec.lognormal_sigma, kill_prob=spec.kill_prob)
    f.tensors = [TensorDesc(**vars(t)) for t in spec.tensors]
    f.groups = [GroupDesc(g.width, g.pinned) for g in spec.groups]
    f.w_elems = spec.w_elems
    folds: List[FoldDesc] = []

    def bias_vec(t: int) -> int:
        td = spec.tensors[t]
        f.vecs.append(VecDesc(f.v_elems, td.out_ch, td.out_group))
        f.v_elems += td.out_ch
        return len(f.vecs) - 1

    last_conv = None
    for op in spec.ops:
        if op[0] == "conv":
            last_conv = op[1]
            f.ops.append(op)
        elif op[0] == "bn":
            g, b_, m, var = op[1]
            bv = bias_vec(last_conv)
            folds.append(FoldDesc(last_conv, g, b_, m, var, -1, f.vecs[bv].offset))
            f.ops.append(("bias", bv, op[2]))
        elif op[0] == "linear" and op[2] is not None:
            bv = bias_vec(op[1])
            folds.append(FoldDesc(op[1], -1, -1, -1, -1, op[2], f.vecs[bv].offset))
            f.ops.append(("linear", op[1], bv, op[3], op[4]))
        else:
            f.ops.append(op)
    return f, folds


def adversarial_arena(kind: str, n: int, seed: int = 0) -> np.ndarray:
    """Value patterns that exercise tie-breaking and special floats."""
    rng = np.random.Generator(np.random.Philox(SEED_BASE + 77 + seed))
    if kind == "ramp":
        return np.arange(1, n + 1, dtype=np.float32)
    if kind == "ramp_desc_signed":
        a = np.arange(n, 0, -1, dtype=np.float32)
        a[::2] *= -1
        return a
    if kind == "all_equal":
        return np.full(n, 0.5, dtype=np.float32)
    if kind == "all_zero":
        return np.zeros(n, dtype=np.float32)
    if kind == "half_zero":
        a = rng.standard_normal(n, dtype=np.float32)
        a[rng.random(n) < 0.5] = 0.0
        return a
    if kind == "quantised":
        a = np.round(rng.standard_normal(n, dtype=np.float32) * 40.0) / 40.0
        return np.clip(a, -3.15, 3.15).astype(np.float32)
    if kind == "denormal":
        bits = rng.integers(0, 1 << 23, size=n, dtype=np.uint32)
        bits |= (rng.integers(0, 2, size=n, dtype=np.uint32) << 31)
        return bits.view(np.float32)
    if kind == "inf_negzero":
        a = rng.standard_normal(n, dtype=np.float32)
        a[::7] = np.float32("inf")
        a[3::11] = -np.float32("inf")
        a[1::5] = np.float32(-0.0)
        a[2::13] = 0.0
        return a
    if kind == "gauss":
        return rng.standard_normal(n, dtype=np.float32)
    raise ValueError(kind)


ADVERSARIAL_KINDS = ("ramp", "ramp_desc_signed", "all_equal", "all_zero", "half_zero",
                     "quantised", "denormal", "inf_negzero", "gauss")


# ---------------------------------------------------------------------------
# Random networks: arbitrary group graphs for parity tests (not timed).
# ---------------------------------------------------------------------------

def random_spec(seed: int, max_weights: int = 250_000) -> NetSpec:
    """A random valid network description: tensors reading and writing a random graph of
    channel groups (several producers per group as residual adds make them, several
    consumers, groups nobody reads), kernel shapes from 1x1 to long thin ones, flatten
    multipliers, non-prunable tensors, gaps and odd offsets in both arenas, vectors on any
    group.  No forward semantics (``ops`` stays empty)."""
    rng = np.random.Generator(np.random.Philox(SEED_BASE + 1000 + seed))
    s = NetSpec(name=f"random{seed}")
    pick = lambda *xs: xs[int(rng.integers(0, len(xs)))]
    s.groups.append(GroupDesc(int(rng.integers(1, 6)), 1))            # the network input
    readable, writable = [0], []
    n_layers = int(rng.integers(2, 9))
    budget = max_weights
    for layer in range(n_layers):
        in_group = pick(*readable)
        in_mult = pick(1, 1, 1, 1, 2, 4) if s.groups[in_group].width <= 64 else 1
        shape = pick((1, 1), (1, 1), (3, 3), (3, 3), (3, 3), (2, 2), (5, 5), (1, 3), (3, 1), (7, 1))
        if rng.random() < 0.04:
            shape = pick((40, 30), (95, 90), (17, 70))    # kernels beyond the small-divisor tables
        if in_mult > 1:
            shape = (1, 1)
        kh, kw = shape
        in_ch = s.groups[in_group].width * in_mult
        last = layer == n_layers - 1
        if not last and writable and rng.random() < 0.3:
            out_group = pick(*writable)                   # a second producer: residual add
        else:
            room = max(1, budget // max(1, in_ch * kh * kw * (n_layers - layer)))
            width = int(min(room, pick(1, 2, 3, 7, 16, 33, 64, 100, 257, 640)))
            s.groups.append(GroupDesc(width, 1 if last or rng.random() < 0.05 else 0))
            out_group = len(s.groups) - 1
            if not s.groups[out_group].pinned:
                writable.append(out_group)
            readable.append(out_group)
        out_ch = s.groups[out_group].width
        s.w_elems += int(rng.integers(0, 10)) if rng.random() < 0.5 else 0      # a gap
        t = TensorDesc(s.w_elems, out_ch, in_ch, kh, kw, in_mult, out_group, in_group,
                       0 if rng.random() < 0.12 else 1)
        s.tensors.append(t)
        s.w_elems += t.numel
        budget -= t.numel
    if not any(t.prunable for t in s.tensors):
        s.tensors[0].prunable = 1
    for g, grp in enumerate(s.groups):
        for _ in range(int(rng.integers(0, 4))):
            s.v_elems += int(rng.integers(0, 4)) if rng.random() < 0.3 else 0
            s.vecs.append(VecDesc(s.v_elems, grp.width, g))
            s.v_elems += grp.width
    s.w_elems += int(rng.integers(0, 5))
    return s


def random_weights(spec: NetSpec, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Arenas for ``random_spec``: per tensor one of the adversarial value patterns or
    filter-scaled Gaussians, then whole filters and whole input features scaled to almost
    nothing or set to zero; gaps hold a sentinel that no step may touch."""
    rng = np.random.Generator(np.random.Philox(SEED_BASE + 2000 + seed))
    w = np.full(max(spec.w_elems, 4), 12345.0, dtype=np.float32)
    v = rng.standard_normal(max(spec.v_elems, 4)).astype(np.float32)
    kinds = ("gauss", "gauss", "gauss", "half_zero", "quantised", "inf_negzero", "denormal",
             "all_equal", "all_zero", "ramp_desc_signed")
    for ti, t in enumerate(spec.tensors):
        kind = kinds[int(rng.integers(0, len(kinds)))]
        x = adversarial_arena(kind, t.numel, seed * 131 + ti).reshape(t.out_ch, t.in_ch, t.kh * t.kw)
        if kind == "gauss":
            x = x * np.exp(rng.normal(0.0, 1.5, size=(t.out_ch, 1, 1))).astype(np.float32)
        rows = rng.random(t.out_ch) < 0.3
        cols = rng.random(t.in_ch) < 0.2
        with np.errstate(invalid="ignore"):
            x[rows] *= np.float32(0.0 if rng.random() < 0.5 else 1e-6)
            x[:, cols] *= np.float32(0.0 if rng.random() < 0.5 else 1e-6)
        x[np.isnan(x)] = np.float32("inf")                # inf * 0: NaN is not a valid weight
        w[t.offset:t.offset + t.numel] = x.reshape(-1)
    return w, v
