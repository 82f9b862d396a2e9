"""Network topologies and seeded weights for the five synthetic workloads.

A network is a DAG of *sites* (tensor positions that own state: the network
input, every pre-activation tensor and every network output) joined by
*edges* (a k x k convolution, optionally followed by a nearest-neighbour 2^n
upsampling, the identity for a residual skip, or a k x k max pooling).
Sites are listed in topological order; edges are listed grouped by source
site and, for one destination, in the order their contributions are applied.

Only data is defined here: shapes, strides, thresholds, weights and biases.
Border widths, ring addressing and everything else the method computes is
derived separately by each consumer.

Weight layout: `w[tap][cout][cin]` with `tap = ky*k + kx`, already rounded to
the storage dtype so every consumer sees the same bits.  Biases are float32.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

CONFIG_NAMES = {
    1: "single_conv_64",
    2: "cnn5_256",
    3: "resnet18_512",
    4: "hrnet_w32_384x288",
    5: "bottleneck_density_128",
}

BASE_SEED = 221009887


@dataclass
class SiteSpec:
    name: str
    C: int
    stride: int          # down-sampling factor relative to the network input
    kind: str            # "input" | "preact" | "output"
    relu: bool
    theta: float
    trunc_free: bool = False   # the site keeps accumulated values only and never truncates (see truncation_free)


@dataclass
class EdgeSpec:
    src: int
    dst: int
    k: int               # 0 = identity edge (residual skip)
    stride: int
    pad: int
    up: int              # log2 of the nearest-neighbour upsampling after the conv
    w: Optional[np.ndarray]   # [k*k, Cout, Cin] storage dtype, None for identity
    b: Optional[np.ndarray]   # [Cout] float32, None = no bias
    pool: bool = False        # True: k x k max pooling of the source's activations (no weights)


@dataclass
class NetSpec:
    name: str
    dtype: str           # "f32" | "f16"  (storage; arithmetic is fp32)
    H: int               # input view height
    W: int               # input view width
    total_stride: int    # camera tile edge in input pixels
    sites: List[SiteSpec] = field(default_factory=list)
    edges: List[EdgeSpec] = field(default_factory=list)

    @property
    def np_dtype(self):
        return np.float16 if self.dtype == "f16" else np.float32

    def site_hw(self, i: int):
        s = self.sites[i].stride
        return self.H // s, self.W // s

    def out_edges(self, i: int):
        return [e for e in self.edges if e.src == i]

    def terminal_sites(self):
        return [i for i, s in enumerate(self.sites) if s.kind == "output"]


class _Builder:
    def __init__(self, net: NetSpec, rng: np.random.Generator, bias_amp: float):
        self.net = net
        self.rng = rng
        self.bias_amp = bias_amp

    def site(self, name, C, stride, kind="preact", relu=True, theta=0.0) -> int:
        self.net.sites.append(SiteSpec(name, C, stride, kind, relu, float(theta)))
        return len(self.net.sites) - 1

    def conv(self, src, dst, k, stride=1, pad=None, up=0, gain=1.0, bias=True):
        cin = self.net.sites[src].C
        cout = self.net.sites[dst].C
        if pad is None:
            pad = k // 2
        std = np.sqrt(2.0 / (k * k * cin)) * gain
        w = self.rng.standard_normal((k * k, cout, cin)) * std
        w = w.astype(np.float32).astype(self.net.np_dtype)
        b = None
        if bias and self.bias_amp > 0:
            b = self.rng.uniform(-self.bias_amp, self.bias_amp, cout).astype(np.float32)
        self.net.edges.append(EdgeSpec(src, dst, k, stride, pad, up, w, b))

    def maxpool(self, src, dst, k, stride, pad=None):
        assert self.net.sites[src].C == self.net.sites[dst].C
        self.net.edges.append(EdgeSpec(src, dst, k, stride, k // 2 if pad is None else pad, 0, None, None, True))

    def identity(self, src, dst):
        assert self.net.sites[src].C == self.net.sites[dst].C
        self.net.edges.append(EdgeSpec(src, dst, 0, 1, 0, 0, None, None))

    def basic_block(self, x, C, stride, theta, name, out_kind="preact", branch_gain=0.5):
        """Two 3x3 convs with a skip; returns the site of the summed pre-activation."""
        sx = self.net.sites[x]
        s_out = sx.stride * stride
        mid = self.site(name + ".mid", C, s_out, "preact", True, theta)
        out = self.site(name + ".sum", C, s_out, out_kind, True, theta)
        self.conv(x, mid, 3, stride)
        # edges of one source site are emitted together: main branch first
        if sx.C != C or stride != 1:
            self.conv(x, out, 1, stride, pad=0)
        else:
            self.identity(x, out)
        self.conv(mid, out, 3, 1, gain=branch_gain)
        return out


def _sort_edges(net: NetSpec):
    """Group edges by source site (stable), the order the path walks them in."""
    net.edges.sort(key=lambda e: e.src)


def _single_conv(rng) -> NetSpec:
    net = NetSpec(CONFIG_NAMES[1], "f32", 64, 64, 1)
    b = _Builder(net, rng, bias_amp=0.0)
    x = b.site("in", 16, 1, "input", False, 0.05)
    y = b.site("out", 16, 1, "output", False, 0.0)
    b.conv(x, y, 3, 1)
    return net


def _cnn5(rng, H=256, W=256) -> NetSpec:
    net = NetSpec(CONFIG_NAMES[2], "f32", H, W, 4)
    b = _Builder(net, rng, bias_amp=0.1)
    th = 0.02
    x = b.site("in", 3, 1, "input", False, th)
    s1 = b.site("c1", 32, 2, theta=th)
    s2 = b.site("c2", 32, 2, theta=th)
    s3 = b.site("c3", 64, 2, theta=th)
    s4 = b.site("c4", 64, 4, theta=th)
    y = b.site("out", 64, 4, "output", False, 0.0)
    b.conv(x, s1, 3, 2)
    b.conv(s1, s2, 3, 1)
    b.conv(s2, s3, 1, 1, pad=0)
    b.conv(s3, s4, 3, 2)
    b.conv(s4, y, 3, 1)
    return net


def _resnet18(rng, H=512, W=512, widths=(64, 128, 256, 512), pool_stem=False, bn_scale=True) -> NetSpec:
    """3x3 stem with stride 2, then four stages of two basic blocks each, stage
    strides 1/2/2/1 (total stride 8), 1x1 projection wherever the shape changes.
    The second conv of every block carries a folded batch-norm scale of 0.5 so
    that activations stay O(1) in fp16 storage (bn_scale=False: plain He-normal weights
    everywhere, the variant the tolerance study compares with).  pool_stem: the usual ResNet
    stem, a 3x3 stride-2 max pooling after the stem convolution (total stride 16)."""
    net = NetSpec(CONFIG_NAMES[3] + ("_poolstem" if pool_stem else ""), "f16", H, W, 16 if pool_stem else 8)
    b = _Builder(net, rng, bias_amp=0.1)
    th_in, th = 0.02, 0.01
    x = b.site("in", 3, 1, "input", False, th_in)
    s = b.site("stem", widths[0], 2, theta=th)
    b.conv(x, s, 3, 2)
    if pool_stem:
        p = b.site("pool", widths[0], 4, "preact", False, th)
        b.maxpool(s, p, 3, 2)
        s = p
    strides = (1, 2, 2, 1)
    for si, (C, st) in enumerate(zip(widths, strides)):
        for bi in range(2):
            last = si == 3 and bi == 1
            s = b.basic_block(s, C, st if bi == 0 else 1, th, f"s{si + 1}b{bi}",
                              out_kind="output" if last else "preact", branch_gain=0.5 if bn_scale else 1.0)
    _sort_edges(net)
    return net


def _hrnet(rng, H=384, W=288, widths=(32, 64, 128, 256), blocks=4, bn_scale=True) -> NetSpec:
    """Two stride-2 3x3 stem convs, then three multi-resolution stages with
    2/3/4 parallel branches of `blocks` basic blocks each.  After every stage all
    branches are fused all-to-all: higher -> lower resolution through chains of
    3x3 stride-2 convs (ReLU between chain links), lower -> higher through a 1x1
    conv followed by nearest upsampling.  A new branch is opened from the fused
    lowest-resolution branch with a 3x3 stride-2 conv.  The network output is
    the fused highest-resolution branch of the last stage.  Total stride 32.
    Folded batch-norm scales (0.25 on the second conv of every block, 0.35 on
    the fusion convs) keep the activations within a few units in fp16; bn_scale=False
    leaves all weights plain He-normal."""
    g_block, g_fuse = (0.25, 0.35) if bn_scale else (1.0, 1.0)
    net = NetSpec(CONFIG_NAMES[4], "f16", H, W, 32)
    b = _Builder(net, rng, bias_amp=0.1)
    th = 0.015
    x = b.site("in", 3, 1, "input", False, th)
    s1 = b.site("stem1", 64, 2, theta=th)
    b.conv(x, s1, 3, 2)
    s2 = b.site("stem2", 64, 4, theta=th)
    b.conv(s1, s2, 3, 2)
    br = [b.site("t1.b0", widths[0], 4, theta=th), b.site("t1.b1", widths[1], 8, theta=th)]
    b.conv(s2, br[0], 3, 1)
    b.conv(s2, br[1], 3, 2)
    for stage in range(2, 5):
        nb = len(br)
        for j in range(nb):
            for k in range(blocks):
                br[j] = b.basic_block(br[j], widths[j], 1, th, f"st{stage}.b{j}.blk{k}", branch_gain=g_block)
        last_stage = stage == 4
        outs = [0] if last_stage else list(range(nb))
        fused = []
        for i in outs:
            kind = "output" if last_stage else "preact"
            fused.append(b.site(f"st{stage}.fuse{i}", widths[i], 4 << i, kind, True, th))
        for oi, i in enumerate(outs):
            for j in range(nb):
                if j == i:
                    b.identity(br[j], fused[oi])
                elif j > i:
                    b.conv(br[j], fused[oi], 1, 1, pad=0, up=j - i, gain=g_fuse)
                else:
                    cur = br[j]
                    for step in range(i - j - 1):
                        nxt = b.site(f"st{stage}.down{j}to{i}.{step}", widths[j],
                                     net.sites[cur].stride * 2, theta=th)
                        b.conv(cur, nxt, 3, 2)
                        cur = nxt
                    b.conv(cur, fused[oi], 3, 2, gain=g_fuse)
        if last_stage:
            br = fused
        else:
            new = b.site(f"t{stage}.b{nb}", widths[nb], 4 << nb, theta=th)
            b.conv(fused[-1], new, 3, 2)
            br = fused + [new]
    _toposort(net)
    return net


def _bottleneck(rng, H=128, W=128, C=256, Cm=64) -> NetSpec:
    net = NetSpec(CONFIG_NAMES[5], "f16", H, W, 1)
    b = _Builder(net, rng, bias_amp=0.1)
    x = b.site("in", C, 1, "input", False, 0.0)
    m1 = b.site("conv1", Cm, 1, theta=0.0)
    m2 = b.site("conv2", Cm, 1, theta=0.0)
    y = b.site("sum", C, 1, "output", True, 0.0)
    b.conv(x, m1, 1, 1, pad=0)
    b.identity(x, y)
    b.conv(m1, m2, 3, 1)
    b.conv(m2, y, 1, 1, pad=0, gain=0.5)
    return net


def _toposort(net: NetSpec):
    """Renumber sites so that every edge goes from a lower to a higher index and
    group the edges by source (stable).  Needed when sites are created out of
    dataflow order (multi-branch fusion)."""
    n = len(net.sites)
    indeg = [0] * n
    for e in net.edges:
        indeg[e.dst] += 1
    order, ready = [], [i for i in range(n) if indeg[i] == 0]
    while ready:
        i = ready.pop(0)
        order.append(i)
        for e in net.edges:
            if e.src == i:
                indeg[e.dst] -= 1
                if indeg[e.dst] == 0:
                    ready.append(e.dst)
        ready.sort()
    assert len(order) == n, "network graph has a cycle"
    new_of = {old: new for new, old in enumerate(order)}
    net.sites = [net.sites[old] for old in order]
    for e in net.edges:
        e.src, e.dst = new_of[e.src], new_of[e.dst]
    _sort_edges(net)


def truncation_free(net: NetSpec, only=None) -> NetSpec:
    """Marks the sites that may run without truncation: inner sites whose only producer is a 1x1
    convolution (no upsampling) - the activation layers that do not follow a 3x3 convolution.  Such a
    site keeps no truncated-values buffer; every update it receives is passed on.  `only`: restrict the
    marking to these site indices.  Returns `net` (modified in place)."""
    for i, s in enumerate(net.sites):
        prods = [e for e in net.edges if e.dst == i]
        ok = (s.kind == "preact" and len(prods) == 1 and prods[0].k == 1 and prods[0].up == 0 and prods[0].pad == 0
              and not prods[0].pool)
        s.trunc_free = bool(ok and (only is None or i in only))
        if s.trunc_free:
            s.theta = 0.0
    return net


def build_net(config: int, **overrides) -> NetSpec:
    """Network of benchmark workload `config` (1..5); `overrides` shrink the input
    size or the widths for quick parity cases (same topology, same seed)."""
    rng = np.random.default_rng(np.random.PCG64(BASE_SEED + 100 + config))
    fn = {1: _single_conv, 2: _cnn5, 3: _resnet18, 4: _hrnet, 5: _bottleneck}[config]
    net = fn(rng, **overrides)
    for s in net.sites:
        assert net.H % s.stride == 0 and net.W % s.stride == 0
        assert net.total_stride % s.stride == 0
    for e in net.edges:
        assert e.src < e.dst
    return net


def tiny_net(dtype="f32", H=6, W=6, C=(1, 2, 1), k=3, stride=1, relu=True, theta=0.0,
             seed=0, bias_amp=0.1, total_stride=None) -> NetSpec:
    """Chain of len(C)-1 convs for brute-force tests."""
    rng = np.random.default_rng(seed)
    ts = total_stride if total_stride is not None else stride ** (len(C) - 1)
    net = NetSpec("tiny", dtype, H, W, ts)
    b = _Builder(net, rng, bias_amp)
    prev = b.site("in", C[0], 1, "input", False, theta)
    st = 1
    for i, c in enumerate(C[1:]):
        st *= stride
        last = i == len(C) - 2
        cur = b.site(f"l{i}", c, st, "output" if last else "preact",
                     False if last else relu, 0.0 if last else theta)
        b.conv(prev, cur, k, stride)
        prev = cur
    return net


def pool_net(dtype="f32", H=16, W=16, C=(2, 4, 3), k=3, stride=2, pad=1, theta=0.0, seed=0, bias_amp=0.1,
             relu=True) -> NetSpec:
    """input -> 3x3 conv -> activation site -> k x k max pooling -> site -> 3x3 conv -> output."""
    rng = np.random.default_rng(seed)
    net = NetSpec("pool", dtype, H, W, stride)
    b = _Builder(net, rng, bias_amp)
    x = b.site("in", C[0], 1, "input", False, theta)
    a = b.site("act", C[1], 1, "preact", relu, theta)
    p = b.site("pool", C[1], stride, "preact", False, theta)
    y = b.site("out", C[2], stride, "output", False, 0.0)
    b.conv(x, a, 3, 1)
    b.maxpool(a, p, k, stride, pad)
    b.conv(p, y, 3, 1)
    return net


def pool_front_net(dtype="f32", H=16, W=16, C=(3, 2), k=3, stride=2, pad=1, theta=0.0, seed=0) -> NetSpec:
    """input -> k x k max pooling -> site -> 1x1 conv -> output (pooling straight on the frames)."""
    rng = np.random.default_rng(seed)
    net = NetSpec("pool_front", dtype, H, W, stride)
    b = _Builder(net, rng, 0.1)
    x = b.site("in", C[0], 1, "input", False, theta)
    p = b.site("pool", C[0], stride, "preact", False, theta)
    y = b.site("out", C[1], stride, "output", False, 0.0)
    b.maxpool(x, p, k, stride, pad)
    b.conv(p, y, 1, 1, pad=0)
    return net


def random_dag_net(seed: int, dtype="f32", tiles=(5, 4), theta=0.05, n_inner=7) -> NetSpec:
    """A seeded random network for differential tests: sites at strides 1 / 2 / 4 with one to
    three producers each - convolutions (1x1, 3x3, strided 3x3 and 5x5), residual skips, 1x1
    convolutions with nearest upsampling, max pooling - and one or two outputs.  Every site but
    the input has a producer and every inner site a consumer; edges go from lower to higher
    site indices and are grouped by source."""
    rng = np.random.default_rng(seed)
    T = 4
    net = NetSpec(f"dag{seed}", dtype, tiles[0] * T, tiles[1] * T, T)
    b = _Builder(net, rng, 0.1)
    chans = [8, 16, 24, 32] if dtype == "f16" else [3, 5, 8, 16]
    b.site("in", int(rng.choice([3, 4, 8])), 1, "input", False, theta)
    pooled = set()

    def connect(src, dst):
        s, d = net.sites[src], net.sites[dst]
        if d.stride == s.stride:
            if s.C == d.C and dst not in pooled and rng.random() < 0.4:
                b.identity(src, dst)
            else:
                k = int(rng.choice([1, 3]))
                b.conv(src, dst, k, 1, gain=0.7)
        elif d.stride > s.stride:
            f = d.stride // s.stride
            if f == 2 and s.C == d.C and s.kind != "input" and dst in pooled:
                k = int(rng.choice([2, 3]))
                b.maxpool(src, dst, k, 2, 0 if k == 2 else 1)
            else:
                b.conv(src, dst, 3 if f == 2 else 5, f, gain=0.7)
        else:
            up = {2: 1, 4: 2}[s.stride // d.stride]
            b.conv(src, dst, 1, 1, pad=0, up=up, gain=0.7)

    for i in range(n_inner):
        stride = int(rng.choice([1, 2, 4]))
        last = i >= n_inner - int(rng.integers(1, 3))
        C = int(rng.choice(chans))
        prods = sorted(set(int(v) for v in rng.choice(len(net.sites), size=int(rng.integers(1, 4)))))
        prods = [p for p in prods if net.sites[p].kind != "output"] or [0]
        # a pooled site takes a pooling from a producer at half its stride with the same channels
        cand = [p for p in prods if net.sites[p].stride * 2 == stride and net.sites[p].kind == "preact"]
        if cand and not last and rng.random() < 0.5:
            C = net.sites[cand[0]].C
        dst = b.site(f"s{i}", C, stride, "output" if last else "preact", bool(rng.random() < 0.7) and not last, 0.0 if last else theta)
        if cand and not last and net.sites[cand[0]].C == C and rng.random() < 0.7:
            pooled.add(dst)
        for p in prods:
            if dst in pooled and p != cand[0] and rng.random() < 0.5:
                continue
            connect(p, dst)
        if dst in pooled and not any(e.pool for e in net.edges if e.dst == dst):
            pooled.discard(dst)
    # inner sites without a consumer feed the last output
    outs = net.terminal_sites()
    for i, s in enumerate(net.sites):
        if s.kind == "preact" and not net.out_edges(i):
            tgt = [o for o in outs if o > i]
            if tgt:
                connect(i, tgt[-1])
            else:
                s.kind, s.relu, s.theta = "output", False, 0.0
    # a pooling edge needs a destination that keeps its previous outputs: PREACT only
    for e in net.edges:
        if e.pool and net.sites[e.dst].kind != "preact":
            e.pool, e.k, e.stride, e.pad = False, 3, 2, 1
            std = np.sqrt(2.0 / (9 * net.sites[e.src].C)) * 0.7
            e.w = (rng.standard_normal((9, net.sites[e.dst].C, net.sites[e.src].C)) * std).astype(np.float32).astype(net.np_dtype)
    _sort_edges(net)
    for e in net.edges:
        assert e.src < e.dst
    return net
