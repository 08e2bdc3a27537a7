"""Seeded synthetic workloads for batch-1 Pipelined Backpropagation.

This module holds *inputs only*: the network descriptors of the benchmark
configurations (which layers sit in which pipeline stage) and the seeded
sample/label pools that stand in for the image-classification data the paper
trains on (Section 4: CIFAR-10 shaped 3x32x32 / 10 classes, ImageNet shaped
3x224x224 / 1000 classes).  None of the method's arithmetic lives here (no
delays, no optimizer coefficients, no initial weights): both the CPU oracle
and the HIP library receive these descriptors as arguments and derive
everything else on their own.

A network is a dict:
    name, in_c, in_h, in_w, n_classes, stages, lr, momentum, act_dtype,
    n_pool, seed_data, ticks
``stages`` is a list of pipeline stages (Section 4: one weight layer per
stage, fused with its normalisation / activation / pooling / residual sum);
a stage is a list of op dicts with keys
    kind  in {"linear","conv","gn","relu","maxpool","gap","add","ce"}
    cin, cout, k, stride, pad, groups, bias, skip_from, proj
"""
from __future__ import annotations

import numpy as np

WEIGHT_SEED = 42


def _op(kind, cin=0, cout=0, k=0, stride=1, pad=0, groups=0, bias=0, skip_from=-1, proj=0):
    return dict(kind=kind, cin=cin, cout=cout, k=k, stride=stride, pad=pad,
                groups=groups, bias=bias, skip_from=skip_from, proj=proj)


def linear(cin, cout, bias=1):
    return _op("linear", cin=cin, cout=cout, k=1, bias=bias)


def conv(cin, cout, k, stride=1, pad=None, bias=0):
    return _op("conv", cin=cin, cout=cout, k=k, stride=stride,
               pad=(k // 2 if pad is None else pad), bias=bias)


def gn(groups, c):
    return _op("gn", cin=c, cout=c, groups=groups)


def relu():
    return _op("relu")


def maxpool(k, stride, pad=0):
    return _op("maxpool", k=k, stride=stride, pad=pad)


def gap():
    return _op("gap")


def add(skip_from, cin, cout, stride=1, proj=0):
    """Residual sum with the tensor that entered stage ``skip_from``; with
    proj=1 that tensor first goes through a 1x1 convolution (cin->cout, given
    stride, no bias) whose weights belong to the stage holding this op."""
    return _op("add", cin=cin, cout=cout, k=1, stride=stride, skip_from=skip_from, proj=proj)


def ce():
    return _op("ce")


# --------------------------------------------------------------------------
# network builders
# --------------------------------------------------------------------------
def mlp(dims=(64, 128, 128, 128, 10)):
    stages = []
    for i in range(len(dims) - 1):
        st = []
        if i > 0:
            st.append(relu())
        st.append(linear(dims[i], dims[i + 1], bias=1))
        if i == len(dims) - 2:
            st.append(ce())
        stages.append(st)
    return stages


def vgg(channels, pool_after, groups, in_c=3, n_classes=10, in_hw=32):
    stages = []
    c = in_c
    hw = in_hw
    for i, co in enumerate(channels):
        st = [conv(c, co, 3, 1, 1), gn(groups, co), relu()]
        if i in pool_after:
            st.append(maxpool(2, 2, 0))
            hw //= 2
        stages.append(st)
        c = co
    stages.append([linear(c * hw * hw, n_classes, bias=1), ce()])   # flatten in C,H,W order
    return stages


def preact_resnet_basic(widths, blocks_per_group, groups, in_c=3, n_classes=10,
                        extra_plain_stages=0):
    """Pre-activation ResNet with basic blocks (CIFAR form): stem conv, then
    blocks of two stages [GN,ReLU,conv] and [GN,ReLU,conv,add], then the head
    [GN,ReLU,global-average-pool,FC,CE]."""
    stages = [[conv(in_c, widths[0], 3, 1, 1)]]
    c = widths[0]
    for gi, w in enumerate(widths):
        for bi in range(blocks_per_group):
            stride = 2 if (gi > 0 and bi == 0) else 1
            a_idx = len(stages)
            stages.append([gn(groups, c), relu(), conv(c, w, 3, stride, 1)])
            need_proj = 1 if (stride != 1 or c != w) else 0
            stages.append([gn(groups, w), relu(), conv(w, w, 3, 1, 1),
                           add(a_idx, c, w, stride, need_proj)])
            c = w
    for _ in range(extra_plain_stages):
        stages.append([gn(groups, c), relu(), conv(c, c, 3, 1, 1)])
    stages.append([gn(groups, c), relu(), gap(), linear(c, n_classes, bias=1), ce()])
    return stages


def preact_resnet_bottleneck(layers=(3, 4, 6, 3), base=64, groups=32, in_c=3, n_classes=1000):
    """Pre-activation ResNet-50 form: 7x7/2 stem with GN, ReLU and a 3x3/2
    max-pool, bottleneck blocks of three stages (stride on the 3x3), head."""
    stages = [[conv(in_c, base, 7, 2, 3), gn(groups, base), relu(), maxpool(3, 2, 1)]]
    c = base
    for gi, n in enumerate(layers):
        mid = base * (2 ** gi)
        out = 4 * mid
        for bi in range(n):
            stride = 2 if (gi > 0 and bi == 0) else 1
            a_idx = len(stages)
            stages.append([gn(groups, c), relu(), conv(c, mid, 1, 1, 0)])
            stages.append([gn(groups, mid), relu(), conv(mid, mid, 3, stride, 1)])
            need_proj = 1 if (stride != 1 or c != out) else 0
            stages.append([gn(groups, mid), relu(), conv(mid, out, 1, 1, 0),
                           add(a_idx, c, out, stride, need_proj)])
            c = out
    stages.append([gn(groups, c), relu(), gap(), linear(c, n_classes, bias=1), ce()])
    return stages


def _net(name, stages, in_c, in_h, in_w, n_classes, lr, momentum, n_pool, seed_data, ticks,
         act_dtype="fp32"):
    return dict(name=name, stages=stages, in_c=in_c, in_h=in_h, in_w=in_w, n_classes=n_classes,
                lr=lr, momentum=momentum, n_pool=n_pool, seed_data=seed_data, ticks=ticks,
                act_dtype=act_dtype)


def config(name):
    """The five benchmark configurations plus small variants used by tests."""
    if name == "mlp":
        return _net("mlp", mlp(), 64, 1, 1, 10, 0.01, 0.9, 1024, 1235, 2000)
    if name == "vgg11":
        st = vgg((64, 128, 256, 256, 512, 512, 512, 512), (0, 1, 3, 5, 7), 8)
        return _net("vgg11", st, 3, 32, 32, 10, 0.005, 0.9, 1024, 1236, 20000)
    if name == "resnet20":
        st = preact_resnet_basic((16, 32, 64), 3, 4)
        return _net("resnet20", st, 3, 32, 32, 10, 0.005, 0.9, 1024, 1237, 50000)
    if name == "resnet50":
        st = preact_resnet_bottleneck()
        return _net("resnet50", st, 3, 224, 224, 1000, 0.001, 0.9, 256, 1238, 5000,
                    act_dtype="bf16")
    if name == "wide":
        st = preact_resnet_basic((64, 128, 256), 3, 4, extra_plain_stages=8)
        # (learning rate: at VGG-11's 0.005 the stages with delays of 38-54 updates diverge -- weights beyond
        # 1e200 within 140 ticks in float64 --, at half of it every weight stays bounded)
        return _net("wide", st, 3, 32, 32, 10, 0.0025, 0.9, 1024, 1239, 20000)
    # ---- small variants for fast tests (same structure, fewer channels) ----
    if name == "tiny_mlp":
        return _net("tiny_mlp", mlp((5, 7, 6, 4)), 5, 1, 1, 4, 0.05, 0.9, 16, 11, 64)
    if name == "tiny_vgg":
        st = vgg((8, 8, 16), (0, 2), 4, in_c=3, n_classes=5, in_hw=8)
        return _net("tiny_vgg", st, 3, 8, 8, 5, 0.02, 0.9, 16, 12, 64)
    if name == "tiny_resnet":
        st = preact_resnet_basic((4, 8), 1, 2, in_c=3, n_classes=5)
        return _net("tiny_resnet", st, 3, 8, 8, 5, 0.02, 0.9, 16, 13, 64)
    if name == "tiny_bottleneck":
        st = preact_resnet_bottleneck(layers=(1, 1), base=4, groups=2, in_c=3, n_classes=6)
        return _net("tiny_bottleneck", st, 3, 16, 16, 6, 0.01, 0.9, 16, 14, 64)
    if name == "resnet50_64":
        # the ResNet-50 stage structure at full channel widths on 64x64 inputs with
        # fp32 activations: exercises the 7x7/2 stem, the 3x3/2 max-pool, 1x1
        # convolutions, stride-2 3x3 convolutions and skips over two stages at a size
        # the float64 oracle handles in a test
        st = preact_resnet_bottleneck()
        return _net("resnet50_64", st, 3, 64, 64, 1000, 0.001, 0.9, 64, 1240, 200)
    if name == "resnet50_fp32":
        st = preact_resnet_bottleneck()
        return _net("resnet50_fp32", st, 3, 224, 224, 1000, 0.001, 0.9, 256, 1238, 5000)
    if name == "small_resnet":
        # ragged sizes: spans several tiles with tails in every kernel
        st = preact_resnet_basic((12, 20), 2, 4, in_c=3, n_classes=7)
        return _net("small_resnet", st, 3, 20, 20, 7, 0.01, 0.9, 32, 15, 200)
    if name == "split_resnet":
        # 32x32 and 16x16 maps with few channels: the weight gradients of these layers are
        # long reductions with few output tiles, which the engine splits over workgroups
        st = preact_resnet_basic((8, 16), 1, 4, in_c=3, n_classes=5)
        return _net("split_resnet", st, 3, 32, 32, 5, 0.01, 0.9, 16, 17, 100)
    if name == "odd_resnet":
        # odd map sizes (6x6, then 3x3): no row or map is a multiple of 4 wide, so the
        # scalar staging paths and the generic fused last stage run
        st = preact_resnet_basic((6, 10), 1, 2, in_c=3, n_classes=5)
        return _net("odd_resnet", st, 3, 6, 6, 5, 0.02, 0.9, 16, 16, 100)
    if name == "thin_vgg":
        # 192-channel 3x3 layers on 4x4 and 2x2 maps: matrix-vector-like layers that the engine runs as dot-product steps and whose weight gradient it
        # computes inside the update step (as for the 512-channel layers of VGG-11)
        st = vgg((16, 192, 192, 192), (0, 2, 3), 8, in_c=3, n_classes=5, in_hw=8)
        return _net("thin_vgg", st, 3, 8, 8, 5, 0.01, 0.9, 32, 18, 100)
    raise KeyError(name)


BENCH_CONFIGS = ("mlp", "vgg11", "resnet20", "resnet50", "wide")


def sample_pool(net, n=None, seed=None):
    """Fixed pool of inputs ~ N(0,1) (float32, NCHW) and labels uniform over
    the classes (int32); tick t consumes pool item t mod n."""
    n = net["n_pool"] if n is None else n
    seed = net["seed_data"] if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((n, net["in_c"], net["in_h"], net["in_w"]), dtype=np.float32)
    y = rng.integers(0, net["n_classes"], size=n, dtype=np.int32)
    return x, y


def stage_shapes(net):
    """[(in_shape, out_shape)] per stage, (C,H,W) tuples; structure only."""
    c, h, w = net["in_c"], net["in_h"], net["in_w"]
    out = []
    for st in net["stages"]:
        cin = (c, h, w)
        for o in st:
            k = o["kind"]
            if k == "conv":
                c = o["cout"]
                h = (h + 2 * o["pad"] - o["k"]) // o["stride"] + 1
                w = (w + 2 * o["pad"] - o["k"]) // o["stride"] + 1
            elif k == "linear":
                c, h, w = o["cout"], 1, 1
            elif k == "maxpool":
                h = (h + 2 * o["pad"] - o["k"]) // o["stride"] + 1
                w = (w + 2 * o["pad"] - o["k"]) // o["stride"] + 1
            elif k == "gap":
                h = w = 1
        out.append((cin, (c, h, w)))
    return out


def count_params(net):
    n = 0
    for st in net["stages"]:
        for o in st:
            if o["kind"] == "conv":
                n += o["cout"] * o["cin"] * o["k"] * o["k"] + (o["cout"] if o["bias"] else 0)
            elif o["kind"] == "linear":
                n += o["cout"] * o["cin"] + (o["cout"] if o["bias"] else 0)
            elif o["kind"] == "gn":
                n += 2 * o["cin"]
            elif o["kind"] == "add" and o["proj"]:
                n += o["cout"] * o["cin"]
    return n
