"""Synthetic workloads: layer lists shaped like the networks the paper trains
(AlexNet, VGG-16, ResNet-50, Inception-v4; Sec. 4) and seeded input generators.

This module holds no layer arithmetic.  It serves both the HIP path and the
tests' CPU oracle, which must see the same values: tensors are drawn on the CPU
with torch's generator and already rounded to their storage type (fp32, or bf16
round-to-nearest-even), so widening them to fp64 for the oracle is exact.
"""
from collections import namedtuple

import torch

# One convolution layer.  relu_in: its input comes after a ReLU (so it is drawn
# as max(N(0,1), 0)); pool: (kernel, stride) of the max-pool that follows, or
# None; mult: how many times the shape occurs in the network; first: the image
# layer (its backward-data is reported apart); lrn: (size, alpha, beta, k) of the LRN
# between the ReLU and the pool, or None.
Layer = namedtuple("Layer", "name C H W K R S stride pad relu_in pool mult first lrn")


def _L(name, C, H, W, K, R, S, stride=(1, 1), pad=(0, 0), relu_in=True, pool=None, mult=1, first=False, lrn=None):
    return Layer(name, C, H, W, K, R, S, stride, pad, relu_in, pool, mult, first, lrn)


def out_hw(layer):
    P = (layer.H + 2 * layer.pad[0] - layer.R) // layer.stride[0] + 1
    Q = (layer.W + 2 * layer.pad[1] - layer.S) // layer.stride[1] + 1
    return P, Q


def _vgg16():
    cfg = [(64, 2, 224), (128, 2, 112), (256, 3, 56), (512, 3, 28), (512, 3, 14)]
    layers, c_in = [], 3
    for bi, (k, reps, hw) in enumerate(cfg, 1):
        for r in range(1, reps + 1):
            layers.append(_L("conv%d_%d" % (bi, r), c_in, hw, hw, k, 3, 3, (1, 1), (1, 1),
                             relu_in=c_in != 3, pool=((2, 2), (2, 2)) if r == reps else None,
                             first=c_in == 3))
            c_in = k
    return layers


def _alexnet():
    return [
        # CONV -> ReLU -> LRN -> POOL, as in the paper's AlexNet example (Sec. 4); AlexNet's LRN constants
        _L("conv1", 3, 227, 227, 96, 11, 11, (4, 4), (0, 0), relu_in=False, pool=((3, 3), (2, 2)), first=True,
           lrn=(5, 1e-4, 0.75, 2.0)),
        _L("conv2", 96, 27, 27, 256, 5, 5, (1, 1), (2, 2), pool=((3, 3), (2, 2)), lrn=(5, 1e-4, 0.75, 2.0)),
        _L("conv3", 256, 13, 13, 384, 3, 3, (1, 1), (1, 1)),
        _L("conv4", 384, 13, 13, 384, 3, 3, (1, 1), (1, 1)),
        _L("conv5", 384, 13, 13, 256, 3, 3, (1, 1), (1, 1), pool=((3, 3), (2, 2))),
    ]


def _resnet50():
    layers = []
    stages = [(64, 56, 3, 64), (128, 28, 4, 256), (256, 14, 6, 512), (512, 7, 3, 1024)]
    for si, (w, hw, blocks, c_prev) in enumerate(stages, 2):
        if si == 2:
            layers.append(_L("s2_reduce_first", 64, hw, hw, w, 1, 1))
            layers.append(_L("s2_project", 64, hw, hw, 4 * w, 1, 1))
            n33 = blocks
        else:
            big = 2 * hw
            # stage entry, stride on the first 1x1 (original form) ...
            layers.append(_L("s%d_reduce_s2" % si, c_prev, big, big, w, 1, 1, (2, 2)))
            # ... or on the 3x3 (later form), fed by an unstrided reduce
            layers.append(_L("s%d_reduce_entry" % si, c_prev, big, big, w, 1, 1))
            layers.append(_L("s%d_conv3x3_s2" % si, w, big, big, w, 3, 3, (2, 2), (1, 1)))
            layers.append(_L("s%d_project_s2" % si, c_prev, big, big, 4 * w, 1, 1, (2, 2)))
            n33 = blocks - 1
        layers.append(_L("s%d_reduce" % si, 4 * w, hw, hw, w, 1, 1, mult=blocks - 1))
        layers.append(_L("s%d_conv3x3" % si, w, hw, hw, w, 3, 3, (1, 1), (1, 1), mult=n33))
        layers.append(_L("s%d_expand" % si, w, hw, hw, 4 * w, 1, 1, mult=blocks))
    return layers


def _inception_like():
    return [
        _L("a_1x1_96", 384, 35, 35, 96, 1, 1),
        _L("a_1x1_64", 384, 35, 35, 64, 1, 1),
        _L("a_1x1_32", 384, 35, 35, 32, 1, 1),
        _L("a_3x3_64_96", 64, 35, 35, 96, 3, 3, (1, 1), (1, 1)),
        _L("a_3x3_96_96", 96, 35, 35, 96, 3, 3, (1, 1), (1, 1)),
        _L("a_5x5_48_64", 48, 35, 35, 64, 5, 5, (1, 1), (2, 2)),
        _L("ra_3x3_s2", 384, 35, 35, 384, 3, 3, (2, 2), (0, 0), pool=None),
        _L("b_1x1_192", 384, 17, 17, 192, 1, 1),
        _L("b_1x7", 192, 17, 17, 224, 1, 7, (1, 1), (0, 3)),
        _L("b_7x1", 224, 17, 17, 256, 7, 1, (1, 1), (3, 0)),
        _L("rb_3x3_s2", 192, 17, 17, 192, 3, 3, (2, 2), (0, 0)),
        _L("c_1x1_256", 384, 8, 8, 256, 1, 1),
        _L("c_3x3_256_384", 256, 8, 8, 384, 3, 3, (1, 1), (1, 1)),
    ]


MiB, GiB = 1 << 20, 1 << 30

# cfg number -> description of the workload (the five configurations of the build's target)
CONFIGS = {
    1: dict(name="cfg1_single_conv_fp32", N=2, dtype="f32", budgets=[0, None],
            layers=[_L("conv", 16, 16, 16, 16, 3, 3, (1, 1), (1, 1), relu_in=False, pool=((2, 2), (2, 2)),
                       first=False)],
            bn=False),
    2: dict(name="cfg2_alexnet_n128", N=128, dtype="bf16", budgets=[0, 64 * MiB, 1 * GiB], layers=_alexnet(),
            bn=False),
    3: dict(name="cfg3_vgg16_n32", N=32, dtype="bf16", budgets=[0, 256 * MiB, 2 * GiB], layers=_vgg16(), bn=True),
    4: dict(name="cfg4_resnet50_n64", N=64, dtype="bf16", budgets=[0, 512 * MiB], layers=_resnet50(), bn=True),
    5: dict(name="cfg5_inception_like_n64", N=64, dtype="bf16", budgets=[0, 32 * MiB], layers=_inception_like(),
            bn=True),
}
# cfg5's max-pools: the 3x3 stride-2 valid pool that sits beside each reduction conv, as (C, H, W)
INCEPTION_POOL_INPUTS = [(384, 35, 35), (384, 17, 17)]


def layer_seed(cfg, index):
    return 0 if cfg == 1 else 1000 * cfg + index


def _store(t, dtype):
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def conv_inputs(layer, N, dtype, seed):
    """x, w, dy for one layer as CPU tensors in their storage type.

    x ~ N(0,1), or max(N(0,1),0) after a ReLU; w ~ N(0, 2/(C*R*S)) (variance);
    dy ~ N(0,1)."""
    g = torch.Generator().manual_seed(seed)
    x = torch.randn((N, layer.C, layer.H, layer.W), generator=g, dtype=torch.float32)
    if layer.relu_in:
        x.clamp_(min=0)
    w = torch.randn((layer.K, layer.C, layer.R, layer.S), generator=g, dtype=torch.float32)
    w.mul_((2.0 / (layer.C * layer.R * layer.S)) ** 0.5)
    P, Q = out_hw(layer)
    dy = torch.randn((N, layer.K, P, Q), generator=g, dtype=torch.float32)
    return _store(x, dtype), _store(w, dtype), _store(dy, dtype)


def bn_params(C, seed):
    """gamma ~ U(0.5,1.5), beta ~ N(0,0.1), fp32."""
    g = torch.Generator().manual_seed(seed + 500)
    gamma = torch.rand(C, generator=g, dtype=torch.float32) + 0.5
    beta = torch.randn(C, generator=g, dtype=torch.float32) * 0.1
    return gamma, beta


def activation(shape, dtype, seed, relu=False, scale=1.0, shift=0.0):
    """A seeded activation / gradient tensor N(shift, scale^2), optionally after ReLU."""
    g = torch.Generator().manual_seed(seed)
    t = torch.randn(tuple(shape), generator=g, dtype=torch.float32) * scale + shift
    if relu:
        t.clamp_(min=0)
    return _store(t, dtype)


def conv_flops(layer, N):
    """(nominal, algorithmic) FLOP of one direction: 2*N*K*C*T_h*T_w with T counting
    all taps (nominal) or only taps that touch real pixels (algorithmic)."""
    P, Q = out_hw(layer)

    def taps(size, out, filt, stride, pad):
        return sum(1 for p in range(out) for r in range(filt) if 0 <= p * stride + r - pad < size)

    th = taps(layer.H, P, layer.R, layer.stride[0], layer.pad[0])
    tw = taps(layer.W, Q, layer.S, layer.stride[1], layer.pad[1])
    nominal = 2 * N * layer.K * layer.C * P * Q * layer.R * layer.S
    return nominal, 2 * N * layer.K * layer.C * th * tw
