"""Seeded synthetic convolution workloads: layer shapes and input tensors.

This module serves the tests, the benchmark and the smoke check.  It holds none of the
method's arithmetic (no output-size rule, no convolution, no search): only the problem
parameters of each layer (Section 2.3 "State space": N, C_in, C_out, K_h, K_w, H, W,
Stride, Padding) and NumPy generators for x and w.

The paper measured on the convolution layers of a Caffe-trained ResNet-18 (Section 3,
N=1, 3x224x224) and on five production layers (Table 1).  Neither the model nor the images
are available, so every tensor here is a seeded random stand-in of the same shape family:
activations uniform on [-1,1] or [0,1] (post-ReLU-like), weights uniform or Kaiming-normal
with std sqrt(2/(C*R*S)).
"""
import math

import numpy as np

FIELDS = ("n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w", "pad_h", "pad_w",
          "dil_h", "dil_w")


def layer(name, n, c, hw, k, rs, stride=1, pad=0, dil=1, x_dist="u01", w_dist="kaiming",
          seed=0, count=1):
    """One convolution layer as a plain dict.  ``hw``, ``rs``, ``stride``, ``pad``, ``dil``
    take an int (square) or an (h, w) pair."""
    def pair(v):
        return (v, v) if isinstance(v, int) else tuple(v)
    (h, w), (r, s) = pair(hw), pair(rs)
    (sh, sw), (ph, pw), (dh, dw) = pair(stride), pair(pad), pair(dil)
    return dict(name=name, n=n, c=c, h=h, w=w, k=k, r=r, s=s, stride_h=sh, stride_w=sw,
                pad_h=ph, pad_w=pw, dil_h=dh, dil_w=dw, x_dist=x_dist, w_dist=w_dist,
                seed=seed, count=count)


def shape_key(l):
    """The 13 integers that identify a convolution problem."""
    return tuple(int(l[f]) for f in FIELDS)


def make_inputs(l):
    """(x, w) float32 arrays, NCHW and KCRS, from the layer's seed and distributions."""
    rx = np.random.default_rng(int(l["seed"]))
    rw = np.random.default_rng(int(l["seed"]) + 500)
    xs = (l["n"], l["c"], l["h"], l["w"])
    ws = (l["k"], l["c"], l["r"], l["s"])
    if l["x_dist"] == "u11":
        x = rx.uniform(-1.0, 1.0, size=xs)
    elif l["x_dist"] == "u01":
        x = rx.uniform(0.0, 1.0, size=xs)
    else:
        raise ValueError(l["x_dist"])
    if l["w_dist"] == "u11":
        w = rw.uniform(-1.0, 1.0, size=ws)
    elif l["w_dist"] == "kaiming":
        w = rw.normal(0.0, math.sqrt(2.0 / (l["c"] * l["r"] * l["s"])), size=ws)
    else:
        raise ValueError(l["w_dist"])
    return x.astype(np.float32), w.astype(np.float32)


def config1():
    """Tiny single layer the oracle finishes instantly."""
    return [layer("cfg1", 1, 16, 14, 16, 3, 1, 1, x_dist="u11", w_dist="u11", seed=0)]


def config2():
    """One 3x3 layer and the 7x7 stride-2 stem, batch 1."""
    return [layer("cfg2.c64_56", 1, 64, 56, 64, 3, 1, 1, x_dist="u11", seed=2000),
            layer("cfg2.stem", 1, 3, 224, 64, 7, 2, 3, x_dist="u11", seed=2001)]


def config3(n=16):
    """The four batched 3x3 layers (C=K) the throughput target is quoted on."""
    return [layer("cfg3.c%d_%d" % (c, hw), n, c, hw, c, 3, 1, 1, seed=3000 + i)
            for i, (c, hw) in enumerate([(64, 56), (128, 28), (256, 14), (512, 7)])]


def config4(n=16):
    """Pointwise and strided layers."""
    return [layer("cfg4.1x1_256_64_56", n, 256, 56, 64, 1, 1, 0, seed=4000),
            layer("cfg4.1x1_512_2048_7", n, 512, 7, 2048, 1, 1, 0, seed=4001),
            layer("cfg4.1x1s2_1024_2048_14", n, 1024, 14, 2048, 1, 2, 0, seed=4002),
            layer("cfg4.3x3s2_128_128_56", n, 128, 56, 128, 3, 2, 1, seed=4003)]


# Feature-map edge in each of the four residual stages of an ImageNet ResNet (224x224 input): the
# sizes are data of the workload, listed, not computed from strides.
STAGE_HW = (56, 28, 14, 7)


def resnet50_stack(n=1):
    """Config 5: every convolution of a ResNet-50 v1 bottleneck network, in network order.

    Stem 7x7/2 to 64; (max-pool halves 112 to 56, not a convolution); stages of [3,4,6,3]
    bottlenecks with widths 64/128/256/512 and expansion 4; the first 3x3 of stages 2-4 has
    stride 2; the first block of every stage has a 1x1 projection shortcut with the block's
    stride.  53 layers; each gets its own seed."""
    out = [layer("stem", n, 3, 224, 64, 7, 2, 3, x_dist="u11", seed=5000)]
    cin, idx = 64, 1
    for stage, (blocks, width) in enumerate(zip([3, 4, 6, 3], [64, 128, 256, 512])):
        for b in range(blocks):
            stride = 2 if (b == 0 and stage > 0) else 1
            # feature-map sizes written out: what the block receives, what its strided layers emit
            hw_out = STAGE_HW[stage]
            hw = STAGE_HW[stage - 1] if stride == 2 else hw_out
            tag = "s%db%d" % (stage + 1, b)
            out.append(layer(tag + ".c1", n, cin, hw, width, 1, 1, 0, seed=5000 + idx)); idx += 1
            out.append(layer(tag + ".c2", n, width, hw, width, 3, stride, 1, seed=5000 + idx)); idx += 1
            out.append(layer(tag + ".c3", n, width, hw_out, 4 * width, 1, 1, 0, seed=5000 + idx)); idx += 1
            if b == 0:
                out.append(layer(tag + ".proj", n, cin, hw, 4 * width, 1, stride, 0,
                                 seed=5000 + idx)); idx += 1
            cin = 4 * width
    return out


def table1_convs(n=1):
    """The five production layers of Table 1 (H, W read as the input size, no padding)."""
    rows = [("conv1a", 112, 96, 3, 64, 1), ("conv1b", 110, 94, 64, 96, 2),
            ("conv2", 54, 46, 96, 128, 2), ("conv3", 26, 22, 128, 256, 2),
            ("conv4", 12, 10, 256, 512, 1)]
    return [layer(nm, n, c, (h, w), k, 3, st, 0, x_dist="u11", seed=6000 + i)
            for i, (nm, h, w, c, k, st) in enumerate(rows)]


def resnet18_stack(n=1):
    """Every convolution of a ResNet-18 (basic blocks), the network of Section 3.1, at the
    224x224 input size: stem 7x7/2 to 64; max-pool to 56; stages of [2,2,2,2] blocks of two 3x3
    layers with widths 64/128/256/512; the first 3x3 of stages 2-4 has stride 2 and that block
    has a 1x1 stride-2 projection shortcut.  20 layers."""
    out = [layer("stem", n, 3, 224, 64, 7, 2, 3, x_dist="u11", seed=7000)]
    cin, idx = 64, 1
    for stage, width in enumerate([64, 128, 256, 512]):
        for b in range(2):
            stride = 2 if (b == 0 and stage > 0) else 1
            hw_out = STAGE_HW[stage]
            hw = STAGE_HW[stage - 1] if stride == 2 else hw_out
            tag = "s%db%d" % (stage + 1, b)
            out.append(layer(tag + ".c1", n, cin, hw, width, 3, stride, 1, seed=7000 + idx)); idx += 1
            out.append(layer(tag + ".c2", n, width, hw_out, width, 3, 1, 1, seed=7000 + idx)); idx += 1
            if stride == 2:
                out.append(layer(tag + ".proj", n, cin, hw, width, 1, 2, 0, seed=7000 + idx)); idx += 1
            cin = width
    return out


def unique_layers(layers):
    """Layers de-duplicated by shape (Section 3.1: same input/output shape, filter size,
    stride and padding means computationally identical), with multiplicities in ``count``."""
    seen, out = {}, []
    for l in layers:
        key = shape_key(l)
        if key in seen:
            out[seen[key]]["count"] += l.get("count", 1)
        else:
            seen[key] = len(out)
            out.append(dict(l))
    return out
