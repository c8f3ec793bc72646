"""Seeded synthetic inputs with the layer shapes and value distributions of the paper's workloads.

This module serves both the CPU oracle's tests and the HIP library's tests and
benchmark.  It holds no arithmetic of the method (no GEMM, no requantization, no
range update): it only draws real-valued tensors and hands them over the way the
layer path receives them, as 8-bit codes with a scale and a zero point.

The paper trains ResNet18 / VGG16 / MobileNetV2 on Tiny ImageNet and ImageNet
(Sec. 5); neither the datasets nor trained weights are used here.  The tensors
below take those networks' layer shapes (Table 5 and the public architectures)
and the distributions the paper describes -- post-ReLU activations, He-normal
weights, heavy-tailed, drifting, Laplace-like gradients (Sec. 1, Sec. 3.1) --
and stand in for them.
"""
from collections import namedtuple

import numpy as np

SEED0 = 210504246

LayerShape = namedtuple("LayerShape", "name kind B H W C R S stride pad Cout")
LINEAR, CONV, DEPTHWISE = 0, 1, 2

QTensor = namedtuple("QTensor", "codes scale zero_point")     # int8 ndarray, np.float32, int


def out_hw(L):
    return ((L.H + 2 * L.pad - L.R) // L.stride + 1, (L.W + 2 * L.pad - L.S) // L.stride + 1)


def in_shape(L):
    return (L.B, L.H, L.W, L.C)


def out_shape(L):
    oh, ow = out_hw(L)
    return (L.B, oh, ow, L.Cout)


def w_shape(L):
    return (L.R, L.S, L.C) if L.kind == DEPTHWISE else (L.Cout, L.R, L.S, L.C)


def macs(L):
    """Multiply-accumulates of one of the three linear operations of the layer."""
    oh, ow = out_hw(L)
    per_out = L.R * L.S * (1 if L.kind == DEPTHWISE else L.C)
    return L.B * oh * ow * L.Cout * per_out


def linear(name, M, K, N):
    return LayerShape(name, LINEAR, M, 1, 1, K, 1, 1, 1, 0, N)


def conv(name, B, HW, Cin, Cout, k, stride=1, pad=None):
    return LayerShape(name, CONV, B, HW, HW, Cin, k, k, stride, k // 2 if pad is None else pad, Cout)


def depthwise(name, B, HW, Ch, k=3, stride=1):
    return LayerShape(name, DEPTHWISE, B, HW, HW, Ch, k, k, stride, k // 2, Ch)


def rng(config, t=0, salt=0):
    return np.random.default_rng([SEED0, int(config), int(t), int(salt)])


# ---------------------------------------------------------------------------
# real tensor -> (codes, scale, zero point): how an operand arrives at the layer
# ---------------------------------------------------------------------------

def to_unsigned_codes(x, scale):
    """Non-negative real tensor on the grid 0..255 with real 0 at code 0, stored shifted by -128."""
    u = np.clip(np.rint(x / np.float32(scale)), 0, 255)
    return QTensor((u - 128).astype(np.int8), np.float32(scale), -128)


def to_symmetric_codes(x, scale):
    q = np.clip(np.rint(x / np.float32(scale)), -127, 127)
    return QTensor(q.astype(np.int8), np.float32(scale), 0)


def to_asymmetric_codes(x):
    """Signed real tensor on an asymmetric 8-bit grid spanning its own min..max (widened to hold 0)."""
    lo, hi = min(float(x.min()), 0.0), max(float(x.max()), 0.0)
    scale = np.float32((hi - lo) / 255.0) if hi > lo else np.float32(1.0)
    z = int(np.clip(np.rint(-128 - lo / scale), -128, 127))
    q = np.clip(np.rint(x / scale) + z, -128, 127)
    return QTensor(q.astype(np.int8), scale, z)


def relu_activation(g, shape, gain=1.0):
    """Post-ReLU activation: gain * max(N(0,1), 0)."""
    x = g.standard_normal(shape, dtype=np.float32)
    np.maximum(x, 0, out=x)
    x *= np.float32(gain)
    return to_unsigned_codes(x, max(float(x.max()), 1e-12) / 255.0)


def relu6_activation(g, shape):
    """ReLU6-clipped activation: min(max(N(0, 3^2), 0), 6), scale 6/255."""
    x = g.standard_normal(shape, dtype=np.float32)
    x *= np.float32(3.0)
    np.clip(x, 0, 6, out=x)
    return to_unsigned_codes(x, 6.0 / 255.0)


def normal_image(g, shape):
    """Network input: N(0,1), asymmetric grid."""
    return to_asymmetric_codes(g.standard_normal(shape, dtype=np.float32))


def normal_weight(g, shape, sigma):
    w = g.standard_normal(shape, dtype=np.float32) * np.float32(sigma)
    return to_symmetric_codes(w, max(float(np.abs(w).max()), 1e-12) / 127.0)


def he_weight(g, L):
    fan_in = L.R * L.S * (1 if L.kind == DEPTHWISE else L.C)
    return normal_weight(g, w_shape(L), np.sqrt(2.0 / fan_in))


def laplace_gradient(g, shape, b, outlier_frac=0.0, outlier_gain=20.0):
    """Activation gradient: Laplace(0, b), optionally a fraction of elements scaled up."""
    x = g.laplace(0.0, b, size=shape).astype(np.float32)
    if outlier_frac > 0:
        mask = g.random(shape, dtype=np.float32) < outlier_frac
        x[mask] *= np.float32(outlier_gain)
    return to_symmetric_codes(x, max(float(np.abs(x).max()), 1e-30) / 127.0)


def real_activation(g, n, gain=1.0, shift=0.0):
    """FP32 tensor as a normalisation layer followed by ReLU hands it on: gain * max(N(0,1) + shift, 0)."""
    x = g.standard_normal(n, dtype=np.float32)
    x += np.float32(shift)
    np.maximum(x, 0, out=x)
    x *= np.float32(gain)
    return x


def real_gradient(g, n, b, outlier_frac=0.01, outlier_gain=20.0):
    """FP32 activation gradient: Laplace(0, b) with a fraction of outliers."""
    x = g.laplace(0.0, b, size=n).astype(np.float32)
    mask = g.random(n, dtype=np.float32) < outlier_frac
    x[mask] *= np.float32(outlier_gain)
    return x


# ---------------------------------------------------------------------------
# the five configurations
# ---------------------------------------------------------------------------

def c1_layer():
    return linear("c1_linear", 256, 512, 512)


def c1_inputs(t):
    """Single linear layer, iteration t: fresh X = ReLU(N(0,1)); fixed W ~ N(0, 0.05^2);
    dY ~ Laplace(0, 1e-2 * 0.8^t)."""
    L = c1_layer()
    X = relu_activation(rng(1, t, 0), in_shape(L))
    W = normal_weight(rng(1, 0, 1), w_shape(L), 0.05)
    dY = laplace_gradient(rng(1, t, 2), out_shape(L), 1e-2 * 0.8 ** t)
    return L, X, W, dY


def c2_layer(B=128):
    return conv("c2_conv3x3_64", B, 56, 64, 64, 3)


def c2_inputs(t, B=128):
    """ResNet-style 3x3 conv 64->64 at 56x56: activation scale grows by 1.05 per iteration."""
    L = c2_layer(B)
    X = relu_activation(rng(2, t, 0), in_shape(L), gain=1.05 ** t)
    W = he_weight(rng(2, 0, 1), L)
    return L, X, W


def c3_layer(B=128):
    return conv("c3_conv3x3_128", B, 28, 128, 128, 3)


def c3_grad_scale(t, T=50):
    """Geometric decay 1 -> 1e-3 over T iterations."""
    return 10.0 ** (-3.0 * t / (T - 1))


def c3_inputs(t, B=128):
    """Backward of a 3x3 conv 128->128 at 28x28: decaying Laplace gradients with 1% outliers at 20x."""
    L = c3_layer(B)
    dY = laplace_gradient(rng(3, t, 0), out_shape(L), c3_grad_scale(t), 0.01, 20.0)
    W = he_weight(rng(3, 0, 1), L)
    X = relu_activation(rng(3, t, 2), in_shape(L))
    return L, X, W, dY


def c4_layers(B=128):
    """MobileNetV2 inverted-residual block at 56x56, expansion 6."""
    return [conv("c4_expand_1x1", B, 56, 32, 192, 1),
            depthwise("c4_dw_3x3", B, 56, 192),
            conv("c4_project_1x1", B, 56, 192, 32, 1)]


def c4_inputs(t, B=128):
    """Independent inputs per layer: ReLU6 activations, He weights, Laplace gradients."""
    out = []
    for i, L in enumerate(c4_layers(B)):
        X = relu6_activation(rng(4, t, 10 * i), in_shape(L))
        W = he_weight(rng(4, 0, 10 * i + 1), L)
        dY = laplace_gradient(rng(4, t, 10 * i + 2), out_shape(L), 1e-3)
        out.append((L, X, W, dY))
    return out


def resnet18_layers(B=256, image=224):
    """ResNet-18-shaped stack: stem on 3-channel images, 4 stages of 3x3 convs with 1x1 stride-2
    shortcuts, FC."""
    s = image // 4                                            # after stem /2 and max-pool /2
    layers = [conv("stem_7x7", B, image, 3, 64, 7, stride=2)]
    layers += [conv("s1_conv%d" % i, B, s, 64, 64, 3) for i in range(4)]
    cin = 64
    for stage, cout in ((2, 128), (3, 256), (4, 512)):
        layers.append(conv("s%d_conv0" % stage, B, s, cin, cout, 3, stride=2))
        layers.append(conv("s%d_short" % stage, B, s, cin, cout, 1, stride=2, pad=0))
        s //= 2
        layers += [conv("s%d_conv%d" % (stage, i), B, s, cout, cout, 3) for i in range(1, 4)]
        cin = cout
    layers.append(linear("fc", B, 512, 1000))
    return layers


def vgg16_layers(B=256, image=64, classes=200):
    """VGG16-shaped stack (13 3x3 convs in five blocks with 2x2 pooling between them, three
    linear layers) on 64x64 3-channel images with 200 classes, the size of the Tiny ImageNet runs."""
    layers, cin, s = [], 3, image
    for block, (cout, n) in enumerate(((64, 2), (128, 2), (256, 3), (512, 3), (512, 3))):
        for i in range(n):
            layers.append(conv("b%d_conv%d" % (block + 1, i), B, s, cin, cout, 3))
            cin = cout
        s //= 2
    layers.append(linear("fc1", B, cin * s * s, 4096))
    layers.append(linear("fc2", B, 4096, 4096))
    layers.append(linear("fc3", B, 4096, classes))
    return layers


def layer_inputs(L, config, t, index, image_input=False, grad_b=1e-3):
    """Independent synthetic operands for one layer of a stack."""
    g = rng(config, t, 100 * index)
    if image_input:
        X = normal_image(g, in_shape(L))
    else:
        X = relu_activation(g, in_shape(L))
    W = he_weight(rng(config, 0, 100 * index + 1), L)
    dY = laplace_gradient(rng(config, t, 100 * index + 2), out_shape(L), grad_b)
    return X, W, dY


# ---------------------------------------------------------------------------
# algorithmic HBM bytes of one operation (each operand byte charged once)
# ---------------------------------------------------------------------------

def nelem(shape):
    n = 1
    for d in shape:
        n *= int(d)
    return n


def fused_bytes(L, op):
    """Bytes the static (in-hindsight) path must move: operands in, low-bit result out."""
    x, y, w = nelem(in_shape(L)), nelem(out_shape(L)), nelem(w_shape(L))
    if op == "fwd":
        return x + w + y
    if op == "dgrad":
        return y + w + x
    if op == "wgrad":
        return x + y + 4 * w
    raise ValueError(op)


def dynamic_bytes(L, op):
    """Bytes of the dynamic two-pass path: adds one save and one load of the 32-bit output."""
    if op == "wgrad":
        return fused_bytes(L, op)
    out = nelem(out_shape(L)) if op == "fwd" else nelem(in_shape(L))
    return fused_bytes(L, op) + 8 * out
