"""Seeded synthetic inputs shaped like the paper's CIFAR ResNet-18 workload.

This module only draws random numbers and names shapes.  It holds none of the
method's arithmetic (no transform, no quantizer, no convolution) and imports
neither the HIP binding nor the CPU oracle, so both sides can be fed the very
same arrays from it.

The paper evaluates on ResNet-18 for CIFAR-10/100 (Sec. 5.1): 3x3 convolutions
with 64/128/256/512 channels at 32/16/8/4 spatial size.  Neither the datasets
nor trained weights are available here, so activations are ReLU(N(0,1)) (what a
post-ReLU feature map looks like to a quantizer: non-negative, sparse-ish, with
a long tail) and weights are Kaiming-normal N(0, sqrt(2 / (9 Cin))).
"""
from dataclasses import dataclass

import numpy as np

SEED_BASE = 200210711 * 1000


@dataclass(frozen=True)
class Layer:
    """One 3x3 convolution problem."""
    name: str
    N: int
    C: int
    K: int
    H: int
    W: int
    m: int = 4            # Winograd output tile (ignored when stride == 2)
    stride: int = 1
    pad: int = 1
    dtype: str = "i8"     # "i8", "f32", "i16" or "i8w16" (see STAGE_QMAX)
    relu_input: bool = True
    flex_sigma: float = 0.0   # std of the noise added to B^T, G, A^T ("flex" transforms)
    seed: int = 0

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - 3) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - 3) // self.stride + 1

    @property
    def direct_ops(self):
        """Direct-convolution-equivalent operations: 2 N K Ho Wo C 9 (all nine taps counted)."""
        return 2 * self.N * self.K * self.Ho * self.Wo * self.C * 9


# Code ranges per quantizer (input x, transformed weights u, transformed input v, Hadamard
# stage m, output y) of the dtypes a Layer can name: "i8" is the paper's INT8 pipeline,
# "i16" its INT16 one (Sec. 5.1), "i8w16" 8-bit activations around a 16-bit Winograd domain
# (Sec. 3.2, one bit-width per stage).
STAGE_QMAX = {
    "i8": dict(x=127, u=127, v=127, m=127, y=127),
    "i16": dict(x=32767, u=32767, v=32767, m=32767, y=32767),
    "i8w16": dict(x=127, u=32767, v=32767, m=32767, y=127),
}


def _seed(config, layer):
    return SEED_BASE + 100 * config + layer


def config1():
    """Single tiny fp32 layer, F(2x2,3x3), N(0,1) data, no quantization."""
    return [Layer("cfg1", 1, 16, 16, 8, 8, m=2, dtype="f32", relu_input=False, seed=_seed(1, 0))]


def config2(dtype="i8", N=64):
    """ResNet-18 stage-1 conv: batch 64, 32x32, 64->64, F(4x4,3x3)."""
    return [Layer("cfg2_" + dtype, N, 64, 64, 32, 32, m=4, dtype=dtype, seed=_seed(2, 0))]


def config3(N=128):
    """Small-spatial, GEMM-dominated stage-3/4 convs, F2 and F4, int8."""
    out = []
    i = 0
    for (C, S) in ((256, 8), (512, 4)):
        for m in (2, 4):
            out.append(Layer("cfg3_c%d_s%d_F%d" % (C, S, m), N, C, C, S, S, m=m, seed=_seed(3, i)))
            i += 1
    return out


def config4(N=64):
    """Relaxed ("flex") transforms: F(6x6,3x3) matrices perturbed by N(0, 0.01)."""
    return [Layer("cfg4_flex_F6", N, 128, 128, 16, 16, m=6, flex_sigma=0.01, seed=_seed(4, 0))]


def config5(N=256):
    """The 16 3x3 convolutions of CIFAR ResNet-18 after the stem, as independent
    layer problems.  Stride-1 layers get a Winograd tile m drawn from {2,4,6} by
    the seed; the three stride-2 layers go to the im2row baseline."""
    rng = np.random.default_rng(_seed(5, 99))
    spec = []
    for (C, S) in ((64, 32),):
        spec += [(C, C, S, 1)] * 4
    for (Cin, C, S) in ((64, 128, 32), (128, 256, 16), (256, 512, 8)):
        spec += [(Cin, C, S, 2)] + [(C, C, S // 2, 1)] * 3
    out = []
    for i, (Cin, Cout, S, stride) in enumerate(spec):
        m = int(rng.choice([2, 4, 6])) if stride == 1 else 0
        out.append(Layer("cfg5_l%02d_%dto%d_s%d_%s" % (i, Cin, Cout, S,
                                                        ("F%d" % m) if stride == 1 else "im2row"),
                         N, Cin, Cout, S, S, m=m, stride=stride, seed=_seed(5, i)))
    return out


def make_inputs(layer):
    """X [N,C,H,W] fp32 and g [K,C,3,3] fp32 for a layer, from its seed."""
    rng = np.random.default_rng(layer.seed)
    X = rng.standard_normal((layer.N, layer.C, layer.H, layer.W), dtype=np.float32)
    if layer.relu_input:
        np.maximum(X, 0, out=X)
    if layer.relu_input:
        std = np.float32(np.sqrt(2.0 / (9.0 * layer.C)))
    else:
        std = np.float32(1.0)
    g = rng.standard_normal((layer.K, layer.C, 3, 3), dtype=np.float32) * std
    return X, g


def input_codes(X, s_x, qmax=127, container=np.int8):
    """Integer codes a layer receives from the layer before it: round(X / s_x) in fp32, ties
    to even, clipped to [-qmax, qmax].  Input preparation only (the path starts from these
    codes); the one place the benchmark takes them from."""
    v = np.asarray(X, np.float32) / np.float32(s_x)
    return np.clip(np.rint(v), -qmax, qmax).astype(container)


def perturb_transforms(BT, G, AT, sigma, seed):
    """Add seeded N(0, sigma) noise to every entry of the three matrices and round
    to fp32 -- stands in for learned ("flex") transforms, which are dense."""
    rng = np.random.default_rng(seed + 7)
    out = []
    for Mx in (BT, G, AT):
        Mx = np.asarray(Mx, np.float64)
        out.append((Mx + sigma * rng.standard_normal(Mx.shape)).astype(np.float32))
    return tuple(out)
