"""Layer shapes of the five synthetic workloads.

Pure shape bookkeeping: no arithmetic of the convolution method lives here. The shapes are
ImageNet-scale CNN layers (a NIN mlpconv block, a GoogLeNet-style inception module, an
AlexNet-shaped conv stack and a GoogLeNet stem) for one GPU's share of a data-parallel
minibatch (paper section 3.4: every peer keeps a replica and works on its own batch share;
section 4: batch 128 per GPU).
"""
from dataclasses import dataclass


@dataclass(frozen=True)
class ConvLayer:
    name: str
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int
    pad: int
    dtype: str = "f32"  # "f32" or "bf16": type of x, w, b, dy (dw, db are always f32)

    @property
    def P(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def x_shape(self):
        return (self.N, self.C, self.H, self.W)

    @property
    def w_shape(self):
        return (self.K, self.C, self.R, self.S)

    @property
    def y_shape(self):
        return (self.N, self.K, self.P, self.Q)

    @property
    def flop_per_pass(self):
        """Dense convention: padded taps count."""
        return 2 * self.N * self.K * self.C * self.R * self.S * self.P * self.Q

    def with_batch(self, n):
        return ConvLayer(self.name, n, self.C, self.H, self.W, self.K, self.R, self.S,
                         self.stride, self.pad, self.dtype)


def _L(name, N, C, HW, K, RS, s, p, dtype="f32"):
    return ConvLayer(name, N, C, HW, HW, K, RS, RS, s, p, dtype)


# config index -> list of conv layers (the FLOP-carrying operators of each workload)
CONV_LAYERS = {
    1: [_L("conv", 2, 3, 16, 8, 3, 1, 1)],
    2: [_L("conv1", 64, 3, 224, 96, 11, 4, 0),
        _L("cccp1", 64, 96, 54, 96, 1, 1, 0),
        _L("cccp2", 64, 96, 54, 96, 1, 1, 0)],
    3: [_L("b1_1x1", 128, 192, 28, 64, 1, 1, 0),
        _L("b2_reduce", 128, 192, 28, 96, 1, 1, 0),
        _L("b2_3x3", 128, 96, 28, 128, 3, 1, 1),
        _L("b3_reduce", 128, 192, 28, 16, 1, 1, 0),
        _L("b3_5x5", 128, 16, 28, 32, 5, 1, 2),
        _L("b4_proj", 128, 192, 28, 32, 1, 1, 0)],
    4: [_L("conv1", 128, 3, 227, 96, 11, 4, 0),
        _L("conv2", 128, 96, 27, 256, 5, 1, 2),
        _L("conv3", 128, 256, 13, 384, 3, 1, 1),
        _L("conv4", 128, 384, 13, 384, 3, 1, 1),
        _L("conv5", 128, 384, 13, 256, 3, 1, 1)],
    5: [_L("stem7x7", 256, 3, 224, 64, 7, 2, 3, "bf16"),
        _L("c1x1", 256, 64, 56, 64, 1, 1, 0, "bf16"),
        _L("c3x3", 256, 64, 56, 192, 3, 1, 1, "bf16")],
}

WORKLOAD_NAMES = {
    1: "cfg1_single_conv3x3_f32_n2",
    2: "cfg2_nin_mlpconv_f32_n64",
    3: "cfg3_inception_f32_n128",
    4: "cfg4_alexnet_conv_stack_f32_n128",
    5: "cfg5_googlenet_stem_bf16_n256",
}


def total_flop(cfg):
    """fwd + bwd-data + bwd-weight over every conv layer of the config."""
    return 3 * sum(l.flop_per_pass for l in CONV_LAYERS[cfg])
