"""Layer shapes of the synthetic workloads (no data, no arithmetic of the method)."""
from dataclasses import dataclass


@dataclass(frozen=True)
class ConvShape:
    """One 2-D convolution: NHWC activations, KRSC filters, NPQK outputs.

    R is the filter height and S the filter width (cross-correlation, dilation 1,
    one group)."""
    N: int
    H: int
    W: int
    C: int
    K: int
    R: int
    S: int
    stride_h: int = 1
    stride_w: int = 1
    pad_h: int = 0
    pad_w: int = 0
    name: str = ""

    @property
    def P(self):
        return (self.H + 2 * self.pad_h - self.R) // self.stride_h + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad_w - self.S) // self.stride_w + 1

    @property
    def macs(self):
        return self.N * self.P * self.Q * self.K * self.C * self.R * self.S

    @property
    def ops(self):
        return 2 * self.macs

    def min_bytes(self, in_bytes=1, w_bytes=1, out_bytes=4):
        return (self.N * self.H * self.W * self.C * in_bytes
                + self.K * self.R * self.S * self.C * w_bytes
                + self.N * self.P * self.Q * self.K * out_bytes)

    def with_batch(self, n):
        d = dict(self.__dict__)
        d["N"] = n
        return ConvShape(**d)


def _c3(n, c, hw, name):
    return ConvShape(n, hw, hw, c, c, 3, 3, 1, 1, 1, 1, name)


def _c1(n, c, k, hw, name):
    return ConvShape(n, hw, hw, c, k, 1, 1, 1, 1, 0, 0, name)


# Small case the oracle finishes at once: values in [-8, 7].
CONFIG1 = [ConvShape(2, 16, 16, 16, 32, 3, 3, 1, 1, 1, 1, "cfg1_3x3_c16_k32")]

# ResNet-50-shaped 3x3 layers, batch 32.
CONFIG2 = [_c3(32, 64, 56, "3x3_c64_56"), _c3(32, 128, 28, "3x3_c128_28"),
           _c3(32, 256, 14, "3x3_c256_14"), _c3(32, 512, 7, "3x3_c512_7")]

# ResNet-50-shaped 1x1 bottleneck layers, batch 64 (memory bound).
CONFIG3 = [_c1(64, 64, 256, 56, "1x1_64_256_56"), _c1(64, 256, 64, 56, "1x1_256_64_56"),
           _c1(64, 512, 128, 28, "1x1_512_128_28"), _c1(64, 1024, 256, 14, "1x1_1024_256_14"),
           _c1(64, 2048, 512, 7, "1x1_2048_512_7")]

# fp16 3x3 layer, batch 16.
CONFIG4 = [_c3(16, 256, 28, "fp16_3x3_c256_28")]


def resnet50_layers(n=128):
    """The 53 convolution shapes of a ResNet-50 v1.5-style network at 224x224:
    a 7x7 stride-2 stem, 16 bottlenecks (1x1, 3x3, 1x1) with the stride on the
    3x3, and 4 projection 1x1 convolutions."""
    layers = [ConvShape(n, 224, 224, 3, 64, 7, 7, 2, 2, 3, 3, "stem")]
    h, in_c = 56, 64
    for stage, (mid, blocks, stride) in enumerate([(64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2)]):
        for b in range(blocks):
            s = stride if b == 0 else 1
            layers.append(ConvShape(n, h, h, in_c, mid, 1, 1, 1, 1, 0, 0, f"s{stage}b{b}.c1"))
            layers.append(ConvShape(n, h, h, mid, mid, 3, 3, s, s, 1, 1, f"s{stage}b{b}.c2"))
            h2 = (h + 2 - 3) // s + 1
            layers.append(ConvShape(n, h2, h2, mid, mid * 4, 1, 1, 1, 1, 0, 0, f"s{stage}b{b}.c3"))
            if b == 0:
                layers.append(ConvShape(n, h, h, in_c, mid * 4, 1, 1, s, s, 0, 0, f"s{stage}b{b}.ds"))
            in_c, h = mid * 4, h2
    return layers
