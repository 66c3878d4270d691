"""Layer shapes of the synthetic workloads (no arithmetic).

VGG-16 / ResNet-50 / Inception-v3-style / wide-ResNet-101-2 layer lists stand in for the
models the paper trains (paper, Table 1: VGG-16 at 3x224x224; Inception-v3 at 3x299x299;
WRN-101-2 at 3x400x400; ResNet-50 at 224 is the smaller stand-in the parity configs name).  Per-GPU batch sizes are the
strong-scaling shards global_batch / g with g a power of two (paper, section 6
"Restricting GPU counts to powers of two").
"""
from collections import namedtuple

Conv = namedtuple("Conv", "name h w c k r s sh sw ph pw bias count")
Linear = namedtuple("Linear", "name in_f out_f bias")

GLOBAL_BATCH = 32
BATCHES = (1, 2, 4, 8, 16, 32)


def _c(name, hw, c, k, r=3, s=3, st=1, ph=None, pw=None, bias=True, count=1):
    ph = (r // 2) if ph is None else ph
    pw = (s // 2) if pw is None else pw
    return Conv(name, hw, hw, c, k, r, s, st, st, ph, pw, bias, count)


def vgg16_convs():
    cfg = [("conv1_1", 224, 3, 64), ("conv1_2", 224, 64, 64),
           ("conv2_1", 112, 64, 128), ("conv2_2", 112, 128, 128),
           ("conv3_1", 56, 128, 256), ("conv3_2", 56, 256, 256), ("conv3_3", 56, 256, 256),
           ("conv4_1", 28, 256, 512), ("conv4_2", 28, 512, 512), ("conv4_3", 28, 512, 512),
           ("conv5_1", 14, 512, 512), ("conv5_2", 14, 512, 512), ("conv5_3", 14, 512, 512)]
    return [_c(n, hw, c, k) for n, hw, c, k in cfg]


def vgg16_linears():
    return [Linear("fc6", 25088, 4096, True), Linear("fc7", 4096, 4096, True),
            Linear("fc8", 4096, 1000, True)]


def vgg16_param_count():
    n = 0
    for l in vgg16_convs():
        n += l.k * l.r * l.s * l.c + l.k
    for l in vgg16_linears():
        n += l.out_f * l.in_f + l.out_f
    return n


def resnet50_convs():
    """Unique conv shapes of ResNet-50 (stride 2 on the 3x3), with multiplicities."""
    L = [_c("stem7x7", 224, 3, 64, 7, 7, 2, 3, 3, bias=False)]
    def add(name, hw, c, k, r=1, st=1, count=1):
        L.append(_c(name, hw, c, k, r, r, st, r // 2, r // 2, bias=False, count=count))
    add("s1_1x1_64_64", 56, 64, 64)
    add("s1_3x3_64", 56, 64, 64, 3, 1, 3)
    add("s1_1x1_64_256", 56, 64, 256, count=4)
    add("s1_1x1_256_64", 56, 256, 64, count=2)
    add("s2_1x1_256_128", 56, 256, 128)
    add("s2_3x3_128_s2", 56, 128, 128, 3, 2)
    add("s2_1x1_128_512", 28, 128, 512, count=4)
    add("s2_proj_256_512_s2", 56, 256, 512, 1, 2)
    add("s2_1x1_512_128", 28, 512, 128, count=3)
    add("s2_3x3_128", 28, 128, 128, 3, 1, 3)
    add("s3_1x1_512_256", 28, 512, 256)
    add("s3_3x3_256_s2", 28, 256, 256, 3, 2)
    add("s3_1x1_256_1024", 14, 256, 1024, count=6)
    add("s3_proj_512_1024_s2", 28, 512, 1024, 1, 2)
    add("s3_1x1_1024_256", 14, 1024, 256, count=5)
    add("s3_3x3_256", 14, 256, 256, 3, 1, 5)
    add("s4_1x1_1024_512", 14, 1024, 512)
    add("s4_3x3_512_s2", 14, 512, 512, 3, 2)
    add("s4_1x1_512_2048", 7, 512, 2048, count=3)
    add("s4_proj_1024_2048_s2", 14, 1024, 2048, 1, 2)
    add("s4_1x1_2048_512", 7, 2048, 512, count=2)
    add("s4_3x3_512", 7, 512, 512, 3, 1, 2)
    return L


def wrn101_2_convs():
    """Unique conv shapes of a wide ResNet-101-2 at 400x400 input (the paper's second image model, Table 1):
    bottlenecks with doubled inner widths 128/256/512/1024, outputs 256/512/1024/2048, 3/4/23/3 blocks,
    stride 2 on the 3x3; spatial sizes 200 (stem) -> 100 -> 50 -> 25 -> 13."""
    L = [_c("stem7x7_400", 400, 3, 64, 7, 7, 2, 3, 3, bias=False)]
    def add(name, hw, c, k, r=1, st=1, count=1):
        L.append(_c(name, hw, c, k, r, r, st, r // 2, r // 2, bias=False, count=count))
    add("w1_1x1_64_128", 100, 64, 128)
    add("w1_3x3_128", 100, 128, 128, 3, 1, 3)
    add("w1_1x1_128_256", 100, 128, 256, count=3)
    add("w1_proj_64_256", 100, 64, 256)
    add("w1_1x1_256_128", 100, 256, 128, count=2)
    add("w2_1x1_256_256", 100, 256, 256)
    add("w2_3x3_256_s2", 100, 256, 256, 3, 2)
    add("w2_1x1_256_512", 50, 256, 512, count=4)
    add("w2_proj_256_512_s2", 100, 256, 512, 1, 2)
    add("w2_1x1_512_256", 50, 512, 256, count=3)
    add("w2_3x3_256", 50, 256, 256, 3, 1, 3)
    add("w3_1x1_512_512", 50, 512, 512)
    add("w3_3x3_512_s2", 50, 512, 512, 3, 2)
    add("w3_1x1_512_1024", 25, 512, 1024, count=23)
    add("w3_proj_512_1024_s2", 50, 512, 1024, 1, 2)
    add("w3_1x1_1024_512", 25, 1024, 512, count=22)
    add("w3_3x3_512", 25, 512, 512, 3, 1, 22)
    add("w4_1x1_1024_1024", 25, 1024, 1024)
    add("w4_3x3_1024_s2", 25, 1024, 1024, 3, 2)
    add("w4_1x1_1024_2048", 13, 1024, 2048, count=3)
    add("w4_proj_1024_2048_s2", 25, 1024, 2048, 1, 2)
    add("w4_1x1_2048_1024", 13, 2048, 1024, count=2)
    add("w4_3x3_1024", 13, 1024, 1024, 3, 1, 2)
    return L


def inception_convs():
    """Inception-v3-style asymmetric layers (channel pairs chosen inside the stated ranges)."""
    L = [
        Conv("3x3s2_299_3_32", 299, 299, 3, 32, 3, 3, 2, 2, 0, 0, False, 1),
        Conv("3x3_149_32_32", 149, 149, 32, 32, 3, 3, 1, 1, 0, 0, False, 1),
        Conv("3x3_147_32_64", 147, 147, 32, 64, 3, 3, 1, 1, 1, 1, False, 1),
        Conv("3x3_73_80_192", 73, 73, 80, 192, 3, 3, 1, 1, 0, 0, False, 1),
        Conv("3x3_35_64_96", 35, 35, 64, 96, 3, 3, 1, 1, 1, 1, False, 1),
        Conv("3x3_35_96_96", 35, 35, 96, 96, 3, 3, 1, 1, 1, 1, False, 1),
        Conv("3x3s2_35_288_384", 35, 35, 288, 384, 3, 3, 2, 2, 0, 0, False, 1),
    ]
    for c, k in ((128, 128), (160, 160), (192, 192), (128, 192)):
        L.append(Conv(f"1x7_17_{c}_{k}", 17, 17, c, k, 1, 7, 1, 1, 0, 3, False, 1))
        L.append(Conv(f"7x1_17_{c}_{k}", 17, 17, c, k, 7, 1, 1, 1, 3, 0, False, 1))
    L += [
        Conv("1x3_8_384_384", 8, 8, 384, 384, 1, 3, 1, 1, 0, 1, False, 1),
        Conv("3x1_8_384_384", 8, 8, 384, 384, 3, 1, 1, 1, 1, 0, False, 1),
        Conv("3x3_8_448_384", 8, 8, 448, 384, 3, 3, 1, 1, 1, 1, False, 1),
    ]
    return L


def out_hw(l):
    return (l.h + 2 * l.ph - l.r) // l.sh + 1, (l.w + 2 * l.pw - l.s) // l.sw + 1


def conv_flops(l, n):
    """Nominal flops of one pass (fwd, dgrad or wgrad): 2*M*K*R*S*C, padding taps counted."""
    ho, wo = out_hw(l)
    return 2.0 * n * ho * wo * l.k * l.r * l.s * l.c


def linear_flops(l, n):
    return 2.0 * n * l.in_f * l.out_f
