"""Seeded synthetic inputs for the secure-layer hot path.

This module holds no protocol arithmetic: it draws random words, encodes
real-valued tensors in 16-bit fixed point, splits values into two additive (or
XOR) shares, and lays out offline material (Beaver triples, A2B masks, B2A bits)
so that the relations the online phase relies on hold.  A matrix or convolution
triple needs C = A*B over the ring; that product is supplied by the caller as a
callable, so tests hand in the CPU oracle's plain product and the benchmark hands
in the device dealer's.  The same arrays are given to whichever implementation
is under test, so "same seed" means "same bytes".

The workloads are synthetic stand-ins for the paper's evaluation models (VGG16,
ResNet-50, one Transformer encoder layer; Sec. 5.3): only shapes and value
distributions matter to the hot path, so no dataset or trained weight is used.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

U64 = np.uint64
FRAC_BITS = 16
BASE_SEED = 220913643
N_AND_TRIPLES = 12  # 1 initial generate + 2 per prefix level, last level needs only 1


def rng_for(config_index: int, *stream: int) -> np.random.Generator:
    """Independent generator for (config, sub-stream...)."""
    return np.random.default_rng(np.random.SeedSequence([BASE_SEED + config_index, *stream]))


def rand_words(rng, shape) -> np.ndarray:
    return rng.integers(0, 1 << 64, size=shape, dtype=U64)


def encode_fixed(v, frac_bits: int = FRAC_BITS) -> np.ndarray:
    """Real tensor -> two's-complement ring elements, round to nearest."""
    return np.rint(np.asarray(v, dtype=np.float64) * float(1 << frac_bits)).astype(np.int64).view(U64)


def normal_fixed(rng, shape, std: float) -> np.ndarray:
    return encode_fixed(rng.standard_normal(shape) * std)


def share_additive(rng, value):
    """(s0, s1) with s0 uniform and s0 + s1 = value mod 2^64."""
    value = np.asarray(value, dtype=U64)
    s0 = rand_words(rng, value.shape)
    return s0, value - s0


def share_xor(rng, value):
    value = np.asarray(value, dtype=U64)
    s0 = rand_words(rng, value.shape)
    return s0, value ^ s0


def deal_product_triple(rng, a_shape, b_shape, product):
    """Additively shared (A, B, C) with C = product(A, B); A, B uniform."""
    A = rand_words(rng, a_shape); B = rand_words(rng, b_shape)
    C = np.asarray(product(A, B), dtype=U64)
    return share_additive(rng, A), share_additive(rng, B), share_additive(rng, C)


def deal_relu_material(rng, n: int) -> dict:
    """Offline material for n secure-ReLU elements; every value a (party0, party1) pair.

    r        A2B masks, n words
    and_a/b/c  [12, n] XOR-shared AND triples (c = a & b after XOR-reconstruction)
    rb, ra   XOR-shared random bit (uint8) and additive shares of the same bit
    ma/mb/mc element-wise multiplication triple for the select step
    """
    m = {}
    m["r"] = (rand_words(rng, n), rand_words(rng, n))
    a = (rand_words(rng, (N_AND_TRIPLES, n)), rand_words(rng, (N_AND_TRIPLES, n)))
    b = (rand_words(rng, (N_AND_TRIPLES, n)), rand_words(rng, (N_AND_TRIPLES, n)))
    m["and_a"], m["and_b"] = a, b
    m["and_c"] = share_xor(rng, (a[0] ^ a[1]) & (b[0] ^ b[1]))
    rb = (rng.integers(0, 2, size=n, dtype=np.uint8), rng.integers(0, 2, size=n, dtype=np.uint8))
    m["rb"] = rb
    m["ra"] = share_additive(rng, (rb[0] ^ rb[1]).astype(U64))
    ma = (rand_words(rng, n), rand_words(rng, n)); mb = (rand_words(rng, n), rand_words(rng, n))
    m["ma"], m["mb"] = ma, mb
    m["mc"] = share_additive(rng, (ma[0] + ma[1]) * (mb[0] + mb[1]))
    return m


# ---------------------------------------------------------------- three parties
N_AND_TRIPLES3 = 13  # majority of the carry-save step + the 12 of the two-addend adder


def share_additive3(rng, value):
    """(s0, s1, s2) with s0, s1 uniform and s0 + s1 + s2 = value mod 2^64."""
    value = np.asarray(value, dtype=U64)
    s0 = rand_words(rng, value.shape); s1 = rand_words(rng, value.shape)
    return s0, s1, value - s0 - s1


def share_xor3(rng, value):
    value = np.asarray(value, dtype=U64)
    s0 = rand_words(rng, value.shape); s1 = rand_words(rng, value.shape)
    return s0, s1, value ^ s0 ^ s1


def deal_product_triple3(rng, a_shape, b_shape, product):
    A = rand_words(rng, a_shape); B = rand_words(rng, b_shape)
    C = np.asarray(product(A, B), dtype=U64)
    return share_additive3(rng, A), share_additive3(rng, B), share_additive3(rng, C)


def deal_trunc3_pair(rng, shape, bits: int = FRAC_BITS):
    """Offline pair of the three-party rescale: shares of r uniform in [0, 2^63) and of r >> bits."""
    r = rng.integers(0, 1 << 63, size=shape, dtype=U64)
    return share_additive3(rng, r), share_additive3(rng, r >> U64(bits))


def deal_relu3_material(rng, n: int) -> dict:
    """Offline material for n three-party ReLU elements; every value a (party 0, 1, 2) triple.

    r0, r1   A2B masks party j sends to party j+1 / j+2 (mod 3), n words each
    and_a/b/c  [13, n] XOR-shared AND triples
    rb, ra   XOR-shared random bit (uint8) and additive shares of the same bit
    ma/mb/mc element-wise multiplication triple for the select step
    """
    m = {}
    m["r0"] = tuple(rand_words(rng, n) for _ in range(3))
    m["r1"] = tuple(rand_words(rng, n) for _ in range(3))
    A = rand_words(rng, (N_AND_TRIPLES3, n)); B = rand_words(rng, (N_AND_TRIPLES3, n))
    m["and_a"] = share_xor3(rng, A); m["and_b"] = share_xor3(rng, B); m["and_c"] = share_xor3(rng, A & B)
    bit = rng.integers(0, 2, size=n, dtype=np.uint8)
    b0 = rng.integers(0, 2, size=n, dtype=np.uint8); b1 = rng.integers(0, 2, size=n, dtype=np.uint8)
    m["rb"] = (b0, b1, bit ^ b0 ^ b1)
    m["ra"] = share_additive3(rng, bit.astype(U64))
    MA = rand_words(rng, n); MB = rand_words(rng, n)
    m["ma"] = share_additive3(rng, MA); m["mb"] = share_additive3(rng, MB); m["mc"] = share_additive3(rng, MA * MB)
    return m


# ------------------------------------------------------------------- workloads
@dataclass
class Gemm:
    """One Beaver GEMM: X[M,K] ~ N(0, x_std^2), W[K,N] ~ N(0, w_std^2)."""
    name: str
    M: int
    K: int
    N: int
    x_std: float
    w_std: float
    batch: int = 1
    relu: bool = False
    repeat: int = 1       # how many layers of this shape the model has (benchmark tables only)


@dataclass
class Conv:
    """One Beaver convolution, NHWC input, [KH,KW,Cin,Cout] filter."""
    name: str
    B: int
    H: int
    W: int
    Cin: int
    Cout: int
    KH: int = 3
    KW: int = 3
    pad: int = 1
    stride: int = 1
    x_std: float = 1.0
    w_std: float = 1.0
    relu: bool = True
    pool: bool = False
    repeat: int = 1

    @property
    def Ho(self): return (self.H + 2 * self.pad - self.KH) // self.stride + 1
    @property
    def Wo(self): return (self.W + 2 * self.pad - self.KW) // self.stride + 1
    @property
    def gemm_mkn(self): return (self.B * self.Ho * self.Wo, self.KH * self.KW * self.Cin, self.Cout)


@dataclass
class Workload:
    index: int
    name: str
    layers: list = field(default_factory=list)


def he_std(fan_in: int) -> float:
    return float(np.sqrt(2.0 / fan_in))


def config_tiny() -> Workload:
    # X[64x256] ~ N(0,1), W[256x128] ~ N(0, 1/256) (second argument read as variance)
    return Workload(0, "tiny-secure-layer",
                    [Gemm("fc", 64, 256, 128, 1.0, 1.0 / 16.0, relu=True)])


def config_vgg_block() -> Workload:
    # batch 64, 128x16x16, 3x3 conv 128->128, weights N(0, 2/(9*128)) (variance)
    return Workload(1, "vgg16-cifar-conv-block",
                    [Conv("conv3x3", 64, 16, 16, 128, 128, x_std=1.0, w_std=he_std(9 * 128))])


def config_resnet_bottleneck() -> Workload:
    # 56x56, batch 32: 1x1 256->64, 3x3 64->64, 1x1 64->256; no batch-norm, no residual
    return Workload(2, "resnet50-bottleneck-56",
                    [Conv("conv1x1a", 32, 56, 56, 256, 64, 1, 1, 0, 1, 1.0, he_std(256)),
                     Conv("conv3x3", 32, 56, 56, 64, 64, 3, 3, 1, 1, 1.0, he_std(9 * 64)),
                     Conv("conv1x1b", 32, 56, 56, 64, 256, 1, 1, 0, 1, 1.0, he_std(64))])


def config_transformer() -> Workload:
    # BERT-base: batch 8, seq 512, hidden 768, 12 heads; weights N(0, 0.02) read as std
    T, H, A, dh = 8 * 512, 768, 12, 64
    return Workload(3, "bert-base-encoder-linear-path",
                    [Gemm("qkv", T, H, 3 * H, 1.0, 0.02),
                     Gemm("qk^t", 512, dh, 512, 1.0, 1.0, batch=8 * A),
                     Gemm("av", 512, 512, dh, 1.0, 1.0, batch=8 * A),
                     Gemm("out", T, H, H, 1.0, 0.02),
                     Gemm("ffn1", T, H, 4 * H, 1.0, 0.02, relu=True),
                     Gemm("ffn2", T, 4 * H, H, 1.0, 0.02)])


VGG16_CIFAR = [(3, 64, False), (64, 64, True), (64, 128, False), (128, 128, True),
               (128, 256, False), (256, 256, False), (256, 256, True),
               (256, 512, False), (512, 512, False), (512, 512, True),
               (512, 512, False), (512, 512, False), (512, 512, True)]


def config_vgg16_pipeline(micro_batch: int = 32) -> Workload:
    # full VGG16 for 32x32x3 inputs, one micro-batch; 2x2 max-pool after the flagged convs
    layers, hw = [], 32
    for i, (cin, cout, pool) in enumerate(VGG16_CIFAR):
        layers.append(Conv(f"conv{i + 1}", micro_batch, hw, hw, cin, cout,
                           x_std=1.0, w_std=he_std(9 * cin), relu=True, pool=pool))
        if pool:
            hw //= 2
    layers += [Gemm("fc1", micro_batch, 512, 512, 1.0, he_std(512), relu=True),
               Gemm("fc2", micro_batch, 512, 512, 1.0, he_std(512), relu=True),
               Gemm("fc3", micro_batch, 512, 10, 1.0, he_std(512))]
    return Workload(4, "vgg16-cifar-inter-batch-pipeline", layers)


# ---- the models of the paper's own evaluation (Sec. 5.2), layer shapes only --------------
def config_paper_transformer(batch: int = 8) -> Workload:
    # one encoder layer, H = 1024, A = 16, sequence length 512 (the BERT-large configuration)
    T, H, A, dh = batch * 512, 1024, 16, 64
    return Workload(5, "paper-transformer-encoder-h1024-a16",
                    [Gemm("qkv", T, H, 3 * H, 1.0, 0.02),
                     Gemm("qk^t", 512, dh, 512, 1.0, 1.0, batch=batch * A),
                     Gemm("av", 512, 512, dh, 1.0, 1.0, batch=batch * A),
                     Gemm("out", T, H, H, 1.0, 0.02),
                     Gemm("ffn1", T, H, 4 * H, 1.0, 0.02, relu=True),
                     Gemm("ffn2", T, 4 * H, H, 1.0, 0.02)])


def config_vgg16_imagenet(batch: int = 2) -> Workload:
    # VGG16 on 224x224x3 inputs: the CIFAR channel plan at ImageNet resolution, 25088-4096-4096-1000 head
    layers, hw = [], 224
    for i, (cin, cout, pool) in enumerate(VGG16_CIFAR):
        layers.append(Conv(f"conv{i + 1}", batch, hw, hw, cin, cout,
                           x_std=1.0, w_std=he_std(9 * cin), relu=True, pool=pool))
        if pool:
            hw //= 2
    layers += [Gemm("fc1", batch, 512 * 7 * 7, 4096, 1.0, he_std(512 * 49), relu=True),
               Gemm("fc2", batch, 4096, 4096, 1.0, he_std(4096), relu=True),
               Gemm("fc3", batch, 4096, 1000, 1.0, he_std(4096))]
    return Workload(6, "paper-vgg16-imagenet", layers)


def config_resnet50_imagenet(batch: int = 2) -> Workload:
    # ResNet-50 on 224x224x3: every distinct convolution shape with its multiplicity
    # (no batch-norm, no residual adds, the 3x3 max-pool after conv1 left out: shapes only)
    def c(name, hw, cin, cout, k, stride, repeat=1, relu=True):
        return Conv(name, batch, hw, hw, cin, cout, k, k, k // 2, stride, 1.0, he_std(k * k * cin), relu, False, repeat)
    layers = [c("conv1_7x7s2", 224, 3, 64, 7, 2)]
    hw, cin = 56, 64
    for stage, (mid, blocks) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)], start=2):
        out = 4 * mid
        s = 1 if stage == 2 else 2
        layers += [c(f"s{stage}_first_1x1a", hw, cin, mid, 1, 1),
                   c(f"s{stage}_first_3x3", hw, mid, mid, 3, s),
                   c(f"s{stage}_down_1x1", hw, cin, out, 1, s, relu=False)]
        hw //= s
        layers += [c(f"s{stage}_1x1b", hw, mid, out, 1, 1, repeat=blocks),
                   c(f"s{stage}_1x1a", hw, out, mid, 1, 1, repeat=blocks - 1),
                   c(f"s{stage}_3x3", hw, mid, mid, 3, 1, repeat=blocks - 1)]
        cin = out
    layers.append(Gemm("fc", batch, 2048, 1000, 1.0, he_std(2048)))
    return Workload(7, "paper-resnet50-imagenet", layers)


PAPER_MODELS = [config_paper_transformer, config_vgg16_imagenet, config_resnet50_imagenet]

CONFIGS = [config_tiny, config_vgg_block, config_resnet_bottleneck, config_transformer,
           config_vgg16_pipeline]
