"""Seeded synthetic inputs and the benchmark configurations.

This module only draws numbers and names shapes.  It holds none of the method's
arithmetic and is the one module that both the HIP path's callers (tests,
bench) and the CPU oracle's callers may import.

The paper measured on MNIST / CIFAR-10 networks (Sec. IV); homomorphic cost does
not depend on the data, so uniform values mod p with the paper's shapes stand in
for the trained weights and images.
"""
from dataclasses import dataclass

import numpy as np

# Parameter set of Sec. IV ("Evaluation"): n = 2048 slots, 60-bit q, 20-bit p.
# p is the largest prime below 2^20 with p = 1 (mod 2n); q is the largest prime
# below 2^60 with q = 1 (mod 2n * p), so that (q-1)/p is an integer.
N = 2048
P = 1032193
Q = 1152921500113727489
GADGET_BITS = 20           # key-switching digits of 20 bits -> 3 digits
SIGMA = 3.2
# Optional second prime used only inside key switching (keys modulo q * SPECIAL, exact division by SPECIAL
# at the end): the largest prime below 2^60 that is 1 (mod 2n); it differs from q.  With it a rotation adds
# almost no noise, which is what lets 3x3 convolutions decrypt at the 20-bit p of Sec. IV.
SPECIAL = 1152921504606830593


@dataclass(frozen=True)
class Params:
    n: int = N
    q: int = Q
    p: int = P
    gadget_bits: int = GADGET_BITS
    special: int = 0           # 0: one-prime key switching


DEFAULT = Params()
# With the special prime the digit width no longer drives the rotation noise (digits * error / P is far below 1
# even for 30-bit digits), so two digits are enough; fewer digits mean fewer transforms per rotation.
DEFAULT_SPECIAL = Params(special=SPECIAL, gadget_bits=30)


@dataclass(frozen=True)
class FcShape:
    name: str
    n_o: int
    n_i: int
    batch: int


@dataclass(frozen=True)
class ConvShape:
    name: str
    c_o: int
    c_i: int
    k_h: int
    k_w: int
    u_h: int
    u_w: int
    batch: int

    @property
    def tuple(self):
        return (self.c_o, self.c_i, self.k_h, self.k_w, self.u_h, self.u_w)


# the five benchmark configurations
FC_16x128 = FcShape("fc_16x128_b1", 16, 128, 1)
FC_128x1024 = FcShape("fc_128x1024_b64", 128, 1024, 64)
FC_1000x2048 = FcShape("fc_1000x2048_b64", 1000, 2048, 64)
CONV_16x16_128_3x3 = ConvShape("conv_16x16x128_3x3x128_b16", 128, 128, 3, 3, 16, 16, 16)


def uniform_mod(p, shape, seed):
    """Uniform integers in [0,p) as uint64, from numpy's PCG64 seeded with ``seed``."""
    return np.random.default_rng(seed).integers(0, p, size=shape, dtype=np.uint64)


def fc_inputs(shape, p=P, seed=0):
    """W (n_o x n_i), x (batch x n_i), r (batch x n_o), all uniform mod p."""
    W = uniform_mod(p, (shape.n_o, shape.n_i), [seed, 1])
    x = uniform_mod(p, (shape.batch, shape.n_i), [seed, 2])
    r = uniform_mod(p, (shape.batch, shape.n_o), [seed, 3])
    return W, x, r


def conv_inputs(shape, p=P, seed=0):
    """K (c_o x c_i x k_h x k_w), x (batch x c_i x u_h x u_w), r (batch x c_o x u_h x u_w)."""
    K = uniform_mod(p, (shape.c_o, shape.c_i, shape.k_h, shape.k_w), [seed, 1])
    x = uniform_mod(p, (shape.batch, shape.c_i, shape.u_h, shape.u_w), [seed, 2])
    r = uniform_mod(p, (shape.batch, shape.c_o, shape.u_h, shape.u_w), [seed, 3])
    return K, x, r


def find_prime_below(limit, modulus):
    """Largest prime below ``limit`` that is 1 modulo ``modulus`` (test parameter sets)."""
    k = (limit - 2) // modulus
    while k > 0 and not _is_prime(k * modulus + 1):
        k -= 1
    return k * modulus + 1


def _is_prime(v):
    if v < 2:
        return False
    small = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37)
    for s in small:
        if v % s == 0:
            return v == s
    d, r = v - 1, 0
    while d % 2 == 0:
        d //= 2
        r += 1
    for a in small:      # deterministic for v < 3.3e24
        x = pow(a, d, v)
        if x in (1, v - 1):
            continue
        for _ in range(r - 1):
            x = x * x % v
            if x == v - 1:
                break
        else:
            return False
    return True


@dataclass(frozen=True)
class ConvLayer:
    """One convolution of a network: c_o kernels of k x k over c_i channels of an in_hw x in_hw image."""
    name: str
    c_o: int
    c_i: int
    k: int
    stride: int
    in_hw: int


def resnet18_layers():
    """The 20 convolutions and the final FC of an ImageNet-shaped ResNet-18 (random weights stand in for a
    trained network): conv1 7x7/2 on 224x224, four stages of two basic blocks at 64/128/256/512 channels on
    56/28/14/7 pixels, 1x1/2 downsample convolutions at the stage transitions, FC 512 -> 1000."""
    layers = [ConvLayer("conv1", 64, 3, 7, 2, 224)]
    layers += [ConvLayer(f"layer1.{b}.conv{c}", 64, 64, 3, 1, 56) for b in (0, 1) for c in (1, 2)]
    ch_in, hw = 64, 56
    for stage, ch in ((2, 128), (3, 256), (4, 512)):
        layers.append(ConvLayer(f"layer{stage}.0.conv1", ch, ch_in, 3, 2, hw))
        layers.append(ConvLayer(f"layer{stage}.0.downsample", ch, ch_in, 1, 2, hw))
        hw //= 2
        layers += [ConvLayer(f"layer{stage}.0.conv2", ch, ch, 3, 1, hw),
                   ConvLayer(f"layer{stage}.1.conv1", ch, ch, 3, 1, hw),
                   ConvLayer(f"layer{stage}.1.conv2", ch, ch, 3, 1, hw)]
        ch_in = ch
    return layers, FcShape("fc_1000x512_b1", 1000, 512, 1)
