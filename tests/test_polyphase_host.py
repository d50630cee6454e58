"""Stride as a polyphase split: the oracle's rearrangement against the written-out definition of a strided
convolution, and the library's host helpers against the oracle's (no GPU)."""
import numpy as np
import pytest

from oracle.oracle import polyphase_split, strided_conv_plain
from paper_2105_01827_amd import binding, workloads as wl

P = 257
CASES = [
    # c_o, c_i, k_h, k_w, stride, H, W
    (2, 3, 3, 3, 2, 8, 8), (2, 2, 7, 7, 2, 10, 12), (3, 2, 1, 1, 2, 9, 5), (2, 2, 3, 3, 2, 7, 9),
    (2, 1, 3, 5, 3, 10, 11), (1, 2, 3, 3, 4, 9, 9), (2, 2, 5, 3, 1, 6, 6), (1, 1, 1, 3, 3, 7, 7),
]


def _inputs(case):
    co, ci, kh, kw, s, H, W = case
    rng = np.random.default_rng(sum(case))
    return (rng.integers(1, P, size=(co, ci, kh, kw), dtype=np.uint64),
            rng.integers(1, P, size=(ci, H, W), dtype=np.uint64))


@pytest.mark.parametrize("case", CASES)
def test_polyphase_split_reproduces_the_strided_definition(case):
    K, x = _inputs(case)
    s = case[4]
    Kp, xp = polyphase_split(K, x, s)
    assert Kp.shape[2] % 2 == 1 and Kp.shape[3] % 2 == 1
    assert np.count_nonzero(Kp) == K.size and sorted(Kp[Kp != 0].tolist()) == sorted(K.ravel().tolist())
    want = strided_conv_plain(K, x, P, s)
    assert np.array_equal(strided_conv_plain(Kp, xp, P, 1), want)
    # stride 1 of the same definition, subsampled, is the same thing (the other way this build evaluates stride)
    assert np.array_equal(strided_conv_plain(K, x, P, 1)[:, ::s, ::s], want)


def test_strided_definition_on_a_hand_computed_case():
    """1 x 1 x 3 x 3 kernel of ones on a 4 x 4 image of ones, stride 2: window sums at (0,0),(0,2),(2,0),(2,2)
    with zero padding are 4, 6, 6, 9."""
    K = np.ones((1, 1, 3, 3), np.uint64)
    x = np.ones((1, 4, 4), np.uint64)
    assert strided_conv_plain(K, x, 1000, 2).tolist() == [[[4, 6], [6, 9]]]


@pytest.mark.parametrize("case", CASES + [(2, 3, 7, 7, 2, 16, 16), (2, 2, 3, 3, 8, 17, 9)])
def test_library_helpers_agree_with_the_oracle(case):
    co, ci, kh, kw, s, H, W = case
    K, x = _inputs(case)
    par = wl.DEFAULT
    ctx = binding.Context(par.n, par.q, par.p, par.gadget_bits)
    pp = ctx.conv_polyphase(ci, H, W, kh, kw, s)
    Kp, xp = polyphase_split(K, x, s)
    assert (pp.c_i_poly, pp.k_h_poly, pp.k_w_poly, pp.out_h, pp.out_w) == (Kp.shape[1], Kp.shape[2], Kp.shape[3],
                                                                          xp.shape[1], xp.shape[2])
    assert np.array_equal(ctx.polyphase_kernel(pp, K), Kp)
    assert np.array_equal(ctx.polyphase_input(pp, x), xp)


def test_resnet_shapes():
    """7x7/2 keeps four phases with a 5x5 window, 3x3/2 four phases with 3x3, 1x1/2 one phase with 1x1."""
    ctx = binding.Context(wl.DEFAULT.n, wl.DEFAULT.q, wl.DEFAULT.p, wl.DEFAULT.gadget_bits)
    for (k, hw, ci), want in {(7, 224, 3): (12, 5, 112), (3, 56, 64): (256, 3, 28), (1, 56, 64): (64, 1, 28)}.items():
        pp = ctx.conv_polyphase(ci, hw, hw, k, k, 2)
        assert (pp.c_i_poly, pp.k_h_poly, pp.out_h) == want
    lib = binding.load()
    assert lib.gala_conv_polyphase_plan(1, 8, 8, 3, 3, 9, None) != 0
    pp = binding.ConvPolyphase()
    assert lib.gala_conv_polyphase_plan(1, 8, 8, 3, 3, 9, pp) != 0       # stride beyond 8
    assert lib.gala_conv_polyphase_plan(1, 8, 8, 2, 3, 2, pp) != 0       # even kernel
