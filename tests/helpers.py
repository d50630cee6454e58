"""Small test-side utilities: independent big-integer references written with
Python ints / numpy object arrays (no oracle, no HIP code)."""
import numpy as np

from paper_2105_01827_amd import workloads as wl


def small_params(n, p_limit=None, p=None, gadget_bits=20):
    """A test parameter set for ring degree n: p = 1 mod 2n, 60-bit q = 1 mod 2n*p."""
    if p is None:
        p = wl.find_prime_below(p_limit or (1 << 20), 2 * n)
    assert p > 2 * n, "no prime p = 1 mod 2n below the limit"
    q = wl.find_prime_below(1 << 60, 2 * n * p)
    return wl.Params(n=n, q=q, p=p, gadget_bits=gadget_bits)


def negacyclic_mul(a, b, n, m):
    """(a*b) mod (X^n+1, m) through numpy's polynomial convolution on Python ints."""
    full = np.convolve(np.array([int(v) for v in a], dtype=object), np.array([int(v) for v in b], dtype=object))
    out = [0] * n
    for k, v in enumerate(full):
        if k < n:
            out[k] = (out[k] + v) % m
        else:
            out[k - n] = (out[k - n] - v) % m
    return np.array(out, dtype=np.uint64)


def poly_eval(a, x, m):
    """Horner evaluation of a(x) mod m with Python ints."""
    acc = 0
    for c in reversed([int(v) for v in a]):
        acc = (acc * x + c) % m
    return acc


def rotate_slots(v, step, swap=False):
    """Left rotation by ``step`` in both half-rows of a slot vector, rows swapped if asked."""
    v = np.asarray(v)
    h = len(v) // 2
    rows = [np.roll(v[:h], -step), np.roll(v[h:], -step)]
    if swap:
        rows = rows[::-1]
    return np.concatenate(rows)


def centred(v, q):
    v = int(v)
    return v - q if v > q // 2 else v


# Layer shapes drawn by a seeded generator: ragged sizes nobody picked by hand (odd channel counts, non-square
# images, 1 x k kernels).  The oracle is pinned on them by its decryption identities, the GPU library by the oracle.
def fc_shapes(count, seed):
    """(n, n_o, n_i, batch, special): padded sizes within what a plan accepts (n_i <= n; n_o <= n/2 when n_i fills the ring)."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        n = int(rng.choice([32, 64, 128, 256, 512]))
        n_i = int(rng.integers(1, n + 1))
        nip = 1 << (n_i - 1).bit_length()
        n_o = int(rng.integers(1, (n // 2 if nip == n else n) + 1))
        out.append((n, n_o, n_i, int(rng.integers(1, 5)), bool(rng.integers(0, 3) == 0)))
    return out


def conv_shapes(count, seed):
    """(n, shape, batch, matrix_cores, special): odd kernel sides, an image of at most n/2 pixels."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        n = int(rng.choice([32, 64, 128, 256, 512]))
        uh = int(rng.integers(1, 9))
        uw = int(rng.integers(1, 9))
        if uh * uw > n // 2:
            continue
        kh, kw = int(rng.choice([1, 3, 5])), int(rng.choice([1, 3, 5]))
        co, ci = int(rng.integers(1, 20)), int(rng.integers(1, 20))
        batch = int(rng.integers(1, 7))
        out.append((n, (co, ci, kh, kw, uh, uw), batch, bool(batch >= 2 and rng.integers(0, 2)),
                    bool(rng.integers(0, 3) == 0)))
    return out
