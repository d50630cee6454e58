"""Host-side spatial tiling and stride helpers of the library against plain numpy slicing (no GPU)."""
import numpy as np
import pytest

from paper_2105_01827_amd import binding, workloads as wl
from tests.helpers import small_params


def numpy_tile(image, oy, ox, th, tw):
    ch, H, W = image.shape
    out = np.zeros((ch, th, tw), np.uint64)
    for ty in range(th):
        for tx in range(tw):
            y, x = oy + ty, ox + tx
            if 0 <= y < H and 0 <= x < W:
                out[:, ty, tx] = image[:, y, x]
    return out


@pytest.mark.parametrize("n,in_h,in_w,k,stride", [
    (2048, 224, 224, 7, 2), (2048, 56, 56, 3, 1), (2048, 56, 56, 3, 2), (2048, 56, 56, 1, 2), (2048, 28, 28, 3, 2),
    (2048, 7, 7, 3, 1), (2048, 100, 20, 3, 1), (2048, 20, 100, 5, 3), (64, 12, 12, 3, 1), (64, 12, 12, 3, 2),
    (64, 9, 5, 3, 2), (256, 30, 17, 5, 1),
])
def test_tiles_cover_every_output_once_and_carry_their_neighbourhood(n, in_h, in_w, k, stride):
    par = small_params(n) if n != 2048 else wl.DEFAULT
    ctx = binding.Context(par.n, par.q, par.p, par.gadget_bits)
    t = ctx.conv_tiling(in_h, in_w, k, k, stride)
    assert t.tile_h * t.tile_w <= n // 2
    assert (t.out_h, t.out_w) == (-(-in_h // stride), -(-in_w // stride))
    rng = np.random.default_rng(in_h * in_w)
    ch = 2
    image = rng.integers(1, 1000, size=(ch, in_h, in_w), dtype=np.uint64)
    r = rng.integers(1, 1000, size=(ch, t.out_h, t.out_w), dtype=np.uint64)
    covered = np.zeros((ch, t.out_h, t.out_w), np.int64)
    stitched = np.zeros((ch, t.out_h, t.out_w), np.uint64)
    ph = k // 2
    for tile in range(t.tiles):
        oy = (tile // t.tiles_x) * t.step_y - t.halo_y
        ox = (tile % t.tiles_x) * t.step_x - t.halo_x
        got = ctx.tile_extract(t, image, tile)
        assert np.array_equal(got, numpy_tile(image, oy, ox, t.tile_h, t.tile_w))
        rt = ctx.tile_mask(t, r, tile)
        # identity "convolution" (copy of the centre pixel): scattering the tile itself must rebuild the subsampled image
        ctx.tile_scatter(t, got, tile, stitched)
        marks = np.zeros((ch, t.out_h, t.out_w), np.uint64)
        ctx.tile_scatter(t, np.ones_like(got), tile, marks)
        covered += marks.astype(np.int64)
        back = np.zeros((ch, t.out_h, t.out_w), np.uint64)
        ctx.tile_scatter(t, rt, tile, back)
        assert np.array_equal(back, r * marks)                       # the tile's mask is r on what it keeps
        assert np.array_equal(rt != 0, rt != 0) and int((rt != 0).sum()) == int(marks.sum())
        # every kept output has its whole k x k neighbourhood inside the tile (or outside the image)
        ys, xs = np.nonzero(marks[0])
        for yo, xo in zip(ys[:50], xs[:50]):
            y, x = yo * stride - oy, xo * stride - ox
            for dy in (-ph, ph):
                for dx in (-ph, ph):
                    inside_tile = 0 <= y + dy < t.tile_h and 0 <= x + dx < t.tile_w
                    inside_image = 0 <= yo * stride + dy < in_h and 0 <= xo * stride + dx < in_w
                    assert inside_tile or not inside_image
    assert np.all(covered == 1)
    assert np.array_equal(stitched, image[:, ::stride, ::stride])
