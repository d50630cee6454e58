"""GPU parity on layer shapes drawn by a seeded generator: he_fc and he_conv against the oracle, bit for bit.

The hand-picked shapes of test_gpu_parity.py cover the cases someone thought of; these cover ragged
sizes nobody picked (odd channel counts, non-square images, 1 x k kernels, batches that leave a column
tile of the matrix-core product partly empty).  Every output ciphertext of every case is recomputed by
the oracle, and the FC cases also decrypt to W x.  A third of the cases use special-prime keys; those
convolutions decrypt to the plain convolution as well.  The paper's two comparison schedules (hybrid
matrix-vector product, output-rotation convolution) run on drawn shapes of their own.
"""
import numpy as np
import pytest

from oracle.oracle import Oracle
from tests.helpers import conv_shapes, fc_shapes, small_params
from tests.test_gpu_parity import conv_case, fc_case, plain_conv, plain_matvec
from tests.test_gpu_special import with_special

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,n_o,n_i,batch,special", fc_shapes(60, seed=20210501))
def test_he_fc_on_drawn_shapes(n, n_o, n_i, batch, special):
    par = small_params(n)
    if special:
        par = with_special(par)
    ctx, o, plan, sk, W, x, r, got = fc_case(par, n_o, n_i, batch, list(range(batch)), seed=7 * n_o + n_i)
    for b in range(batch):
        share = plan.unpack_share(ctx.decrypt(sk, got[b]))
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_matvec(W, x[b], par.p))


@pytest.mark.parametrize("n,shape,batch,matrix_cores,special", conv_shapes(60, seed=20210502))
def test_he_conv_on_drawn_shapes(n, shape, batch, matrix_cores, special):
    par = small_params(n, p_limit=1 << 14, gadget_bits=4)
    if special:
        par = with_special(par)
    nout = Oracle(par.n, par.q, par.p, par.gadget_bits).conv_geometry(*shape)["nout"]
    ctx, o, plan, sk, K, x, r, got, cnt = conv_case(par, shape, batch, [(b, O) for b in range(batch) for O in range(nout)],
                                                    seed=n + shape[0], matrix_cores=matrix_cores)
    if not special:
        return
    co, ci, kh, kw, uh, uw = shape
    for b in range(batch):
        share = np.zeros((co, uh, uw), np.uint64)
        for O in range(plan.nout):
            plan.unpack_share(O, ctx.decrypt(sk, got[b, O]), share)
        assert np.array_equal((share + r[b]) % np.uint64(par.p), plain_conv(K, x[b], par.p))


# The paper's comparison schedules on drawn shapes (Sec. III-A(2), Sec. III-B(2)): ciphertexts equal the oracle's.
@pytest.mark.parametrize("n,n_o,n_i,batch,special", fc_shapes(30, seed=20210503))
def test_he_fc_hybrid_on_drawn_shapes(n, n_o, n_i, batch, special):
    from tests.test_gpu_gazelle import hybrid_case
    par = small_params(n, p_limit=1 << 14, gadget_bits=4)
    if special:
        par = with_special(par)
    hybrid_case(par, n_o, n_i, batch, list(range(batch)), seed=3 * n_o + n_i)


@pytest.mark.parametrize("n,shape,batch,matrix_cores,special", conv_shapes(30, seed=20210504))
def test_he_conv_outrot_on_drawn_shapes(n, shape, batch, matrix_cores, special):
    from tests.test_gpu_gazelle import outrot_case
    par = small_params(n, p_limit=1 << 14, gadget_bits=4)
    if special:
        par = with_special(par)
    nout = Oracle(par.n, par.q, par.p, par.gadget_bits).conv_geometry(*shape)["nout"]
    ctx, o, plan, sk, K, x, r, got, cnt, got_gala, cnt_gala = outrot_case(
        par, shape, batch, [(b, O) for b in range(batch) for O in range(nout)], seed=n + shape[1])
    # Table "Complexity comparison of convolution": c_i/c_n times GALA's Perms, everything else equal
    assert cnt["perm"] == plan.nin * cnt_gala["perm"]
    assert all(cnt[k] == cnt_gala[k] for k in ("decperm_in", "hstperm_in", "scmult", "add"))
