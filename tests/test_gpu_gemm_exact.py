"""Bit-exact GEMM parity: Eq. (3) and Eq. (10) on operands whose every partial sum is exact.

Weights are non-zero integers of magnitude at most 15 (stored exactly in bf16 / fp32) and every token
row holds at most four non-zero entries from {-2, -1, 1, 2}, placed so that over the tokens every
contraction index is hit.  Every product is an integer, every sum of at most four of them has magnitude
at most 120, so fp32 accumulation in any order is exact and the bf16 output (integers up to 256) is
exact: the kernels' outputs must EQUAL the float64 oracle, element for element.  One dropped, doubled
or misplaced product -- a wrong index nibble, a wrong slot, a wrong column of g(Y)[:, P], a row tile or
stage read from the wrong place -- changes some output by at least 1.

The shapes select every GEMM kernel family of the library in both directions (named beside each case),
with the permutation and with the identity.
"""
import numpy as np
import pytest

import oracle
import paper_2302_06058_amd as bm
from paper_2302_06058_amd import synth
from helpers import to_dev, i32_dev, words, from_dev_f64

pytestmark = pytest.mark.gpu


def int_weights(I, J, rng):
    mag = rng.integers(1, 16, size=(I, J))
    sign = rng.integers(0, 2, size=(I, J)) * 2 - 1
    return (mag * sign).astype(np.float32)


def sparse_rows(T, C, rng):
    """T x C, four non-zeros from {-2, -1, 1, 2} per row; the rows walk over all C columns in an order
    drawn once, so with 4 T >= C every column is non-zero in some row."""
    a = np.zeros((T, C), dtype=np.float32)
    order = rng.permutation(C)
    vals = np.array([-2, -1, 1, 2], dtype=np.float32)
    for q in range(4):
        cols = order[(4 * np.arange(T) + q) % C]
        a[np.arange(T), cols] = vals[rng.integers(0, 4, size=T)]
    return a


def exact_layer(I, J, T, N, M, dtype, seed, perm=True):
    import torch
    rng = np.random.default_rng(seed)
    Wh = synth.store(int_weights(I, J, rng), dtype)
    W64 = synth.to_f64(Wh, dtype)
    Xh = synth.store(sparse_rows(T, J, rng), dtype)
    dYh = synth.store(sparse_rows(T, I, rng), dtype)
    assert (Xh != 0).any(axis=0).all() and (dYh != 0).any(axis=0).all()      # every contraction index is exercised
    P_h = rng.permutation(I).astype(np.int32) if perm else None
    W, X, dY = to_dev(Wh, dtype), to_dev(Xh, dtype), to_dev(dYh, dtype)
    P = i32_dev(P_h) if perm else None
    B, vals, index = bm.bimask_forward_mask_compress(W, N, M)
    Bbar, vb, ib = bm.bimask_backward_mask_compress(W, N, M, B, P)
    B_o = oracle.forward_mask(W64, N, M)
    Bbar_o, _ = oracle.backward_mask(W64, B_o, P_h, N, M)
    assert (words(B) == oracle.pack_bits(B_o)).all() and (words(Bbar) == oracle.pack_bits(Bbar_o)).all()
    Y = bm.bimask_sparse_gemm_fwd(X, vals, index, I, J, N, M)
    dX = bm.bimask_sparse_gemm_bwd(dY, P, vb, ib, I, J, N, M)
    torch.cuda.synchronize()
    Y_o = oracle.gemm_fwd(synth.to_f64(Xh, dtype), W64, B_o)
    dX_o = oracle.gemm_bwd(synth.to_f64(dYh, dtype), W64, Bbar_o, P_h)
    assert np.abs(Y_o).max() <= 120 and np.abs(dX_o).max() <= 120 and np.abs(Y_o).max() > 0 and np.abs(dX_o).max() > 0
    gy, gx = from_dev_f64(Y, dtype), from_dev_f64(dX, dtype)
    bad_y, bad_x = np.argwhere(gy != Y_o), np.argwhere(gx != dX_o)
    assert bad_y.shape[0] == 0, f"forward: {bad_y.shape[0]} wrong outputs, first at (t, i) = {bad_y[0].tolist()}"
    assert bad_x.shape[0] == 0, f"backward: {bad_x.shape[0]} wrong outputs, first at (t, j) = {bad_x[0].tolist()}"


# (I, J, T): forward kernel / backward kernel (with a permutation)
SP24_SHAPES = [
    (64, 148, 300),      # wavefront-private, 296-byte rows / wavefront-private, 5 row tiles, 296-byte output rows
    (256, 64, 300),      # wavefront-private, two sibling wavefronts / wavefront-private 2 x 2 stages
    (224, 64, 150),      # wavefront-private, 7 row tiles over 2 x 4 / ...
    (64, 512, 600),      # wavefront-private, 4 stages / resident-token 256 x 64
    (160, 128, 200),     # wavefront-private, 5 row tiles / wavefront-private split
    (128, 256, 700),     # streaming 128 x 64 / wavefront-private split with the fused gather
    (512, 128, 300),     # resident-token 256 x 64, one stage / resident-token 128 x 32 ... 4 stages: 256 x 64
    (1024, 192, 300),    # resident-token, two stages / streaming after the separate gather (few tokens)
    (256, 124, 300),     # resident-token / resident-token 128 x 32, two stages
    (124, 128, 300),     # wavefront-private / resident-token 128 x 32, one stage, contraction 124
    (512, 128, 16400),   # ... / row-resident <2,1> (at least 512 tiles of 32 tokens)
    (384, 384, 16400),   # streaming 128 x 64 / row-resident <3,1>
    (512, 512, 16400),   # streaming 256 x 64 / row-resident <2,2>
    (1536, 384, 400),    # streaming / row-resident, 12 stages
    (2048, 512, 600),    # streaming / row-resident <2,2>, 16 stages
    (64, 576, 500),      # streaming 64 x 64 with a ragged last stage / resident-token 256 x 64
    (64, 576, 66000),    # ... / resident-token 256 x 64, persistent
    (256, 576, 66000),   # streaming 256 x 128 / resident-token 256 x 64 persistent, two stages
    (256, 2304, 2400),   # streaming 256 x 64, 18 stages / resident-token, two stages
    (384, 640, 700),     # streaming 128 x 64 (384 rows = 1.5 tiles of 256)
    (2100, 64, 600),     # resident-token, ragged rows / separate gather, then streaming 64 x 64 with 17 stages
    (1024, 1028, 300),   # streaming, ragged last stage / separate gather
    (2560, 1024, 2600),  # streaming 256 x 128 both ways (the tile of the largest layers), separate gather
    (4096, 2048, 8200),  # forward: 512 x 128 tiles (8 x 65 tiles, the last token tile ragged) / separate gather, streaming 256 x 128
    (3200, 1152, 22037), # 512 x 128 tiles both ways (the backward one behind the separate gather): 6.25 and 2.25 weight tiles, ragged last token tile
    (1024, 1152, 65600), # 512 x 128 tiles: two / three weight tiles, 513 token tiles (65 per XCD, the last XCD's run shorter)
    (4352, 256, 2051),   # ... / separate gather with four token rows interleaved per tile (8.5 KB rows), ragged last tile
    (8704, 128, 2305),   # ... / separate gather with two token rows interleaved per tile (17 KB rows), one row in the last tile
    (4224, 1024, 11200), # 512 x 128 tiles: nine weight tiles (the last with 128 rows) x 88 token tiles, 99 tiles per XCD on 32 workgroups (3 or 4 each)
]


@pytest.mark.parametrize("I,J,T", SP24_SHAPES)
@pytest.mark.parametrize("perm", [True, False], ids=["perm", "identity"])
def test_sparse_core_gemms_are_exact_on_integer_operands(I, J, T, perm):
    exact_layer(I, J, T, 2, 4, synth.BF16, 7000 + I + J + T, perm=perm)


@pytest.mark.parametrize("N,M", [(1, 4), (2, 8), (1, 16)])
def test_other_ratios_on_the_sparse_cores_are_exact(N, M):
    exact_layer(256, 384, 500, N, M, synth.BF16, 7100 + M + N)
    exact_layer(64, 128, 200, N, M, synth.BF16, 7200 + M + N)


@pytest.mark.parametrize("I,J,T", [(384, 384, 500), (1536, 384, 600), (384, 1536, 1600), (136, 1032, 1100), (64, 72, 80),
                                   (1152, 384, 16400)])
@pytest.mark.parametrize("perm", [True, False], ids=["perm", "identity"])
def test_dense_core_gemms_4of8_are_exact(I, J, T, perm):
    exact_layer(I, J, T, 4, 8, synth.BF16, 7300 + I + J, perm=perm)


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8)])
def test_fp32_gemms_are_exact(N, M):
    exact_layer(64, 128, 40, N, M, synth.F32, 7400 + M)
    exact_layer(136, 264, 300, N, M, synth.F32, 7500 + M)


def test_large_shapes_with_padded_leading_dimensions():
    """The 512 x 128 forward kernel and the row-interleaved gather of the backward pass on activations whose rows
    are longer than the matrices (ldx > J, lddy > I, ldy > I, lddx > J): the outputs must equal those of the
    packed call (which the exact tests above compare with the oracle), and the padding must stay untouched."""
    import torch
    I, J, T, pad = 4096, 1024, 16400, 8
    rng = np.random.default_rng(515)
    Wh = synth.store(int_weights(I, J, rng), synth.BF16)
    Xh = synth.store(sparse_rows(T, J, rng), synth.BF16)
    dYh = synth.store(sparse_rows(T, I, rng), synth.BF16)
    W, X, dY = to_dev(Wh, synth.BF16), to_dev(Xh, synth.BF16), to_dev(dYh, synth.BF16)
    P = i32_dev(rng.permutation(I).astype(np.int32))
    B, vals, index = bm.bimask_forward_mask_compress(W, 2, 4)
    _, vb, ib = bm.bimask_backward_mask_compress(W, 2, 4, B, P)
    Y = bm.bimask_sparse_gemm_fwd(X, vals, index, I, J, 2, 4)
    dX = bm.bimask_sparse_gemm_bwd(dY, P, vb, ib, I, J, 2, 4)
    fill = -3.0
    Xp = torch.full((T, J + pad), fill, dtype=torch.bfloat16, device=X.device)
    dYp = torch.full((T, I + pad), fill, dtype=torch.bfloat16, device=X.device)
    Xp[:, :J], dYp[:, :I] = X, dY
    Yp = torch.full((T, I + pad), fill, dtype=torch.bfloat16, device=X.device)
    dXp = torch.full((T, J + pad), fill, dtype=torch.bfloat16, device=X.device)
    bm.bimask_sparse_gemm_fwd(Xp[:, :J], vals, index, I, J, 2, 4, Y=Yp[:, :I])
    bm.bimask_sparse_gemm_bwd(dYp[:, :I], P, vb, ib, I, J, 2, 4, dX=dXp[:, :J])
    torch.cuda.synchronize()
    assert torch.equal(Yp[:, :I], Y) and torch.equal(dXp[:, :J], dX)
    assert bool((Yp[:, I:] == fill).all()) and bool((dXp[:, J:] == fill).all())
    assert float(Y.float().abs().max()) > 0 and float(dX.float().abs().max()) > 0
