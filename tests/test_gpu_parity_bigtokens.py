"""GPU parity of the two GEMMs at the token counts of the workloads' first layers.

Which kernel variant the library picks for Eq. (3) / Eq. (10) depends on the token count as well as on
the weight shape: hundreds of thousands of tokens select persistent workgroups (a loop over token tiles
with the next tile's rows requested one tile ahead) and larger streaming tiles.  The tests here run
those variants at token counts that select them and compare EVERY output element with the float64
oracle matmul, in token chunks: all 25 ResNet-50 layers with more than 16384 tokens at their full token
count, and synthetic layers aimed at one variant each (variant named beside the case).  The masks and
compressed operands of the same layers are compared bit for bit as well (the weights are small).
"""
import numpy as np
import pytest

import oracle
import paper_2302_06058_amd as bm
from paper_2302_06058_amd import synth
from helpers import to_dev, i32_dev, words, from_dev_f64, GemmError

pytestmark = pytest.mark.gpu

TOL = 2e-2
CHUNK = 1 << 16


def whole_output_errors(out_dev, act_h, Wm64, dtype=synth.BF16):
    """Every element of out = act @ Wm64.T against the float64 library matmul, chunked over tokens."""
    T = act_h.shape[0]
    absW = np.abs(Wm64).astype(np.float32)
    e = GemmError(K=Wm64.shape[1])
    for t0 in range(0, T, CHUNK):
        a64 = synth.to_f64(act_h[t0:t0 + CHUNK], dtype)
        ref = a64 @ Wm64.T
        S = (np.abs(a64).astype(np.float32) @ absW.T).astype(np.float64)
        e.add(from_dev_f64(out_dev[t0:t0 + CHUNK], dtype), ref, S)
    return e


def run_layer_gemms(I, J, T, seed, w_std=0.05, x_relu=False, j_real=None, perm=True, ld_extra=0):
    """Masks and operands through the library (checked against the oracle), then both GEMMs at T tokens
    with every output compared.  Returns the two GemmError records."""
    import torch
    dt = synth.BF16
    L = synth.Layer("big", I, J, T, 2, 4, 1, dt, seed, w_std, x_relu, 1.0, 1e-2, j_real)
    Wh = synth.gen_weights(L)
    W64 = synth.to_f64(Wh, dt)
    W = to_dev(Wh, dt)
    B_o = oracle.forward_mask(W64, 2, 4)
    B, vals, index = bm.bimask_forward_mask_compress(W, 2, 4)
    assert (words(B) == oracle.pack_bits(B_o)).all()
    P_h = synth.gen_perms(L, 1)[0] if perm else None
    P = i32_dev(P_h) if perm else None
    Bbar_o, _ = oracle.backward_mask(W64, B_o, P_h, 2, 4)
    Bbar, vb, ib = bm.bimask_backward_mask_compress(W, 2, 4, B, P)
    assert (words(Bbar) == oracle.pack_bits(Bbar_o)).all()

    Xh, dYh = synth.gen_activations(L), synth.gen_out_grad(L)
    if ld_extra:                     # rows embedded in wider buffers: leading dimension > columns
        def embed(a):
            t = to_dev(a, dt)
            big = torch.zeros((t.shape[0], t.shape[1] + ld_extra), dtype=t.dtype, device=t.device)
            big[:, :t.shape[1]] = t
            return big[:, :t.shape[1]]
        X, dY = embed(Xh), embed(dYh)
    else:
        X, dY = to_dev(Xh, dt), to_dev(dYh, dt)
    Y = bm.bimask_sparse_gemm_fwd(X, vals, index, I, J, 2, 4)
    dX = bm.bimask_sparse_gemm_bwd(dY, P, vb, ib, I, J, 2, 4)
    torch.cuda.synchronize()
    assert Y.shape == (T, I) and dX.shape == (T, J)
    ey = whole_output_errors(Y, Xh, W64 * B_o)
    Wp = W64 if P_h is None else W64[P_h, :]
    dYp = dYh if P_h is None else np.ascontiguousarray(dYh[:, P_h])
    ex = whole_output_errors(dX, dYp, np.ascontiguousarray((Wp * Bbar_o).T))
    print(f"  {I}x{J} T={T}: Y {ey}; dX {ex}", flush=True)
    assert ey.rel <= TOL and ex.rel <= TOL, (ey, ex)
    assert ey.excess <= 1.0 and ex.excess <= 1.0, (ey, ex)
    return ey, ex


BIG = [L for L in synth.get_config(3) if L.T > 16384]


def test_there_are_25_such_layers():
    assert len(BIG) == 25 and min(L.T for L in BIG) == 50176 and max(L.T for L in BIG) == 802816


@pytest.mark.parametrize("idx", range(len(BIG)), ids=[L.name for L in BIG])
def test_config3_layers_with_many_tokens_at_full_token_count(idx):
    L = BIG[idx]
    run_layer_gemms(L.I, L.J, L.T, L.seed, w_std=L.w_std, x_relu=L.x_relu, j_real=L.j_real)


@pytest.mark.parametrize("I,J,T,perm,ld_extra", [
    # wavefront-private kernel, several tiles per wavefront (one-tile-ahead prefetch, LDS area reused):
    (64, 148, 140017, True, 0),      # forward 2 row tiles x 2 stages, rows of 296 bytes; backward 5 row tiles, 296-byte output rows
    (256, 64, 140017, True, 0),      # forward: 8 row tiles over two sibling wavefronts; backward 2 x 2
    (64, 256, 140017, True, 0),      # backward: two sibling wavefronts with the fused gather
    (224, 64, 140017, True, 0),      # forward: 7 row tiles over two wavefronts of 4 (the last one re-reads tile 6)
    (160, 128, 70001, False, 0),     # 5 row tiles in one wavefront, identity permutation
    # resident-token kernel, persistent 256 x 64 variant (at least 1024 tiles of 64 tokens):
    (64, 576, 70019, True, 0),       # backward: one stage, fused gather
    (256, 576, 70019, True, 0),      # backward: two stages (more in-features than out-features: the row-resident kernel declines)
    (512, 128, 70019, False, 0),     # forward: one stage, no permutation; backward identity: streaming tiles
    (1024, 192, 66000, True, 0),     # forward: two stages; backward: row-resident kernel with 4 stages... K = 1024
    # resident-token kernel, persistent 128 x 32 variant with more than 768 tiles:
    (256, 124, 30011, True, 0),      # backward: 124 in-features (no multiple of 8), two stages
    (124, 128, 30011, True, 0),      # backward: contraction 124 with a permutation, one stage
    (128, 96, 30011, False, 8),      # leading dimensions that are no multiple of 8... + 8 keeps 16-byte rows; identity
    (96, 200, 30011, True, 4),       # rows not 16-byte aligned: the guarded paths of the workgroup kernels at many tokens
    # row-resident backward kernel at many tokens, and the streaming tiles chosen for them:
    (512, 128, 50176 + 13, True, 0), (256, 512, 50176 + 13, True, 0), (1536, 384, 66000, True, 0),
])
def test_token_counts_that_select_the_persistent_variants(I, J, T, perm, ld_extra):
    run_layer_gemms(I, J, T, 5000 + I + J, perm=perm, ld_extra=ld_extra)
