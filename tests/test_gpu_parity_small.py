"""GPU parity, small sizes: every entry point of the C-ABI library against the CPU
oracle on the same seeded inputs.  Shapes span several tiles and ragged tails.
Masks, scores, permutation choice and compressed operands are compared bit for bit;
GEMM outputs within 2e-2 (bf16 in, fp32 accumulate) / 1e-5 (fp32) of the float64
oracle in max|err| / max|ref|."""
import numpy as np
import pytest

import oracle
import paper_2302_06058_amd as bm
from paper_2302_06058_amd import synth
from helpers import to_dev, i32_dev, words, from_dev_f64, raw_bits, f64_to_raw, rel_err, untile24, untile_dense

pytestmark = pytest.mark.gpu

TOL = {synth.BF16: 2e-2, synth.F32: 1e-5}
NMS = [(2, 4), (1, 4), (4, 8), (2, 8), (1, 16)]


def make_w(I, J, dtype, seed, kind="normal"):
    r = np.random.default_rng(seed)
    if kind == "normal":
        w = r.standard_normal((I, J), dtype=np.float32)
    elif kind == "integers":                      # ties everywhere
        w = r.integers(-3, 4, size=(I, J)).astype(np.float32)
    elif kind == "special":
        w = r.standard_normal((I, J), dtype=np.float32)
        w[0] = 0.0
        w[1 % I] = 1.0
        w[2 % I] = -w[2 % I]
        w[3 % I, ::2] = -0.0
        w[3 % I, 1::2] = 0.0
        w[:, :4] = np.array([0.5, -0.5, 0.5, -0.5], dtype=np.float32)
    return synth.store(w, dtype)


def perms_of(I, K, seed, identity_first=False):
    r = np.random.default_rng(seed)
    p = np.stack([r.permutation(I) for _ in range(K)]).astype(np.int32)
    if identity_first:
        p[0] = np.arange(I)
    return p


def check_layer(I, J, N, M, dtype, K, seed, kind="normal", T=0):
    """Runs every call on one synthetic layer and compares with the oracle."""
    Wh = make_w(I, J, dtype, seed, kind)
    W64 = synth.to_f64(Wh, dtype)
    perms = perms_of(I, K, seed + 1, identity_first=(seed % 2 == 0))
    W = to_dev(Wh, dtype)
    s24 = N <= 2          # operands in the 2-of-4 format of the sparse matrix instruction

    # ---- forward mask (+ fused compress, + stand-alone compress)
    B_o = oracle.forward_mask(W64, N, M)
    Bw_o = oracle.pack_bits(B_o)
    B = bm.bimask_forward_mask(W, N, M)
    assert (words(B) == Bw_o).all(), "forward mask"
    B2, vals, index = bm.bimask_forward_mask_compress(W, N, M)
    assert (words(B2) == Bw_o).all(), "fused forward mask"
    vals_s, index_s = bm.bimask_compress_nm(W, N, M, B, None, 0)
    got_v, got_vs = raw_bits(vals, dtype), raw_bits(vals_s, dtype)
    if s24:
        # (2, 4): the method's own compression.  Other ratios with N <= 2: the mask already holds at
        # most two ones per aligned group of 4, and the oracle compresses that mask as 2-of-4.
        val_o, idx_o = oracle.compress_fwd(W64, B_o, 2, 4)
        want_v, want_i = f64_to_raw(val_o, dtype), oracle.pack_index(idx_o, 4)
        got_v, got_i, pz = untile24(got_v, words(index), I, J)
        got_vs, got_is, pzs = untile24(got_vs, words(index_s), I, J)
        assert pz and pzs, "forward operand padding must be zero"
        assert (got_i == want_i).all() and (got_is == want_i).all(), "forward index"
    else:
        want_v = f64_to_raw(W64 * B_o, dtype)
        got_v, pz = untile_dense(got_v, I, J)
        got_vs, pzs = untile_dense(got_vs, I, J)
        assert pz and pzs, "forward operand padding must be zero"
    # -0.0 weights: a kept -0 stays -0, a dropped slot is +0 -> compare bit patterns of the oracle's
    # exact values, treating +-0 alike
    def same_bits(a, b):
        za = (a & (0x7FFF if dtype == synth.BF16 else 0x7FFFFFFF)) == 0
        zb = (b & (0x7FFF if dtype == synth.BF16 else 0x7FFFFFFF)) == 0
        return ((a == b) | (za & zb)).all()
    assert same_bits(got_v, want_v), "fused forward values"
    assert same_bits(got_vs, want_v), "stand-alone forward values"

    # ---- permutation search
    sc_o = oracle.perm_scores(B_o, perms, N, M)
    best_o = oracle.argmax_first(sc_o)
    Pd = i32_dev(perms)
    scores, best, best_perm = bm.bimask_perm_search(B, I, J, N, M, Pd)
    assert (scores.cpu().numpy().astype(np.int64) == sc_o).all(), "scores"
    assert int(best.item()) == best_o, "best"
    assert (best_perm.cpu().numpy() == perms[best_o]).all(), "best_perm"

    # ---- backward mask (+ fused / stand-alone transposed compress), with P and with identity
    for P_h, P_d in ((perms[best_o], best_perm), (None, None)):
        Bbar_o, _ = oracle.backward_mask(W64, B_o, P_h, N, M)
        Bbw_o = oracle.pack_bits(Bbar_o)
        Bbar = bm.bimask_backward_mask(W, N, M, B, P_d)
        assert (words(Bbar) == Bbw_o).all(), "backward mask"
        Bbar2, vb, ib = bm.bimask_backward_mask_compress(W, N, M, B, P_d)
        assert (words(Bbar2) == Bbw_o).all(), "fused backward mask"
        vb_s, ib_s = bm.bimask_compress_nm(W, N, M, Bbar, P_d, 1)
        got_vb, got_vbs = raw_bits(vb, dtype), raw_bits(vb_s, dtype)
        if s24:
            if (N, M) == (2, 4):
                valb_o, idxb_o = oracle.compress_bwd(W64, B_o, P_h, N, M)
            else:       # the transposed masked matrix, compressed as 2-of-4 along the permuted rows
                Wp = W64 if P_h is None else W64[P_h, :]
                valb_o, idxb_o = oracle.compress_fwd(np.ascontiguousarray(Wp.T), np.ascontiguousarray(Bbar_o.T), 2, 4)
            want_vb, want_ib = f64_to_raw(valb_o, dtype), oracle.pack_index(idxb_o, 4)
            got_vb, got_ib, pz = untile24(got_vb, words(ib), J, I)
            got_vbs, got_ibs, pzs = untile24(got_vbs, words(ib_s), J, I)
            assert pz and pzs, "backward operand padding must be zero"
            assert (got_ib == want_ib).all() and (got_ibs == want_ib).all(), "backward index"
        else:
            Wp = W64 if P_h is None else W64[P_h, :]
            want_vb = f64_to_raw(np.ascontiguousarray((Wp * Bbar_o).T), dtype)
            got_vb, pz = untile_dense(got_vb, J, I)
            got_vbs, pzs = untile_dense(got_vbs, J, I)
            assert pz and pzs, "backward operand padding must be zero"
        assert same_bits(got_vb, want_vb), "fused backward values"
        assert same_bits(got_vbs, want_vb), "stand-alone backward values"

        # ---- GEMMs
        if T > 0:
            r = np.random.default_rng(seed + 7)
            Xh = synth.store(r.standard_normal((T, J), dtype=np.float32), dtype)
            dYh = synth.store(r.standard_normal((T, I), dtype=np.float32), dtype)
            X, dY = to_dev(Xh, dtype), to_dev(dYh, dtype)
            Y = bm.bimask_sparse_gemm_fwd(X, vals, index, I, J, N, M)
            Y_o = oracle.gemm_fwd(synth.to_f64(Xh, dtype), W64, B_o)
            assert rel_err(from_dev_f64(Y, dtype), Y_o) <= TOL[dtype], "forward GEMM"
            dX = bm.bimask_sparse_gemm_bwd(dY, P_d, vb, ib, I, J, N, M)
            dX_o = oracle.gemm_bwd(synth.to_f64(dYh, dtype), W64, Bbar_o, P_h)
            assert rel_err(from_dev_f64(dX, dtype), dX_o) <= TOL[dtype], "backward GEMM"


@pytest.mark.parametrize("dtype", [synth.BF16, synth.F32])
@pytest.mark.parametrize("N,M", NMS)
def test_small_layers_all_calls(dtype, N, M):
    # several tiles + ragged tails in every dimension (I, J multiples of M only)
    check_layer(I=9 * 16, J=13 * 16 + M, N=N, M=M, dtype=dtype, K=7, seed=100 + M + N, T=77)
    check_layer(I=272, J=144, N=N, M=M, dtype=dtype, K=11, seed=200 + M + N, T=130)


@pytest.mark.parametrize("dtype", [synth.BF16, synth.F32])
@pytest.mark.parametrize("kind", ["integers", "special"])
def test_adversarial_values(dtype, kind):
    for (N, M) in [(2, 4), (4, 8)]:
        check_layer(I=64, J=160, N=N, M=M, dtype=dtype, K=5, seed=300 + N, kind=kind, T=33)


@pytest.mark.parametrize("dtype", [synth.BF16, synth.F32])
def test_degenerate_shapes(dtype):
    check_layer(I=4, J=4, N=2, M=4, dtype=dtype, K=1, seed=401, T=1)          # one group, one block
    check_layer(I=4, J=148, N=2, M=4, dtype=dtype, K=3, seed=402, T=5)        # single row block, ragged J
    check_layer(I=1000, J=64, N=2, M=4, dtype=dtype, K=9, seed=403, T=64)     # ragged I (fc-like)
    check_layer(I=16, J=16, N=1, M=16, dtype=dtype, K=2, seed=404, T=3)


@pytest.mark.parametrize("I,J,N,M", [
    (64, 4224, 2, 4),     # row pitch 528 B: not a multiple of 128 -> wide slices, 16-byte row starts
    (32, 4360, 2, 4),     # 137 words per row: rows not 16-byte aligned, wide slices, ragged last slice
    (96, 2080, 2, 4),     # narrow slices, ragged last slice (2080 = 2 * 1024 + 32)
    (136, 1032, 4, 8),    # M = 8, row blocks not a multiple of the per-step group
    (208, 1040, 1, 16),   # M = 16
])
def test_perm_search_slice_paths(I, J, N, M):
    rng = np.random.default_rng(700 + J)
    Bo = np.zeros((I, J), dtype=np.uint8)
    for g in range(J // M):                                   # any N-per-group mask will do here
        idx = np.argsort(rng.random((I, M)), axis=1)[:, :N]
        np.put_along_axis(Bo[:, g * M:(g + 1) * M], idx, 1, axis=1)
    perms = perms_of(I, 13, 701 + J)
    wpr = (J + 31) // 32
    bits = np.zeros((I, wpr * 32), dtype=np.uint8)
    bits[:, :J] = Bo
    words = (bits.reshape(I, wpr, 32).astype(np.uint64) << np.arange(32, dtype=np.uint64)).sum(axis=2).astype(np.uint32)
    B = i32_dev(words.view(np.int32))
    scores, best, best_perm = bm.bimask_perm_search(B, I, J, N, M, i32_dev(perms))
    sc_o = oracle.perm_scores(Bo, perms, N, M)
    assert (scores.cpu().numpy() == sc_o).all()
    assert int(best.item()) == oracle.argmax_first(sc_o)
    assert (best_perm.cpu().numpy() == perms[int(best.item())]).all()


def test_duplicate_candidates_pick_the_first():
    I, J, N, M = 64, 128, 2, 4
    Wh = make_w(I, J, synth.BF16, 501)
    B_o = oracle.forward_mask(synth.to_f64(Wh, synth.BF16), N, M)
    base = perms_of(I, 3, 502)
    perms = np.concatenate([base, base, base[::-1]])
    B = bm.bimask_forward_mask(to_dev(Wh, synth.BF16), N, M)
    scores, best, best_perm = bm.bimask_perm_search(B, I, J, N, M, i32_dev(perms))
    sc_o = oracle.perm_scores(B_o, perms, N, M)
    assert (scores.cpu().numpy() == sc_o).all()
    assert int(best.item()) == oracle.argmax_first(sc_o) < 3


def test_identical_rows_closed_form_score():
    # every row has the same pattern -> each column is all ones or all zeros ->
    # score = (I/M) * J * (1 - N/M) for every permutation
    I, J, N, M = 128, 256, 2, 4
    row = np.random.default_rng(601).standard_normal((1, J), dtype=np.float32)
    Wh = synth.store(np.repeat(row, I, axis=0), synth.BF16)
    B = bm.bimask_forward_mask(to_dev(Wh, synth.BF16), N, M)
    scores, _, _ = bm.bimask_perm_search(B, I, J, N, M, i32_dev(perms_of(I, 6, 602)))
    assert (scores.cpu().numpy() == (I // M) * J // 2).all()


def test_config1_whole_step_fp32():
    layer = synth.get_config(1)[0]
    d = synth.gen_layer(layer)
    ref = oracle.bimask_step(synth.to_f64(d.W, layer.dtype), synth.to_f64(d.X, layer.dtype),
                             synth.to_f64(d.dY, layer.dtype), d.perms, layer.N, layer.M)
    W, X, dY = to_dev(d.W, layer.dtype), to_dev(d.X, layer.dtype), to_dev(d.dY, layer.dtype)
    B, vals, index = bm.bimask_forward_mask_compress(W, 2, 4)
    Y = bm.bimask_sparse_gemm_fwd(X, vals, index, layer.I, layer.J, 2, 4)
    scores, best, P = bm.bimask_perm_search(B, layer.I, layer.J, 2, 4, i32_dev(d.perms))
    Bbar, vb, ib = bm.bimask_backward_mask_compress(W, 2, 4, B, P)
    dX = bm.bimask_sparse_gemm_bwd(dY, P, vb, ib, layer.I, layer.J, 2, 4)
    assert (words(B) == oracle.pack_bits(ref["B"])).all()
    assert (scores.cpu().numpy() == ref["scores"]).all() and int(best.item()) == ref["best"]
    assert (words(Bbar) == oracle.pack_bits(ref["Bbar"])).all()
    assert rel_err(from_dev_f64(Y, layer.dtype), ref["Y"]) <= 1e-5
    assert rel_err(from_dev_f64(dX, layer.dtype), ref["dX"]) <= 1e-5
    # loops-based oracle GEMM as well (independent of the library matmul)
    Yl = oracle.gemm_fwd_loops(synth.to_f64(d.X, layer.dtype), synth.to_f64(d.W, layer.dtype), ref["B"])
    assert rel_err(from_dev_f64(Y, layer.dtype), Yl) <= 1e-5


def test_results_are_reproducible_bit_for_bit():
    I, J, N, M, K = 256, 512, 2, 4, 16
    Wh = make_w(I, J, synth.BF16, 701)
    W = to_dev(Wh, synth.BF16)
    Pd = i32_dev(perms_of(I, K, 702))
    outs = []
    for _ in range(2):
        B, v, ix = bm.bimask_forward_mask_compress(W, N, M)
        s, b, P = bm.bimask_perm_search(B, I, J, N, M, Pd)
        Bb, vb, ib = bm.bimask_backward_mask_compress(W, N, M, B, P)
        outs.append([words(B), raw_bits(v, synth.BF16), words(ix), s.cpu().numpy(), b.cpu().numpy(),
                     words(Bb), raw_bits(vb, synth.BF16), words(ib)])
    for a, b in zip(*outs):
        assert (a == b).all()


@pytest.mark.parametrize("I,J,T", [(256, 384, 200), (384, 256, 130), (128, 1152, 64), (640, 128, 333),
                                   (384, 640, 150), (640, 384, 90),    # 384 weight rows: 128-row tiles
                                   (512, 128, 150), (384, 64, 100),    # narrow backward operand, 3-4 stages
                                   (64, 640, 150), (48, 768, 70), (1024, 64, 90),    # <= 64 weight rows, long contraction: 64 x 64 tiles
                                   (64, 576, 150), (256, 328, 100), (576, 1032, 70), (320, 840, 90)])   # aligned rows, ragged last stage
def test_streaming_gemm_shapes(I, J, T):
    # contraction lengths that are multiples of 128 take the streaming 2:4 kernel in both
    # directions; ragged token counts and weight-row counts exercise its edge tiles
    check_layer(I=I, J=J, N=2, M=4, dtype=synth.BF16, K=6, seed=800 + I + J, T=T)


@pytest.mark.parametrize("I,J,T", [(1024, 128, 70), (640, 256, 100), (2560, 128, 70), (2100, 64, 45),
                                   (1024, 256, 333), (1536, 384, 130), (2048, 512, 45), (520, 40, 77), (1152, 384, 1),
                                   (1024, 1028, 40)])
def test_long_contraction_backward_uses_gather_pass(I, J, T):
    # 512 < I <= 2048 with J <= 512: whole rows of g(Y) resident in LDS, gather fused (520: ragged last
    # stage; 333 / 130 / 77 tokens: ragged last tile; J = 1028: too wide, falls back to the gather pass).
    # Otherwise g(Y)[:, P] is gathered into the workspace, then the streaming kernel runs;
    # I > 2048: the gather keeps its permutation entries in registers (2100: ragged last 16 bytes)
    check_layer(I=I, J=J, N=2, M=4, dtype=synth.BF16, K=4, seed=900 + I, T=T)


@pytest.mark.parametrize("I,J,T", [(384, 128, 16400), (256, 256, 16385), (512, 40, 16390), (136, 72, 16400),
                                   (512, 512, 16384), (260, 128, 16400)])
def test_short_contraction_backward_with_many_tokens(I, J, T):
    # 128 < I <= 512 and at least 512 tiles of 32 tokens: the backward GEMM keeps whole rows of g(Y) in LDS
    # (ragged last tile: 16400 = 512 x 32 + 16, 16385 = 512 x 32 + 1; I = 136: ragged second stage;
    # I = 260 is no multiple of 8: that one stays with the token-resident kernel)
    check_layer(I=I, J=J, N=2, M=4, dtype=synth.BF16, K=4, seed=950 + I, T=T)


@pytest.mark.parametrize("I,J,T", [(64, 148, 131), (68, 148, 131), (132, 260, 77), (64, 148, 4100), (36, 12, 9),
                                   (64, 64, 1), (224, 64, 31), (192, 96, 65), (64, 256, 8200)])
def test_narrow_weights_and_unaligned_contiguous_rows(I, J, T):
    # narrow weight matrices run one wavefront per 32-token tile (weights in registers; more than 160
    # weight rows are split over two wavefronts); row pitches of 296 / 136 / 520 / 24 bytes (the 7x7 stem's im2col width is 148): token tiles are
    # fetched and written as aligned contiguous blocks; odd last tiles end in a partial 16-byte piece
    check_layer(I=I, J=J, N=2, M=4, dtype=synth.BF16, K=4, seed=1000 + I + T, T=T)


@pytest.mark.parametrize("I,J,T", [(256, 384, 100), (1024, 256, 96),
                                   (64, 128, 77), (160, 64, 33), (256, 64, 70)])   # narrow weights: one wavefront per token tile
def test_leading_dimensions_side_stream_many_candidates(I, J, T):
    """Operands embedded in wider buffers (ld > columns), calls issued on a non-default stream,
    K > 128 candidates; the padding columns of the outputs must stay untouched."""
    import torch
    N, M, dtype, K = 2, 4, synth.BF16, 150
    Wh = make_w(I, J, dtype, 1201)
    W64 = synth.to_f64(Wh, dtype)
    perms = perms_of(I, K, 1202)
    r = np.random.default_rng(1203)
    Xh = synth.store(r.standard_normal((T, J), dtype=np.float32), dtype)
    dYh = synth.store(r.standard_normal((T, I), dtype=np.float32), dtype)

    def embed(a, extra):                       # device tensor whose rows sit in a wider buffer
        t = to_dev(a, dtype)
        big = torch.full((t.shape[0], t.shape[1] + extra), 7.0, dtype=t.dtype, device=t.device)
        big[:, :t.shape[1]] = t
        return big[:, :t.shape[1]]

    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        W, X, dY = embed(Wh, 24), embed(Xh, 8), embed(dYh, 16)
        Ybig = torch.full((T, I + 8), 3.0, dtype=torch.bfloat16, device="cuda")
        dXbig = torch.full((T, J + 40), 3.0, dtype=torch.bfloat16, device="cuda")
        B, vals, index = bm.bimask_forward_mask_compress(W, N, M)
        scores, best, P = bm.bimask_perm_search(B, I, J, N, M, i32_dev(perms))
        Bbar, vb, ib = bm.bimask_backward_mask_compress(W, N, M, B, P)
        bm.bimask_sparse_gemm_fwd(X, vals, index, I, J, N, M, Y=Ybig[:, :I])
        bm.bimask_sparse_gemm_bwd(dY, P, vb, ib, I, J, N, M, dX=dXbig[:, :J])
    side.synchronize()

    B_o = oracle.forward_mask(W64, N, M)
    sc_o = oracle.perm_scores(B_o, perms, N, M)
    best_o = oracle.argmax_first(sc_o)
    assert (words(B) == oracle.pack_bits(B_o)).all()
    assert (scores.cpu().numpy() == sc_o).all() and int(best.item()) == best_o
    assert (P.cpu().numpy() == perms[best_o]).all()
    Bbar_o, _ = oracle.backward_mask(W64, B_o, perms[best_o], N, M)
    assert (words(Bbar) == oracle.pack_bits(Bbar_o)).all()
    Y_o = oracle.gemm_fwd(synth.to_f64(Xh, dtype), W64, B_o)
    dX_o = oracle.gemm_bwd(synth.to_f64(dYh, dtype), W64, Bbar_o, perms[best_o])
    assert rel_err(Ybig[:, :I].float().cpu().numpy().astype(np.float64), Y_o) <= TOL[dtype]
    assert rel_err(dXbig[:, :J].float().cpu().numpy().astype(np.float64), dX_o) <= TOL[dtype]
    assert bool((Ybig[:, I:] == 3.0).all()) and bool((dXbig[:, J:] == 3.0).all()), "output padding was written"


GROUP_SHAPES = [(64, 148), (64, 64), (64, 576), (256, 64), (128, 1152), (512, 128), (32, 36), (8, 8), (256, 2304),
                (1024, 256), (100, 260), (64, 4100), (2048, 512), (16, 1028), (96, 96), (384, 384), (40, 44),
                (1000, 2048), (128, 256), (512, 256), (4096, 2048), (12, 20), (64, 256)]
GROUP_SHAPES += [(16 + 8 * (i % 7), 24 + 12 * (i % 11)) for i in range(50)]       # 73 layers: more than one launch holds


@pytest.mark.parametrize("N,M,dtype,nl", [(2, 4, synth.BF16, len(GROUP_SHAPES)), (1, 4, synth.BF16, 9), (2, 8, synth.BF16, 6),
                                          (2, 4, synth.F32, 7), (4, 8, synth.BF16, 5)])
def test_grouped_calls_equal_per_layer_calls(N, M, dtype, nl):
    """The grouped entry points (all layers of a network in a few launches) give bit-identical results
    to the per-layer calls (which the tests above tie to the oracle); one layer is also checked against
    the oracle directly.  73 layers are more than one launch's argument table holds (35-63 entries); the 4096 x 2048 layer is
    large enough to be launched on its own inside the grouped backward call."""
    import torch
    K = 12
    code = bm.BF16 if dtype == synth.BF16 else bm.F32
    tdt = torch.bfloat16 if dtype == synth.BF16 else torch.float32
    shapes = [(-(-I // M) * M, -(-J // M) * M) for I, J in GROUP_SHAPES[:nl]]
    entries, singles, hosts = [], [], []
    for li, (I, J) in enumerate(shapes):
        Wh = make_w(I, J, dtype, 3000 + li, "integers" if li % 5 == 4 else "normal")
        perms = perms_of(I, K, 3100 + li, identity_first=(li % 2 == 0))
        W, Pd = to_dev(Wh, dtype), i32_dev(perms)
        hosts.append((Wh, perms))
        # per-layer reference results
        B, vf, xf = bm.bimask_forward_mask_compress(W, N, M)
        scores, best, P = bm.bimask_perm_search(B, I, J, N, M, Pd)
        Bbar, vb, xb = bm.bimask_backward_mask_compress(W, N, M, B, P)
        singles.append((B, vf, xf, scores, best, P, Bbar, vb, xb))
        dev = W.device
        z = lambda t: None if t is None else torch.full_like(t, 0x55 if t.dtype == torch.int32 else 1.0)
        ws = torch.empty((max(16, bm.workspace_bytes(bm.WS_PERM_SEARCH, I, J, 0, K, code, N, M)),), dtype=torch.uint8, device=dev)
        entries.append(dict(W=W, B_bits=z(B), Wf_values=z(vf), Wf_index=z(xf), perms=Pd, scores=z(scores), best=z(best),
                            best_perm=z(P), workspace=ws, Bbar_bits=z(Bbar), Wb_values=z(vb), Wb_index=z(xb)))
    layers = bm.group_layers(entries)
    bm.bimask_forward_mask_compress_group(layers, code, N, M)
    bm.bimask_perm_search_group(layers, N, M, K)
    bm.bimask_backward_mask_compress_group(layers, code, N, M)
    torch.cuda.synchronize()
    names = ("B_bits", "Wf_values", "Wf_index", "scores", "best", "best_perm", "Bbar_bits", "Wb_values", "Wb_index")
    for li, (e, ref) in enumerate(zip(entries, singles)):
        for name, r in zip(names, ref):
            if r is None:
                continue
            got = e[name]
            a = got.view(torch.int16) if got.dtype == torch.bfloat16 else (got.view(torch.int32) if got.dtype == torch.float32 else got)
            b = r.view(torch.int16) if r.dtype == torch.bfloat16 else (r.view(torch.int32) if r.dtype == torch.float32 else r)
            assert torch.equal(a, b), f"layer {li} {shapes[li]}: {name}"
    # one layer straight against the oracle
    li = 2
    I, J = shapes[li]
    Wh, perms = hosts[li]
    W64 = synth.to_f64(Wh, dtype)
    B_o = oracle.forward_mask(W64, N, M)
    assert (words(entries[li]["B_bits"]) == oracle.pack_bits(B_o)).all()
    sc_o = oracle.perm_scores(B_o, perms, N, M)
    assert (entries[li]["scores"].cpu().numpy().astype(np.int64) == sc_o).all()
    best_o = oracle.argmax_first(sc_o)
    assert int(entries[li]["best"].item()) == best_o
    Bbar_o, _ = oracle.backward_mask(W64, B_o, perms[best_o], N, M)
    assert (words(entries[li]["Bbar_bits"]) == oracle.pack_bits(Bbar_o)).all()


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8)])
def test_other_binarisation_criteria_through_the_same_calls(N, M):
    """The criteria the paper compares for the backward mask (Sec. 4.4, "Binarization Criteria": gradient
    magnitude, random) need no other kernel: the mask call ranks whatever matrix it is given, so the
    criterion matrix G goes in where W went, and the stand-alone compression then packs W with that mask."""
    dtype, I, J, T = synth.BF16, 128, 192, 70
    Wh = make_w(I, J, dtype, 4001)
    Gh = make_w(I, J, dtype, 4002)                    # stands for |dL/dW| (or random keys)
    W64, G64 = synth.to_f64(Wh, dtype), synth.to_f64(Gh, dtype)
    P_h = perms_of(I, 1, 4003)[0]
    W, G, P = to_dev(Wh, dtype), to_dev(Gh, dtype), i32_dev(P_h)
    B = bm.bimask_forward_mask(W, N, M)
    B_o = oracle.forward_mask(W64, N, M)
    Bbar = bm.bimask_backward_mask(G, N, M, B, P)
    Bbar_o, _ = oracle.backward_mask(G64, B_o, P_h, N, M)
    assert (words(Bbar) == oracle.pack_bits(Bbar_o)).all()
    assert (Bbar_o <= B_o[P_h, :]).all() and (Bbar_o.reshape(I // M, M, J).sum(1) <= N).all()
    vb, ib = bm.bimask_compress_nm(W, N, M, Bbar, P, 1)
    r = np.random.default_rng(4004)
    dYh = synth.store(r.standard_normal((T, I), dtype=np.float32), dtype)
    dX = bm.bimask_sparse_gemm_bwd(to_dev(dYh, dtype), P, vb, ib, I, J, N, M)
    dX_o = oracle.gemm_bwd(synth.to_f64(dYh, dtype), W64, Bbar_o, P_h)
    assert rel_err(from_dev_f64(dX, dtype), dX_o) <= TOL[dtype]


# ---------------------------------------------------------------------------------------------
# refinement of a permutation by proposed exchanges (Limitations: future work)
# ---------------------------------------------------------------------------------------------
def _mask_with_n_per_group(I, J, N, M, seed, density=1.0):
    """A forward-mask-shaped 0/1 matrix: exactly N ones per group of M columns (fewer with density < 1)."""
    rng = np.random.default_rng(seed)
    Bo = np.zeros((I, J), dtype=np.uint8)
    for g in range(J // M):
        idx = np.argsort(rng.random((I, M)), axis=1)[:, :N]
        np.put_along_axis(Bo[:, g * M:(g + 1) * M], idx, 1, axis=1)
    if density < 1.0:
        Bo &= (rng.random((I, J)) < density).astype(np.uint8)
    return Bo


def _pack_mask(Bo):
    I, J = Bo.shape
    wpr = (J + 31) // 32
    bits = np.zeros((I, wpr * 32), dtype=np.uint8)
    bits[:, :J] = Bo
    w = (bits.reshape(I, wpr, 32).astype(np.uint64) << np.arange(32, dtype=np.uint64)).sum(axis=2).astype(np.uint32)
    return i32_dev(w.view(np.int32))


def _refine_both(Bo, N, M, P0, swaps):
    I, J = Bo.shape
    perm_dev = None if P0 is None else i32_dev(P0)
    out, res = bm.bimask_perm_refine(_pack_mask(Bo), I, J, N, M, i32_dev(swaps), perm=perm_dev)
    P_o, before, after, kept = oracle.perm_refine(Bo, P0, swaps, N, M)
    got = out.cpu().numpy()
    assert (got == P_o).all(), np.flatnonzero(got != P_o)[:8]
    assert res.cpu().numpy().tolist() == [after - before, kept]
    return kept, after - before


@pytest.mark.parametrize("I,J,N,M,S", [
    (64, 128, 2, 4, 700),        # few blocks: almost every round of 16 proposals meets a stale one
    (256, 2304, 2, 4, 1500),     # the config-2 layer
    (512, 100, 2, 4, 1200),      # ragged last word
    (128, 36, 1, 4, 600),
    (256, 4200, 4, 8, 900),      # more than 64 words per row: two passes of the lanes
    (192, 264, 2, 8, 900),
    (320, 208, 1, 16, 900),
    (4096, 64, 2, 4, 2500),      # many blocks: whole rounds without a stale proposal
])
def test_perm_refine_equals_one_by_one_hill_climbing(I, J, N, M, S):
    rng = np.random.default_rng(900 + I + J)
    Bo = _mask_with_n_per_group(I, J, N, M, 901 + J)
    swaps = rng.integers(0, I, size=(S, 2)).astype(np.int32)
    swaps[5] = (-1, 3)                                      # positions that do not exist are skipped
    swaps[6] = (2, I)
    swaps[7] = (M, M + 1)                                   # inside one block: never kept
    P0 = rng.permutation(I).astype(np.int32)
    kept, gain = _refine_both(Bo, N, M, P0, swaps)
    assert kept > 0 and gain >= kept
    _refine_both(Bo, N, M, None, swaps[:40])                # NULL = identity


def test_perm_refine_edge_cases():
    N, M, I, J = 2, 4, 64, 64
    Bo = _mask_with_n_per_group(I, J, N, M, 950)
    B = _pack_mask(Bo)
    P0 = np.random.default_rng(951).permutation(I).astype(np.int32)
    # no proposals: a copy
    out, res = bm.bimask_perm_refine(B, I, J, N, M, i32_dev(np.zeros((0, 2), np.int32)), perm=i32_dev(P0))
    assert (out.cpu().numpy() == P0).all() and res.cpu().numpy().tolist() == [0, 0]
    # in place, one proposal, and a number of proposals that is no multiple of the round or the staging chunk
    for S in (1, 15, 17, 63, 65, 129, 1023, 1025, 2050):
        swaps = np.random.default_rng(952 + S).integers(0, I, size=(S, 2)).astype(np.int32)
        buf = i32_dev(P0)
        out, res = bm.bimask_perm_refine(B, I, J, N, M, i32_dev(swaps), perm=buf, perm_out=buf)
        P_o, before, after, kept = oracle.perm_refine(Bo, P0, swaps, N, M)
        assert (out.cpu().numpy() == P_o).all() and res.cpu().numpy().tolist() == [after - before, kept]
    # the same proposal many times in a row: kept once at most
    swaps = np.tile(np.array([[1, 9]], np.int32), (40, 1))
    _refine_both(Bo, N, M, P0, swaps)
    # an all-zero mask: every block is eligible already, nothing can grow
    Z = np.zeros((I, J), np.uint8)
    kept, gain = _refine_both(Z, N, M, P0, np.random.default_rng(953).integers(0, I, size=(100, 2)).astype(np.int32))
    assert kept == 0 and gain == 0


def test_perm_refine_largest_permutation_and_limit():
    N, M, I, J = 2, 4, 32768, 32                           # the whole 128 KB of permutation in LDS
    Bo = _mask_with_n_per_group(I, J, N, M, 960)
    swaps = np.random.default_rng(961).integers(0, I, size=(200, 2)).astype(np.int32)
    _refine_both(Bo, N, M, None, swaps)
    with pytest.raises(bm.BimaskError) as e:
        bm.bimask_perm_refine(_pack_mask(np.zeros((32768 + 4, 32), np.uint8)), 32768 + 4, 32, N, M, i32_dev(swaps))
    assert e.value.status == 5


@pytest.mark.parametrize("I,J,T,N,M", [(128, 256, 200, 2, 4), (1024, 256, 150, 2, 4), (64, 128, 96, 4, 8)])
def test_whole_step_recorded_as_a_hip_graph_replays_like_eager_calls(I, J, T, N, M):
    """The library allocates nothing and records no memset, so a whole step can be captured into a HIP
    graph.  Replayed several times, with new weights and activations written (eager work on the same
    stream) between the replays, every replay must give what the eager calls give on the same inputs,
    and those agree with the oracle."""
    import torch
    dtype, K = synth.BF16, 20
    perms_h = perms_of(I, K, 1302)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        W = to_dev(make_w(I, J, dtype, 1301), dtype)
        X = torch.empty((T, J), dtype=torch.bfloat16, device="cuda")
        dY = torch.empty((T, I), dtype=torch.bfloat16, device="cuda")
        perms = i32_dev(perms_h)
        # every output and workspace allocated before the capture
        B, vals, index = bm.bimask_forward_mask_compress(W, N, M)
        scores, best, P = bm.bimask_perm_search(B, I, J, N, M, perms)
        ws = torch.empty((max(16, bm.workspace_bytes(bm.WS_PERM_SEARCH, I, J, 0, K, bm.BF16, N, M)),), dtype=torch.uint8, device="cuda")
        Bbar, vb, ib = bm.bimask_backward_mask_compress(W, N, M, B, P)
        Y = torch.empty((T, I), dtype=torch.bfloat16, device="cuda")
        dX = torch.empty((T, J), dtype=torch.bfloat16, device="cuda")
        wsb = torch.empty((max(16, bm.workspace_bytes(bm.WS_GEMM_BWD, I, J, T, 0, bm.BF16, N, M)),), dtype=torch.uint8, device="cuda")

        def step():
            bm.bimask_forward_mask_compress(W, N, M, B_bits=B, values=vals, index=index)
            bm.bimask_sparse_gemm_fwd(X, vals, index, I, J, N, M, Y=Y)
            bm.bimask_perm_search(B, I, J, N, M, perms, scores=scores, best=best, best_perm=P, workspace=ws)
            bm.bimask_backward_mask_compress(W, N, M, B, P, Bbar_bits=Bbar, values=vb, index=ib)
            bm.bimask_sparse_gemm_bwd(dY, P, vb, ib, I, J, N, M, dX=dX, workspace=wsb)

        def fill(seed):
            r = np.random.default_rng(seed)
            Wn = make_w(I, J, dtype, seed)
            Xn = synth.store(r.standard_normal((T, J), dtype=np.float32), dtype)
            dYn = synth.store(r.standard_normal((T, I), dtype=np.float32), dtype)
            W.copy_(to_dev(Wn, dtype)); X.copy_(to_dev(Xn, dtype)); dY.copy_(to_dev(dYn, dtype))
            return Wn, Xn, dYn

        outputs = (B, vals, scores, best, P, Bbar, vb, Y, dX)
        fill(1310)
        step()                                               # warm-up: one-time set-up calls happen here
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for rep in range(3):
            Wn, Xn, dYn = fill(1320 + rep)
            step()
            side.synchronize()
            want = [t.clone() for t in outputs]
            for t in outputs:
                t.fill_(0)                                   # a replay must rewrite everything
            side.synchronize()
            graph.replay()
            side.synchronize()
            for got, w in zip(outputs, want):
                assert torch.equal(got, w), rep
        # the last replay against the oracle
        W64 = synth.to_f64(Wn, dtype)
        B_o = oracle.forward_mask(W64, N, M)
        sc_o = oracle.perm_scores(B_o, perms_h, N, M)
        best_o = oracle.argmax_first(sc_o)
        assert (words(B) == oracle.pack_bits(B_o)).all()
        assert (scores.cpu().numpy() == sc_o).all() and int(best.item()) == best_o
        Bbar_o, _ = oracle.backward_mask(W64, B_o, perms_h[best_o], N, M)
        assert (words(Bbar) == oracle.pack_bits(Bbar_o)).all()
        assert rel_err(Y.float().cpu().numpy().astype(np.float64), oracle.gemm_fwd(synth.to_f64(Xn, dtype), W64, B_o)) <= TOL[dtype]
        assert rel_err(dX.float().cpu().numpy().astype(np.float64),
                       oracle.gemm_bwd(synth.to_f64(dYn, dtype), W64, Bbar_o, perms_h[best_o])) <= TOL[dtype]


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8), (1, 16)])
def test_perm_refine_group_equals_per_layer_calls(N, M):
    """Many layers refined by one launch (one workgroup each, permutations refined in place) give what the
    per-layer call gives, which the tests above tie to the oracle; one layer is checked against it here too."""
    import torch
    shapes = [(64, 128), (256, 2304 if M == 4 else 640), (512, 96), (4096, 64), (128, 32 * M), (16 * M, 16 * M)] * 12   # 72 layers: two launches
    rng = np.random.default_rng(1400 + M)
    entries, want, keep = [], [], []
    for n, (I, J) in enumerate(shapes):
        Bo = _mask_with_n_per_group(I, J, N, M, 1401 + n)
        B = _pack_mask(Bo)
        P0 = rng.permutation(I).astype(np.int32)
        S = int(rng.integers(0, 300)) if n % 7 else 0
        swaps_h = rng.integers(0, I, size=(S, 2)).astype(np.int32)
        swaps = i32_dev(swaps_h) if S else None
        if S:
            out, res = bm.bimask_perm_refine(B, I, J, N, M, swaps, perm=i32_dev(P0))
        else:
            out, res = i32_dev(P0), torch.zeros(2, dtype=torch.int32, device="cuda")
        want.append((out.cpu().numpy(), res.cpu().numpy()))
        P = i32_dev(P0)
        result = torch.full((2,), -7, dtype=torch.int32, device="cuda")
        keep.append((B, P, swaps, result, Bo, P0, swaps_h))
        entries.append(dict(W=torch.empty((I, J), dtype=torch.bfloat16, device="cuda"), B_bits=B, best_perm=P, swaps=swaps,
                            refine_result=result))
    arr = bm.group_layers(entries)
    bm.bimask_perm_refine_group(arr, N, M)
    torch.cuda.synchronize()
    for (B, P, swaps, result, Bo, P0, swaps_h), (wp, wr) in zip(keep, want):
        assert (P.cpu().numpy() == wp).all()
        assert (result.cpu().numpy() == wr).all()
    B, P, swaps, result, Bo, P0, swaps_h = keep[1]
    P_o, before, after, kept = oracle.perm_refine(Bo, P0, swaps_h, N, M)
    assert (P.cpu().numpy() == P_o).all() and result.cpu().numpy().tolist() == [after - before, kept]


@pytest.mark.parametrize("I,K", [(64, 9), (1000, 5), (11008, 6), (100000, 3), (1 << 20, 2)])
def test_check_perms_flags(I, K):
    rng = np.random.default_rng(1500 + K)
    perms = np.stack([rng.permutation(I) for _ in range(K)]).astype(np.int32)
    perms[1, I // 3] = perms[1, I // 2]                     # a repeated value
    if K > 2:
        perms[2, I - 1] = I                                 # out of range
    if K > 4:
        perms[4, 0] = -1
    ok = bm.bimask_check_perms(i32_dev(perms))
    assert (ok.cpu().numpy() == oracle.is_permutation(perms)).all()
    assert ok.cpu().numpy().tolist()[:2] == [1, 0]


@pytest.mark.parametrize("I,J,N,M", [(4, 131072, 2, 4), (131072, 4, 2, 4), (16, 65536, 1, 16), (65536, 16, 1, 16),
                                     (8, 100000, 4, 8), (100000, 8, 4, 8)])
def test_extreme_aspect_ratios(I, J, N, M):
    # one block of permuted rows against very long rows, and the transpose of that: the row / column
    # tilings of every kernel meet their smallest and their longest dimension (few tokens: the GEMMs are
    # here for their indexing, not their speed)
    check_layer(I=I, J=J, N=N, M=M, dtype=synth.BF16, K=3, seed=1600 + M, T=9)


@pytest.mark.parametrize("I,J,T,N,M", [(256, 384, 300, 2, 4), (128, 192, 200, 1, 4), (192, 256, 260, 4, 8)])
def test_gradient_gap_against_the_oracle(I, J, T, N, M):
    """Sec. 3.3's gradient gap ||g-bar(X) - g(X)|| / ||g(X)||: g-bar(X) of Eq. (10) from the library's masks, search
    and backward GEMM, against the oracle's float64 gap for the same permutation; g(X) is Eq. (5) from the oracle.
    For the identity and for the search's winner; the two must agree to 1e-2 relative (bf16 outputs)."""
    dtype = synth.BF16
    Wh = make_w(I, J, dtype, 5001)
    W64 = synth.to_f64(Wh, dtype)
    r = np.random.default_rng(5002)
    dYh = synth.store(r.standard_normal((T, I), dtype=np.float32), dtype)
    dY64 = synth.to_f64(dYh, dtype)
    perms = perms_of(I, 16, 5003)
    W, dY = to_dev(Wh, dtype), to_dev(dYh, dtype)
    B = bm.bimask_forward_mask(W, N, M)
    B_o = oracle.forward_mask(W64, N, M)
    exact = oracle.grad_exact(dY64, W64, B_o)
    scores, best, P = bm.bimask_perm_search(B, I, J, N, M, i32_dev(perms))
    gaps = []
    for P_d, P_h in ((None, None), (P, perms[int(best.item())])):
        Bbar, vb, ib = bm.bimask_backward_mask_compress(W, N, M, B, P_d)
        approx = from_dev_f64(bm.bimask_sparse_gemm_bwd(dY, P_d, vb, ib, I, J, N, M), dtype)
        got = oracle.relative_gap(approx, exact)
        want = oracle.gradient_gap(dY64, W64, B_o, P_h, N, M)
        assert 0.05 < want < 1.0                          # a real gap: these masks drop entries
        assert abs(got - want) <= 1e-2 * want, (got, want)
        gaps.append(want)
