"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- hand-worked cases, the paper's literal formulas where they
are unambiguous (no ties), invariants the paper states, closed forms, brute
force in a different formulation, and library routines."""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
NMS = [(2, 4), (1, 4), (4, 8), (2, 8), (1, 16)]   # the patterns of Table 5 / Table 6


def rng_of(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------------------
# independent formulations used as pins (numpy, different loop structure)
# ----------------------------------------------------------------------------
def brute_topn_rows(W, N, M):
    """Stable sort of each group by descending magnitude; first N win."""
    I, J = W.shape
    g = np.abs(W).reshape(I, J // M, M)
    order = np.argsort(-g, axis=2, kind="stable")
    B = np.zeros_like(g, dtype=np.uint8)
    np.put_along_axis(B, order[:, :, :N], 1, axis=2)
    return B.reshape(I, J)


def literal_eq4(W, N, M):
    """Eq. (4) as printed: 0 where |w| < N-th largest of the group, else 1."""
    I, J = W.shape
    g = np.abs(W).reshape(I, J // M, M)
    nth = np.sort(g, axis=2)[:, :, M - N][:, :, None]
    return (g >= nth).astype(np.uint8).reshape(I, J)


def literal_eq11(W, B, P, N, M):
    """Eq. (11) as printed, on (B.*W)[P,:] along columns."""
    Wp, Bp = (W * B)[P, :], B[P, :]
    I, J = Wp.shape
    g = np.abs(Wp).reshape(I // M, M, J)
    nth = np.sort(g, axis=1)[:, M - N, :][:, None, :]
    out = np.where(g < nth, 0, Bp.reshape(I // M, M, J))
    return out.reshape(I, J).astype(np.uint8)


def brute_scores(B, perms, N, M):
    out = []
    for P in perms:
        Bp = B[P, :].astype(np.int64)
        cnt = Bp.reshape(B.shape[0] // M, M, B.shape[1]).sum(axis=1)
        out.append(int((cnt <= N).sum()))
    return np.array(out, dtype=np.int64)


# ----------------------------------------------------------------------------
# O1 forward mask
# ----------------------------------------------------------------------------
def _read_cases(name, widths):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            parts = [p.split() for p in line.split("|")]
            assert [len(p) for p in parts] == widths, line
            rows.append(parts)
    return rows


def test_forward_hand_cases():
    for w, b in _read_cases("topn_2of4_hand_cases.txt", [4, 4]):
        W = np.array([[float(x) for x in w]])
        want = np.array([[int(x) for x in b]], dtype=np.uint8)
        got = oracle.forward_mask(W, 2, 4)
        assert (got == want).all(), (w, got, want)


@pytest.mark.parametrize("N,M", NMS)
def test_forward_exactly_n_and_order(N, M):
    r = rng_of(11)
    W = r.standard_normal((24, 16 * M))
    W[3] = np.round(W[3] * 2) / 2          # many ties
    W[4] = 0.0
    W[5] = 1.0
    B = oracle.forward_mask(W, N, M)
    g = B.reshape(24, -1, M)
    assert (g.sum(axis=2) == N).all()                        # Eq. (2), exactly N
    a = np.abs(W).reshape(24, -1, M)
    for i, q in itertools.product(range(24), range(g.shape[1])):
        kept = [m for m in range(M) if g[i, q, m]]
        drop = [m for m in range(M) if not g[i, q, m]]
        for k_ in kept:
            for d in drop:
                assert a[i, q, k_] > a[i, q, d] or (a[i, q, k_] == a[i, q, d] and k_ < d)
    assert (B == brute_topn_rows(W, N, M)).all()


@pytest.mark.parametrize("N,M", NMS)
def test_forward_equals_literal_eq4_without_ties(N, M):
    W = rng_of(12).standard_normal((32, 8 * M))
    assert (oracle.forward_mask(W, N, M) == literal_eq4(W, N, M)).all()


def test_forward_scale_and_sign_invariance():
    W = rng_of(13).standard_normal((16, 64))
    W[2] = np.round(W[2])
    B = oracle.forward_mask(W, 2, 4)
    for a in (0.25, 8.0, -1.0, -4.0):
        assert (oracle.forward_mask(a * W, 2, 4) == B).all()


def test_forward_exhaustive_three_symbols():
    vecs = np.array(list(itertools.product([-1.0, 0.0, 2.0], repeat=4)))
    assert vecs.shape == (81, 4)
    for N in (1, 2, 3):
        assert (oracle.forward_mask(vecs, N, 4) == brute_topn_rows(vecs, N, 4)).all()


def test_forward_groups_do_not_overlap_or_shift():
    # a large value at position j only ever influences its own group
    W = np.full((1, 16), 0.1)
    for j in range(16):
        V = W.copy()
        V[0, j] = 5.0
        B = oracle.forward_mask(V, 1, 4).reshape(4, 4)
        for g in range(4):
            want = np.zeros(4, dtype=np.uint8)
            want[j % 4 if g == j // 4 else 0] = 1
            assert (B[g] == want).all()


# ----------------------------------------------------------------------------
# O2 / O3 permutation scores and argmax
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("N,M", NMS)
def test_scores_brute_force_and_identity(N, M):
    r = rng_of(21)
    I, J = 8 * M, 6 * M
    W = r.standard_normal((I, J))
    B = oracle.forward_mask(W, N, M)
    perms = np.stack([np.arange(I)] + [r.permutation(I) for _ in range(7)]).astype(np.int32)
    s = oracle.perm_scores(B, perms, N, M)
    assert (s == brute_scores(B, perms, N, M)).all()
    direct = sum(int(B[k:k + M, l].sum() <= N) for k in range(0, I, M) for l in range(J))
    assert s[0] == direct
    assert ((0 <= s) & (s <= (I // M) * J)).all()


def test_scores_tiny_by_hand():
    # 4 rows, 4 columns, 2:4 along rows; columns' counts are known by eye
    B = np.array([[1, 1, 0, 0],
                  [1, 1, 0, 0],
                  [1, 0, 1, 0],
                  [0, 1, 0, 1]], dtype=np.uint8)
    # column sums: 3, 3, 1, 1 -> two eligible blocks for any order of the 4 rows
    for P in itertools.permutations(range(4)):
        assert oracle.perm_scores(B, np.array([P]), 2, 4)[0] == 2
    # 8 rows: pairing matters
    B8 = np.vstack([B, B])
    # identity: both blocks have sums (3,3,1,1) -> 4 eligible
    assert oracle.perm_scores(B8, np.array([np.arange(8)]), 2, 4)[0] == 4
    # rows {0,1,4,5} / {2,3,6,7}: sums (4,4,0,0) and (2,2,2,2) -> 2 + 4 = 6
    assert oracle.perm_scores(B8, np.array([[0, 1, 4, 5, 2, 3, 6, 7]]), 2, 4)[0] == 6


def test_scores_block_and_within_block_invariance():
    r = rng_of(22)
    I, J, N, M = 32, 24, 2, 4
    B = oracle.forward_mask(r.standard_normal((I, J)), N, M)
    P = r.permutation(I)
    base = oracle.perm_scores(B, P[None], N, M)[0]
    blocks = P.reshape(I // M, M)
    shuffled_blocks = blocks[r.permutation(I // M)].reshape(-1)
    within = np.stack([b[r.permutation(M)] for b in blocks]).reshape(-1)
    assert oracle.perm_scores(B, shuffled_blocks[None], N, M)[0] == base
    assert oracle.perm_scores(B, within[None], N, M)[0] == base


@pytest.mark.parametrize("N,M", NMS)
def test_scores_closed_form_identical_rows(N, M):
    r = rng_of(23)
    I, J = 12 * M, 10 * M
    row = oracle.forward_mask(r.standard_normal((1, J)), N, M)
    B = np.repeat(row, I, axis=0)
    perms = np.stack([r.permutation(I) for _ in range(5)])
    want = (I // M) * J * (M - N) // M
    assert (oracle.perm_scores(B, perms, N, M) == want).all()


@pytest.mark.parametrize("N,M,p", [(2, 4, 11 / 16), (1, 4, 189 / 256), (4, 8, 163 / 256)])
def test_scores_expectation_iid(N, M, p):
    # rows of a column block come from different rows of W => independent
    # Bernoulli(N/M) bits => P[eligible] = P[Binomial(M, N/M) <= N]
    r = rng_of(24)
    I, J = 256, 512
    B = oracle.forward_mask(r.standard_normal((I, J)), N, M)
    perms = np.stack([r.permutation(I) for _ in range(6)])
    s = oracle.perm_scores(B, perms, N, M)
    n = (I // M) * J
    sigma = np.sqrt(n * p * (1 - p))
    assert (np.abs(s - n * p) < 6 * sigma).all(), (s, n * p, sigma)


def test_scores_single_block_all_equal():
    r = rng_of(25)
    B = oracle.forward_mask(r.standard_normal((4, 64)), 2, 4)
    perms = np.array(list(itertools.permutations(range(4))))
    s = oracle.perm_scores(B, perms, 2, 4)
    assert (s == s[0]).all()


def test_argmax_first_of_equals():
    assert oracle.argmax_first([3, 9, 9, 1]) == 1
    assert oracle.argmax_first([7]) == 0
    assert oracle.argmax_first([5, 5, 5]) == 0
    assert oracle.argmax_first([1, 2, 3, 10]) == 3
    s = rng_of(26).integers(0, 50, size=200)
    assert oracle.argmax_first(s) == int(np.argmax(s))       # numpy: first max


# ----------------------------------------------------------------------------
# O4 backward mask
# ----------------------------------------------------------------------------
def test_backward_hand_cases():
    for w, b, want, elig in _read_cases("backward_block_hand_cases.txt", [4, 4, 4, 1]):
        W = np.array([[float(x)] for x in w])
        B = np.array([[int(x)] for x in b], dtype=np.uint8)
        Bbar, _ = oracle.backward_mask(W, B, None, 2, 4)
        assert (Bbar[:, 0] == [int(x) for x in want]).all(), (w, b, Bbar[:, 0])
        assert oracle.perm_scores(B, np.arange(4)[None], 2, 4)[0] == int(elig[0])


@pytest.mark.parametrize("N,M", NMS)
def test_backward_invariants_and_score_link(N, M):
    r = rng_of(31)
    I, J = 16 * M, 12 * M
    W = r.standard_normal((I, J))
    B = oracle.forward_mask(W, N, M)
    perms = np.stack([r.permutation(I) for _ in range(9)]).astype(np.int32)
    scores = oracle.perm_scores(B, perms, N, M)
    for c in range(perms.shape[0]):
        P = perms[c]
        Bbar, sel = oracle.backward_mask(W, B, P, N, M)
        Bp = B[P, :]
        assert (Bbar <= Bp).all()                                     # B = 0 => Bbar = 0
        blk = Bbar.reshape(I // M, M, J)
        assert (blk.sum(axis=1) <= N).all()                           # Eq. (7)
        assert (sel.reshape(I // M, M, J).sum(axis=1) == N).all()
        assert (Bbar == (sel & Bp)).all()
        same = (blk == Bp.reshape(I // M, M, J)).all(axis=1)
        already = Bp.reshape(I // M, M, J).sum(axis=1) <= N
        assert (same == already).all()                                # Sec. 3.3 motivation 1
        assert same.sum() == scores[c]                                # links O2 and O4


@pytest.mark.parametrize("N,M", NMS)
def test_backward_equals_literal_eq11_without_ties(N, M):
    r = rng_of(32)
    I, J = 8 * M, 5 * M
    W = r.standard_normal((I, J))
    B = oracle.forward_mask(W, N, M)
    P = r.permutation(I).astype(np.int32)
    Bbar, _ = oracle.backward_mask(W, B, P, N, M)
    assert (Bbar == literal_eq11(W, B, P, N, M)).all()
    # Eq. (9) is Eq. (11) at the identity
    B0, _ = oracle.backward_mask(W, B, None, N, M)
    B1, _ = oracle.backward_mask(W, B, np.arange(I, dtype=np.int32), N, M)
    assert (B0 == B1).all()
    assert (B0 == literal_eq11(W, B, np.arange(I), N, M)).all()


def test_backward_is_forward_rule_on_the_transpose():
    r = rng_of(33)
    I, J, N, M = 32, 20, 2, 4
    W = np.round(r.standard_normal((I, J)) * 2) / 2      # ties included
    B = oracle.forward_mask(W, N, M)
    P = r.permutation(I).astype(np.int32)
    Bbar, sel = oracle.backward_mask(W, B, P, N, M)
    masked_t = np.ascontiguousarray(((W * B)[P, :]).T)   # J x I, groups along rows
    sel_t = brute_topn_rows(masked_t, N, M)
    assert (sel == sel_t.T).all()
    assert (Bbar == (sel_t.T & B[P, :])).all()


def test_backward_uses_the_permutation_direction_gather():
    # one heavy row: it must land in the block where P places it
    I, J = 8, 4
    W = np.full((I, J), 0.01)
    W[6] = 10.0
    B = np.ones((I, J), dtype=np.uint8)
    P = np.array([6, 0, 1, 2, 3, 4, 5, 7], dtype=np.int32)   # permuted row 0 = original row 6
    Bbar, _ = oracle.backward_mask(W, B, P, 1, 4)
    assert (Bbar[0] == 1).all() and (Bbar[1:4] == 0).all()


# ----------------------------------------------------------------------------
# O5 compression and packing
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("N,M", NMS)
def test_compress_roundtrip(N, M):
    r = rng_of(41)
    I, J = 8 * M, 6 * M
    W = np.round(r.standard_normal((I, J)) * 4) / 4
    B = oracle.forward_mask(W, N, M)
    val, idx = oracle.compress_fwd(W, B, N, M)
    assert val.shape == (I, J // M * N)
    dense = np.zeros((I, J))
    for i in range(I):
        for s in range(val.shape[1]):
            dense[i, (s // N) * M + idx[i, s]] += val[i, s]
    assert (dense == W * B).all()
    ii = idx.reshape(I, J // M, N).astype(int)
    assert (np.diff(ii, axis=2) > 0).all() and (ii < M).all()

    P = r.permutation(I).astype(np.int32)
    Bbar, sel = oracle.backward_mask(W, B, P, N, M)
    valb, idxb = oracle.compress_bwd(W, B, P, N, M)
    assert valb.shape == (J, I // M * N)
    dense_t = np.zeros((J, I))
    for l in range(J):
        for s in range(valb.shape[1]):
            dense_t[l, (s // N) * M + idxb[l, s]] += valb[l, s]
    assert (dense_t == ((W[P, :] * Bbar).T)).all()
    jj = idxb.reshape(J, I // M, N).astype(int)
    assert (np.diff(jj, axis=2) > 0).all() and (jj < M).all()
    # positions are exactly the pre-AND selection
    selpos = np.zeros((J, I), dtype=np.uint8)
    for l in range(J):
        for s in range(valb.shape[1]):
            selpos[l, (s // N) * M + idxb[l, s]] = 1
    assert (selpos == sel.T).all()


def test_pack_bits_matches_numpy_packbits():
    r = rng_of(42)
    for cols in (32, 64, 148, 20, 1):
        bits = (r.random((5, cols)) < 0.5).astype(np.uint8)
        words = oracle.pack_bits(bits)
        pad = np.zeros((5, words.shape[1] * 32), dtype=np.uint8)
        pad[:, :cols] = bits
        ref = np.packbits(pad, axis=1, bitorder="little").view("<u4")
        assert (words == ref).all()


@pytest.mark.parametrize("M", [4, 8, 16])
def test_pack_index_fields(M):
    r = rng_of(43)
    b = {4: 2, 8: 3, 16: 4}[M]
    idx = r.integers(0, M, size=(3, 21)).astype(np.uint8)
    words = oracle.pack_index(idx, M)
    assert words.shape[1] == (21 * b + 31) // 32
    for row in range(3):
        big = 0
        for w in reversed(words[row].tolist()):
            big = (big << 32) | w
        for s in range(21):
            assert (big >> (s * b)) & (M - 1) == idx[row, s]
        assert big >> (21 * b) == 0


def test_pack_index_2of4_hand_word():
    # groups (0,1) (0,2) (0,3) (1,2) (1,3) (2,3) (0,1) (2,3): 4 bits each, first slot low
    idx = np.array([[0, 1, 0, 2, 0, 3, 1, 2, 1, 3, 2, 3, 0, 1, 2, 3]], dtype=np.uint8)
    nib = [0b0100, 0b1000, 0b1100, 0b1001, 0b1101, 0b1110, 0b0100, 0b1110]
    want = sum(n << (4 * g) for g, n in enumerate(nib))
    assert oracle.pack_index(idx, 4)[0, 0] == want


# ----------------------------------------------------------------------------
# O6 GEMMs
# ----------------------------------------------------------------------------
def test_gemms_against_library_matmul_and_each_other():
    r = rng_of(51)
    T, I, J, N, M = 9, 16, 24, 2, 4
    W, X, dY = r.standard_normal((I, J)), r.standard_normal((T, J)), r.standard_normal((T, I))
    B = oracle.forward_mask(W, N, M)
    P = r.permutation(I).astype(np.int32)
    Bbar, _ = oracle.backward_mask(W, B, P, N, M)
    Y = oracle.gemm_fwd_loops(X, W, B)
    assert np.allclose(Y, X @ (W * B).T, rtol=1e-13, atol=1e-13)
    assert np.allclose(Y, oracle.gemm_fwd(X, W, B), rtol=1e-13, atol=1e-13)
    dX = oracle.gemm_bwd_loops(dY, W, Bbar, P)
    # un-permuted equivalent: M_bwd[P[r]] = Bbar[r]
    Mb = np.zeros_like(Bbar)
    Mb[P] = Bbar
    assert np.allclose(dX, dY @ (W * Mb), rtol=1e-13, atol=1e-13)
    assert np.allclose(dX, oracle.gemm_bwd(dY, W, Bbar, P), rtol=1e-13, atol=1e-13)
    ts, cs = np.array([0, 3, 8, 8]), np.array([0, 5, 15, 2])
    assert np.allclose(oracle.gemm_fwd_at(X, W, B, ts, cs), Y[ts, cs], rtol=1e-13, atol=1e-13)
    assert np.allclose(oracle.gemm_bwd_at(dY, W, Bbar, P, ts, cs), dX[ts, cs], rtol=1e-13, atol=1e-13)


def test_backward_gemm_permutation_leaves_unmasked_gradient_unchanged():
    # Sec. 3.3: permuting rows of W and columns of g(Y) together changes nothing
    r = rng_of(52)
    T, I, J = 5, 12, 8
    W, dY = r.standard_normal((I, J)), r.standard_normal((T, I))
    ones = np.ones((I, J), dtype=np.uint8)
    base = dY @ W
    for _ in range(4):
        P = r.permutation(I).astype(np.int32)
        assert np.allclose(oracle.gemm_bwd_loops(dY, W, ones, P), base, rtol=1e-12, atol=1e-12)


def test_gemms_identity_inputs_read_back_masked_weights():
    r = rng_of(53)
    I, J, N, M = 8, 8, 2, 4
    W = r.standard_normal((I, J))
    B = oracle.forward_mask(W, N, M)
    Y = oracle.gemm_fwd_loops(np.eye(J), W, B)                 # Y = (B.*W)^T
    assert (Y == (W * B).T).all()
    Bbar, _ = oracle.backward_mask(W, B, None, N, M)
    dX = oracle.gemm_bwd_loops(np.eye(I), W, Bbar, None)       # dX = Bbar.*W  (Eq. 8)
    assert (dX == W * Bbar).all()


def test_whole_step_is_consistent():
    r = rng_of(54)
    T, I, J, N, M = 6, 16, 16, 2, 4
    W, X, dY = r.standard_normal((I, J)), r.standard_normal((T, J)), r.standard_normal((T, I))
    perms = np.stack([r.permutation(I) for _ in range(5)]).astype(np.int32)
    out = oracle.bimask_step(W, X, dY, perms, N, M)
    assert out["best"] == int(np.argmax(brute_scores(out["B"], perms, N, M)))
    assert (out["P"] == perms[out["best"]]).all()


def test_compress_completes_short_groups_with_lowest_zero_positions():
    # hand-worked: mask 0010 -> slots {0, 2}; mask 0000 -> {0, 1}; mask 1000 -> {0, 1}; 0001 -> {0, 3}
    W = np.array([[5.0, 6.0, 7.0, 8.0] * 4])
    B = np.array([[0, 0, 1, 0, 0, 0, 0, 0, 1, 0, 0, 0, 0, 0, 0, 1]], dtype=np.uint8)
    val, idx = oracle.compress_fwd(W, B, 2, 4)
    assert idx.tolist() == [[0, 2, 0, 1, 0, 1, 0, 3]]
    assert val.tolist() == [[0.0, 7.0, 0.0, 0.0, 5.0, 0.0, 0.0, 8.0]]


@pytest.mark.parametrize("N,M", NMS)
def test_backward_compress_equals_generic_rule_on_bbar(N, M):
    # the slots of the transposed backward operand (selection before the AND) are exactly
    # the ones of Bbar completed with the lowest zero positions
    r = rng_of(44)
    I, J = 8 * M, 3 * M
    W = np.round(r.standard_normal((I, J)) * 2) / 2
    W[r.random((I, J)) < 0.2] = 0.0
    B = oracle.forward_mask(W, N, M)
    P = r.permutation(I).astype(np.int32)
    Bbar, _ = oracle.backward_mask(W, B, P, N, M)
    valb, idxb = oracle.compress_bwd(W, B, P, N, M)
    val2, idx2 = oracle.compress_fwd(np.ascontiguousarray(W[P, :].T), np.ascontiguousarray(Bbar.T), N, M)
    assert (idxb == idx2).all() and (valb == val2).all()


# ----------------------------------------------------------------------------
# refinement of a permutation by proposed exchanges (Limitations: future work)
# ----------------------------------------------------------------------------
def _read_refine_case():
    rows, swaps, exp, perm = [], [], None, None
    for line in open(os.path.join(GOLDEN, "perm_refine_hand_case.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        v = [int(x) for x in t[1:]]
        if t[0] == "B":
            rows.append(v)
        elif t[0] == "S":
            swaps.append(v)
        elif t[0] == "E":
            exp = v
        elif t[0] == "P":
            perm = v
    return np.array(rows, dtype=np.uint8), np.array(swaps, dtype=np.int32), exp, perm


def test_refine_hand_case():
    B, swaps, exp, perm = _read_refine_case()
    P, before, after, kept = oracle.perm_refine(B, None, swaps, 2, 4)
    assert [before, after, kept] == exp
    assert P.tolist() == perm
    # the order of the proposals matters: "2 7" alone is dropped
    P1, b1, a1, k1 = oracle.perm_refine(B, None, swaps[:1], 2, 4)
    assert (P1.tolist(), b1, a1, k1) == (list(range(8)), 3, 3, 0)


@pytest.mark.parametrize("N,M", NMS)
def test_refine_invariants(N, M):
    r = rng_of(61)
    I, J = 6 * M, 5 * M
    B = oracle.forward_mask(r.standard_normal((I, J)), N, M)
    P0 = r.permutation(I).astype(np.int32)
    swaps = r.integers(0, I, size=(150, 2)).astype(np.int32)
    P, before, after, kept = oracle.perm_refine(B, P0, swaps, N, M)
    assert sorted(P.tolist()) == list(range(I))
    assert before == brute_scores(B, P0[None], N, M)[0]
    assert after == brute_scores(B, P[None], N, M)[0]
    assert after >= before + kept and kept <= len(swaps)      # every kept proposal gains at least one block
    assert (kept == 0) == (P.tolist() == P0.tolist())
    # no proposals / proposals inside one block / positions that do not exist: nothing changes
    for sw in (np.zeros((0, 2), np.int32),
               np.array([[k * M + a, k * M + b] for k in range(I // M) for a in range(M) for b in range(M)], np.int32),
               np.array([[-1, 0], [0, I], [I + 5, -3]], np.int32)):
        Q, b, a, k = oracle.perm_refine(B, P0, sw, N, M)
        assert Q.tolist() == P0.tolist() and b == a == before and k == 0
    # the input permutation is not modified
    assert sorted(P0.tolist()) == list(range(I))


def test_refine_reaches_a_local_optimum_and_never_beats_the_global_one():
    r = rng_of(62)
    N, M, I, J = 2, 4, 8, 12
    B = (r.random((I, J)) < 0.55).astype(np.uint8)
    pairs = np.array([(a, b) for a in range(I) for b in range(a + 1, I)], dtype=np.int32)
    P, before = np.arange(I, dtype=np.int32), None
    for _ in range(20):                                        # sweeps over all exchanges until one keeps nothing
        P, b, a, kept = oracle.perm_refine(B, P, pairs, N, M)
        before = b if before is None else before
        if kept == 0:
            break
    assert kept == 0
    here = brute_scores(B, P[None], N, M)[0]
    assert here == a >= before
    for x, y in pairs:                                         # no single exchange improves it
        Q = P.copy()
        Q[x], Q[y] = Q[y], Q[x]
        assert brute_scores(B, Q[None], N, M)[0] <= here
    # all 35 ways of splitting 8 rows into two blocks of 4
    best = max(brute_scores(B, np.array([list(c) + [i for i in range(I) if i not in c]]), N, M)[0]
               for c in itertools.combinations(range(I), 4) if 0 in c)
    assert here <= best


def test_is_permutation_by_cases():
    good = np.array([3, 0, 2, 1])
    assert oracle.is_permutation(good).tolist() == [1]
    bad = np.array([[0, 1, 2, 3], [0, 1, 1, 3], [0, 1, 2, 4], [-1, 1, 2, 3], [3, 2, 1, 0]])
    assert oracle.is_permutation(bad).tolist() == [1, 0, 0, 0, 1]
    for P in itertools.permutations(range(5)):
        assert oracle.is_permutation(np.array(P))[0] == 1
    assert oracle.is_permutation(np.array(list(itertools.product(range(3), repeat=3)))).sum() == 6   # 3! of 27 triples


# ---------------------------------------------------------------------------------------------
# Eq. (5): exact input gradient, and the gap of Eq. (10)'s approximation to it (Sec. 3.3)
# ---------------------------------------------------------------------------------------------
def test_grad_exact_is_the_masked_matmul():
    rng = np.random.default_rng(2101)
    T, I, J = 9, 12, 20
    W = rng.standard_normal((I, J))
    dY = rng.standard_normal((T, I))
    B = oracle.forward_mask(W, 2, 4)
    want = dY @ (W * B)                                   # g(Y) (B .* W): the plain definition
    assert np.allclose(oracle.grad_exact_loops(dY, W, B), want, rtol=0, atol=1e-12)
    assert np.allclose(oracle.grad_exact(dY, W, B), want, rtol=0, atol=1e-12)
    # a one-hot g(Y) reads back row i of the masked weights; a transposed operand would read a column
    e = np.zeros((1, I)); e[0, 5] = 1.0
    assert (oracle.grad_exact_loops(e, W, B)[0] == (W * B)[5]).all()


def test_gradient_gap_hand_case():
    vals = {}
    with open(os.path.join(GOLDEN, "gradient_gap_hand_case.txt")) as f:
        for line in f:
            if line.startswith("#") or "|" not in line:
                continue
            k, v = line.split("|")
            vals[k.strip()] = np.array([float(x) for x in v.split()])
    W = np.array([[4, 3, 1, 0], [2, 0, 5, 1], [1, 0, 2, 6], [3, 1, 0, 2]], dtype=np.float64)
    B = oracle.forward_mask(W, 2, 4)
    assert B.tolist() == [[1, 1, 0, 0], [1, 0, 1, 0], [0, 0, 1, 1], [1, 0, 0, 1]]
    dY = np.ones((1, 4))
    Bbar, _ = oracle.backward_mask(W, B, None, 2, 4)
    assert (oracle.grad_exact_loops(dY, W, B)[0] == vals["exact"]).all()
    assert (oracle.gemm_bwd_loops(dY, W, Bbar, None)[0] == vals["approx"]).all()
    want = float(vals["gap_num"][0]) / np.sqrt(float(vals["gap_den2"][0]))
    assert abs(oracle.gradient_gap(dY, W, B, None, 2, 4) - want) < 1e-15
    e0 = np.array([[1.0, 0, 0, 0]])
    assert oracle.gradient_gap(e0, W, B, None, 2, 4) == 0.0


@pytest.mark.parametrize("N,M", NMS)
def test_gradient_gap_is_zero_when_every_block_is_eligible(N, M):
    # every column block of B[P,:] already holds at most N ones -> Bbar == B[P,:] (Sec. 3.3, motivation 1)
    # -> Eq. (10) reproduces Eq. (5) exactly, whatever P is
    rng = np.random.default_rng(2200 + M)
    I, J, T = 4 * M, 6 * M, 5
    B = np.zeros((I, J), dtype=np.uint8)
    P = rng.permutation(I).astype(np.int32)
    for k in range(I // M):
        for l in range(J):
            on = rng.choice(M, size=rng.integers(0, N + 1), replace=False)
            B[P[k * M + on], l] = 1
    W = rng.standard_normal((I, J))
    dY = rng.standard_normal((T, I))
    assert oracle.perm_scores(B, P, N, M)[0] == (I // M) * J
    assert oracle.gradient_gap(dY, W, B, P, N, M) < 1e-14
    # and it is positive as soon as one block loses an entry
    B2 = B.copy()
    B2[P[:M], 0] = 1
    assert oracle.gradient_gap(dY, W, B2, P, N, M) > 1e-6


def test_relative_gap_definition():
    rng = np.random.default_rng(2301)
    a, b = rng.standard_normal((7, 5)), rng.standard_normal((7, 5))
    assert abs(oracle.relative_gap(a, b) - np.linalg.norm(a - b) / np.linalg.norm(b)) < 1e-14
    assert oracle.relative_gap(b, b) == 0.0
    assert oracle.relative_gap(np.zeros((2, 2)), np.zeros((2, 2))) == 0.0
