/*
 * CPU oracle for the Bi-Mask hot path (arXiv 2302.06058).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, single-threaded loops in double
 * precision, written from the paper's equations.  Nothing here is shared with,
 * included by, or derived from the HIP path, and the product never calls it:
 * only tests, the smoke check and the benchmark's cpu_baseline leg do.
 *
 * Conventions (zero-based, row-major):
 *   W     I x J   weights as exact doubles (bf16 / fp32 convert exactly)
 *   B     I x J   forward mask, one byte (0/1) per entry, N:M along rows (Eq. 2)
 *   P     I       row permutation, gather form: permuted row r is original row P[r]
 *   Bbar  I x J   backward mask in PERMUTED row coordinates, N:M along columns (Eq. 7)
 *
 * Readings where the paper's text leaves a choice:
 *   - Eq. (4)/(11) keep everything >= the N-th largest magnitude; with ties that can
 *     keep more than N and break Eq. (2)/(7).  Here exactly N positions are selected
 *     per group, the lowest index winning among equal magnitudes.
 *   - An "eligible N:M block" (Sec. 3.3, motivation 1; Alg. 1) is a block of M
 *     consecutive permuted rows in one column of (B .* W)[P,:] holding at most N
 *     entries of the forward mask.  It is counted on mask bits.
 *   - Eq. (10): g(Y) is permuted along its out-feature axis with the same P.
 *
 * Pins: every function below is checked in tests/test_oracle_pins.py against
 * closed forms, brute force and invariants the paper states.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Top-N of M by magnitude; among equal magnitudes the lower index ranks first.
 * sel[m] = 1 for exactly N positions.   (Eq. 4, with the tie reading above) */
static void select_top_n(const double *v, int M, int N, uint8_t *sel)
{
    for (int m = 0; m < M; ++m) {
        int ahead = 0;
        for (int q = 0; q < M; ++q) {
            if (q == m) continue;
            double a = fabs(v[q]), b = fabs(v[m]);
            if (a > b || (a == b && q < m)) ++ahead;
        }
        sel[m] = (uint8_t)(ahead < N);
    }
}

/* Eq. (4): forward mask, groups of M consecutive columns in each row. */
void oracle_forward_mask(const double *W, int64_t I, int64_t J, int N, int M, uint8_t *B)
{
    for (int64_t i = 0; i < I; ++i)
        for (int64_t j = 0; j < J; j += M)
            select_top_n(W + i * J + j, M, N, B + i * J + j);
}

/* Sec. 3.3 / Alg. 1: for each candidate, the number of column blocks of
 * (B .* W)[P,:] that already satisfy N:M, i.e. hold at most N mask entries. */
void oracle_perm_scores(const uint8_t *B, int64_t I, int64_t J, int N, int M,
                        const int32_t *perms, int K, int64_t *scores)
{
    for (int c = 0; c < K; ++c) {
        const int32_t *P = perms + (int64_t)c * I;
        int64_t eligible = 0;
        for (int64_t k = 0; k < I; k += M)
            for (int64_t l = 0; l < J; ++l) {
                int nnz = 0;
                for (int m = 0; m < M; ++m)
                    nnz += B[(int64_t)P[k + m] * J + l];
                if (nnz <= N) ++eligible;
            }
        scores[c] = eligible;
    }
}

/* Refinement of a permutation (the Limitations section leaves "a better permutation than a
 * random one" to future work; this is hill climbing on the objective Sec. 3.3 / Alg. 1 already
 * use).  Proposal t exchanges the entries at positions a_t and b_t of P; it is kept if and
 * only if the number of eligible blocks of the whole matrix grows strictly.  Proposals are
 * taken one after the other, each against the permutation the earlier ones left.  A
 * proposal naming a position outside [0, I) changes nothing.
 * score[0] = eligible blocks before, score[1] = after; *accepted = proposals kept.
 * Every proposal is scored by counting the whole matrix again: no shortcut. */
void oracle_perm_refine(const uint8_t *B, int64_t I, int64_t J, int N, int M, int32_t *P,
                        const int32_t *swaps, int64_t S, int64_t *score, int64_t *accepted)
{
    int64_t cur;
    oracle_perm_scores(B, I, J, N, M, P, 1, &cur);
    score[0] = cur;
    *accepted = 0;
    for (int64_t t = 0; t < S; ++t) {
        const int64_t a = swaps[2 * t], b = swaps[2 * t + 1];
        if (a < 0 || a >= I || b < 0 || b >= I) continue;
        int32_t tmp = P[a]; P[a] = P[b]; P[b] = tmp;
        int64_t cand;
        oracle_perm_scores(B, I, J, N, M, P, 1, &cand);
        if (cand > cur) {
            cur = cand;
            ++*accepted;
        } else {
            tmp = P[a]; P[a] = P[b]; P[b] = tmp;                /* undo */
        }
    }
    score[1] = cur;
}

/* Alg. 1: the candidate with the most eligible blocks; first one among equals. */
int oracle_argmax(const int64_t *scores, int K)
{
    int best = 0;
    for (int c = 1; c < K; ++c)
        if (scores[c] > scores[best]) best = c;
    return best;
}

/* Eq. (11) (Eq. (9) when P is NULL = identity): backward mask on the permuted,
 * forward-masked weights.  sel_out (optional) receives the N selected positions of
 * every block before they are AND-ed with the forward mask. */
void oracle_backward_mask(const double *W, const uint8_t *B, int64_t I, int64_t J, int N, int M,
                          const int32_t *P, uint8_t *Bbar, uint8_t *sel_out)
{
    double v[64];
    uint8_t s[64];
    for (int64_t k = 0; k < I; k += M)
        for (int64_t l = 0; l < J; ++l) {
            for (int m = 0; m < M; ++m) {
                int64_t src = P ? (int64_t)P[k + m] : k + m;
                v[m] = B[src * J + l] ? W[src * J + l] : 0.0;
            }
            select_top_n(v, M, N, s);
            for (int m = 0; m < M; ++m) {
                int64_t src = P ? (int64_t)P[k + m] : k + m;
                Bbar[(k + m) * J + l] = (uint8_t)(s[m] && B[src * J + l]);
                if (sel_out) sel_out[(k + m) * J + l] = s[m];
            }
        }
}

/* Slot positions of one group given its mask bits: the ones (lowest first, at most N),
 * completed with the lowest-index zeros until N positions are chosen. */
static void slots_of_mask(const uint8_t *bits, int M, int N, uint8_t *chosen)
{
    int n = 0;
    memset(chosen, 0, (size_t)M);
    for (int m = 0; m < M && n < N; ++m)
        if (bits[m]) { chosen[m] = 1; ++n; }
    for (int m = 0; m < M && n < N; ++m)
        if (!bits[m]) { chosen[m] = 1; ++n; }
}

/* Compressed forward operand: per row and group N slots in ascending position order
 * with their positions.  A slot whose mask bit is 0 (only possible when the mask holds
 * fewer than N ones in that group) carries the value 0.  val: I x (J/M*N), idx: same. */
void oracle_compress_fwd(const double *W, const uint8_t *B, int64_t I, int64_t J, int N, int M,
                         double *val, uint8_t *idx)
{
    uint8_t chosen[64];
    int64_t S = J / M * N;
    for (int64_t i = 0; i < I; ++i)
        for (int64_t g = 0; g < J / M; ++g) {
            const uint8_t *bits = B + i * J + g * M;
            slots_of_mask(bits, M, N, chosen);
            int n = 0;
            for (int m = 0; m < M; ++m)
                if (chosen[m]) {
                    val[i * S + g * N + n] = bits[m] ? W[i * J + g * M + m] : 0.0;
                    idx[i * S + g * N + n] = (uint8_t)m;
                    ++n;
                }
        }
}

/* Compressed backward operand, TRANSPOSED: row l of the output is column l of
 * (B .* W)[P,:], its groups run along the permuted rows.  The N positions are the
 * selection before AND-ing with B; a selected position with B = 0 carries value 0.
 * val: J x (I/M*N), idx: same shape. */
void oracle_compress_bwd(const double *W, const uint8_t *B, const int32_t *P,
                         int64_t I, int64_t J, int N, int M, double *val, uint8_t *idx)
{
    double v[64];
    uint8_t s[64];
    int64_t S = I / M * N;
    for (int64_t l = 0; l < J; ++l)
        for (int64_t k = 0; k < I / M; ++k) {
            for (int m = 0; m < M; ++m) {
                int64_t src = P ? (int64_t)P[k * M + m] : k * M + m;
                v[m] = B[src * J + l] ? W[src * J + l] : 0.0;
            }
            select_top_n(v, M, N, s);
            int n = 0;
            for (int m = 0; m < M; ++m)
                if (s[m]) {
                    val[l * S + k * N + n] = v[m];
                    idx[l * S + k * N + n] = (uint8_t)m;
                    ++n;
                }
        }
}

/* Bit packing of a 0/1 byte matrix: ceil(cols/32) words per row, entry j is bit
 * (j % 32) of word (j / 32); unused high bits are zero. */
void oracle_pack_bits(const uint8_t *bits, int64_t rows, int64_t cols, uint32_t *words)
{
    int64_t wpr = (cols + 31) / 32;
    memset(words, 0, (size_t)(rows * wpr) * sizeof(uint32_t));
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t j = 0; j < cols; ++j)
            if (bits[r * cols + j])
                words[r * wpr + j / 32] |= (uint32_t)1 << (j % 32);
}

/* Packing of position indices: log2(M) bits per slot, slot s of a row sits at bit
 * offset s*log2(M) of that row's little-endian bit stream (bit q of the stream is
 * bit q%32 of word q/32); ceil(slots*log2(M)/32) words per row. */
void oracle_pack_index(const uint8_t *idx, int64_t rows, int64_t slots, int M, uint32_t *words)
{
    int b = 0;
    while ((1 << b) < M) ++b;
    int64_t wpr = (slots * b + 31) / 32;
    memset(words, 0, (size_t)(rows * wpr) * sizeof(uint32_t));
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t s = 0; s < slots; ++s)
            for (int q = 0; q < b; ++q) {           /* one bit at a time: fields may straddle words */
                int64_t off = s * b + q;
                if ((idx[r * slots + s] >> q) & 1)
                    words[r * wpr + off / 32] |= (uint32_t)1 << (off % 32);
            }
}

/* Eq. (3) in the T x J / T x I layout:  Y[t][i] = sum_j X[t][j] * (B .* W)[i][j]. */
void oracle_gemm_fwd(const double *X, const double *W, const uint8_t *B,
                     int64_t T, int64_t I, int64_t J, double *Y)
{
    for (int64_t t = 0; t < T; ++t)
        for (int64_t i = 0; i < I; ++i) {
            double acc = 0.0;
            for (int64_t j = 0; j < J; ++j)
                if (B[i * J + j]) acc += X[t * J + j] * W[i * J + j];
            Y[t * I + i] = acc;
        }
}

/* Eq. (10):  dX[t][j] = sum_r dY[t][P[r]] * (Bbar[r][j] ? W[P[r]][j] : 0). */
void oracle_gemm_bwd(const double *dY, const double *W, const uint8_t *Bbar, const int32_t *P,
                     int64_t T, int64_t I, int64_t J, double *dX)
{
    for (int64_t t = 0; t < T; ++t)
        for (int64_t j = 0; j < J; ++j) {
            double acc = 0.0;
            for (int64_t r = 0; r < I; ++r) {
                int64_t src = P ? (int64_t)P[r] : r;
                if (Bbar[r * J + j]) acc += dY[t * I + src] * W[src * J + j];
            }
            dX[t * J + j] = acc;
        }
}

/* Eq. (5), the exact input gradient the approximation of Eq. (8)/(10) stands in for:
 *   g(X)[t][j] = sum_i g(Y)[t][i] * (B .* W)[i][j]     (the paper writes (B .* W)^T * g(Y)). */
void oracle_grad_exact(const double *dY, const double *W, const uint8_t *B,
                       int64_t T, int64_t I, int64_t J, double *gX)
{
    for (int64_t t = 0; t < T; ++t)
        for (int64_t j = 0; j < J; ++j) {
            double acc = 0.0;
            for (int64_t i = 0; i < I; ++i)
                if (B[i * J + j]) acc += dY[t * I + i] * W[i * J + j];
            gX[t * J + j] = acc;
        }
}

/* Gradient gap (Sec. 3.3: what the permutation is chosen to shrink): the Frobenius norm of
 * approx - exact over the Frobenius norm of exact, both T x J.  0 / 0 counts as 0. */
double oracle_relative_gap(const double *approx, const double *exact, int64_t n)
{
    double num = 0.0, den = 0.0;
    for (int64_t q = 0; q < n; ++q) {
        double d = approx[q] - exact[q];
        num += d * d;
        den += exact[q] * exact[q];
    }
    if (den == 0.0) return num == 0.0 ? 0.0 : INFINITY;
    return sqrt(num / den);
}

/* The same two sums evaluated only at listed output coordinates (for sizes where
 * the full triple loop would take minutes). */
void oracle_gemm_fwd_at(const double *X, const double *W, const uint8_t *B,
                        int64_t I, int64_t J, const int64_t *ts, const int64_t *is, int64_t n,
                        double *out)
{
    (void)I;
    for (int64_t q = 0; q < n; ++q) {
        int64_t t = ts[q], i = is[q];
        double acc = 0.0;
        for (int64_t j = 0; j < J; ++j)
            if (B[i * J + j]) acc += X[t * J + j] * W[i * J + j];
        out[q] = acc;
    }
}

void oracle_gemm_bwd_at(const double *dY, const double *W, const uint8_t *Bbar, const int32_t *P,
                        int64_t I, int64_t J, const int64_t *ts, const int64_t *js, int64_t n,
                        double *out)
{
    for (int64_t q = 0; q < n; ++q) {
        int64_t t = ts[q], j = js[q];
        double acc = 0.0;
        for (int64_t r = 0; r < I; ++r) {
            int64_t src = P ? (int64_t)P[r] : r;
            if (Bbar[r * J + j]) acc += dY[t * I + src] * W[src * J + j];
        }
        out[q] = acc;
    }
}
