/*
 * Host sanitizer driver for the CPU oracle (test infrastructure).
 *
 * Built by tests/test_sanitizers.py together with oracle/bimask_oracle.c under
 * -fsanitize=address,undefined and run as a plain executable: every oracle function is
 * called on small buffers allocated at exactly their stated sizes, over shapes that include
 * the smallest legal ones (I = M, J = M, K = 1, no proposals), so that any read or write past
 * a buffer, any signed overflow or misaligned access stops the run.  A few invariants the
 * paper states (exactly N kept per forward group, Bbar <= B[P,:], at most N per column
 * block: Eq. (2), Eq. (7), Sec. 3.3) are checked on the way.  Exit status 0 = clean.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void oracle_forward_mask(const double *W, int64_t I, int64_t J, int N, int M, uint8_t *B);
void oracle_perm_scores(const uint8_t *B, int64_t I, int64_t J, int N, int M, const int32_t *perms, int K, int64_t *scores);
void oracle_perm_refine(const uint8_t *B, int64_t I, int64_t J, int N, int M, int32_t *P, const int32_t *swaps, int64_t S,
                        int64_t *score, int64_t *accepted);
int oracle_argmax(const int64_t *scores, int K);
void oracle_backward_mask(const double *W, const uint8_t *B, int64_t I, int64_t J, int N, int M, const int32_t *P,
                          uint8_t *Bbar, uint8_t *sel_out);
void oracle_compress_fwd(const double *W, const uint8_t *B, int64_t I, int64_t J, int N, int M, double *val, uint8_t *idx);
void oracle_compress_bwd(const double *W, const uint8_t *B, const int32_t *P, int64_t I, int64_t J, int N, int M,
                         double *val, uint8_t *idx);
void oracle_pack_bits(const uint8_t *bits, int64_t rows, int64_t cols, uint32_t *words);
void oracle_pack_index(const uint8_t *idx, int64_t rows, int64_t slots, int M, uint32_t *words);
void oracle_gemm_fwd(const double *X, const double *W, const uint8_t *B, int64_t T, int64_t I, int64_t J, double *Y);
void oracle_gemm_bwd(const double *dY, const double *W, const uint8_t *Bbar, const int32_t *P, int64_t T, int64_t I,
                     int64_t J, double *dX);
void oracle_grad_exact(const double *dY, const double *W, const uint8_t *B, int64_t T, int64_t I, int64_t J, double *gX);
double oracle_relative_gap(const double *approx, const double *exact, int64_t n);
void oracle_gemm_fwd_at(const double *X, const double *W, const uint8_t *B, int64_t I, int64_t J, const int64_t *ts,
                        const int64_t *is, int64_t n, double *out);
void oracle_gemm_bwd_at(const double *dY, const double *W, const uint8_t *Bbar, const int32_t *P, int64_t I, int64_t J,
                        const int64_t *ts, const int64_t *js, int64_t n, double *out);

static uint64_t state = 88172645463325252ull;
static uint32_t rnd(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return (uint32_t)(state >> 11); }
static double rndval(void) { return ((int)(rnd() % 17) - 8) * 0.25; }      /* few distinct magnitudes: ties, zeros */

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); exit(3); } } while (0)

static void one_shape(int64_t I, int64_t J, int64_t T, int N, int M, int K, int64_t S)
{
    double *W = malloc(sizeof(double) * I * J), *X = malloc(sizeof(double) * T * J), *dY = malloc(sizeof(double) * T * I);
    uint8_t *B = malloc(I * J), *Bbar = malloc(I * J), *sel = malloc(I * J);
    int32_t *perms = malloc(sizeof(int32_t) * K * I), *P = malloc(sizeof(int32_t) * I);
    int64_t *scores = malloc(sizeof(int64_t) * K);
    for (int64_t q = 0; q < I * J; ++q) W[q] = rndval();
    for (int64_t q = 0; q < T * J; ++q) X[q] = rndval();
    for (int64_t q = 0; q < T * I; ++q) dY[q] = rndval();
    for (int c = 0; c < K; ++c) {
        int32_t *p = perms + c * I;
        for (int64_t i = 0; i < I; ++i) p[i] = (int32_t)i;
        for (int64_t i = I - 1; i > 0; --i) { int64_t j = rnd() % (i + 1); int32_t t = p[i]; p[i] = p[j]; p[j] = t; }
    }
    oracle_forward_mask(W, I, J, N, M, B);
    for (int64_t i = 0; i < I; ++i)
        for (int64_t g = 0; g < J / M; ++g) {
            int n = 0;
            for (int m = 0; m < M; ++m) n += B[i * J + g * M + m];
            CHECK(n == N);                                              /* Eq. (2), exactly N */
        }
    oracle_perm_scores(B, I, J, N, M, perms, K, scores);
    int best = oracle_argmax(scores, K);
    CHECK(best >= 0 && best < K && scores[best] <= (I / M) * J);
    memcpy(P, perms + (int64_t)best * I, sizeof(int32_t) * I);
    for (int pass = 0; pass < 2; ++pass) {
        const int32_t *Pp = pass ? NULL : P;
        oracle_backward_mask(W, B, I, J, N, M, Pp, Bbar, pass ? NULL : sel);
        for (int64_t k = 0; k < I; k += M)
            for (int64_t l = 0; l < J; ++l) {
                int n = 0;
                for (int m = 0; m < M; ++m) {
                    int64_t src = Pp ? Pp[k + m] : k + m;
                    CHECK(Bbar[(k + m) * J + l] <= B[src * J + l]);     /* B = 0 => Bbar = 0 */
                    n += Bbar[(k + m) * J + l];
                }
                CHECK(n <= N);                                          /* Eq. (7) */
            }
        double *vb = malloc(sizeof(double) * J * (I / M * N)), *dX = malloc(sizeof(double) * T * J);
        uint8_t *ib = malloc(J * (I / M * N));
        oracle_compress_bwd(W, B, Pp, I, J, N, M, vb, ib);
        oracle_gemm_bwd(dY, W, Bbar, Pp, T, I, J, dX);
        int64_t ts[3] = {0, T - 1, T / 2}, cs[3] = {0, J - 1, J / 2};
        double at[3];
        oracle_gemm_bwd_at(dY, W, Bbar, Pp, I, J, ts, cs, 3, at);
        for (int q = 0; q < 3; ++q) CHECK(at[q] == dX[ts[q] * J + cs[q]]);
        free(vb); free(ib); free(dX);
    }
    {
        int64_t slots = J / M * N;
        double *vf = malloc(sizeof(double) * I * slots), *Y = malloc(sizeof(double) * T * I), *gX = malloc(sizeof(double) * T * J);
        uint8_t *xf = malloc(I * slots);
        int b = 0;
        while ((1 << b) < M) ++b;
        uint32_t *bw = malloc(sizeof(uint32_t) * I * ((J + 31) / 32)), *iw = malloc(sizeof(uint32_t) * I * ((slots * b + 31) / 32));
        oracle_compress_fwd(W, B, I, J, N, M, vf, xf);
        oracle_pack_bits(B, I, J, bw);
        oracle_pack_index(xf, I, slots, M, iw);
        oracle_gemm_fwd(X, W, B, T, I, J, Y);
        int64_t ts[2] = {0, T - 1}, is[2] = {I - 1, 0};
        double at[2];
        oracle_gemm_fwd_at(X, W, B, I, J, ts, is, 2, at);
        CHECK(at[0] == Y[ts[0] * I + is[0]] && at[1] == Y[ts[1] * I + is[1]]);
        oracle_grad_exact(dY, W, B, T, I, J, gX);
        CHECK(oracle_relative_gap(gX, gX, T * J) == 0.0);
        free(vf); free(xf); free(bw); free(iw); free(Y); free(gX);
    }
    {
        int32_t *swaps = malloc(sizeof(int32_t) * 2 * (S > 0 ? S : 1));
        for (int64_t t = 0; t < S; ++t) {
            swaps[2 * t] = (int32_t)(rnd() % (I + 2)) - 1;             /* -1 and I appear: positions that do not exist */
            swaps[2 * t + 1] = (int32_t)(rnd() % (I + 2)) - 1;
        }
        int64_t sc[2], kept;
        oracle_perm_refine(B, I, J, N, M, P, swaps, S, sc, &kept);
        CHECK(sc[1] >= sc[0] && kept >= 0 && kept <= S);
        free(swaps);
    }
    free(W); free(X); free(dY); free(B); free(Bbar); free(sel); free(perms); free(P); free(scores);
}

int main(void)
{
    static const int nm[][2] = {{2, 4}, {1, 4}, {4, 8}, {2, 8}, {1, 16}, {3, 4}, {15, 16}};
    for (unsigned q = 0; q < sizeof(nm) / sizeof(nm[0]); ++q) {
        int N = nm[q][0], M = nm[q][1];
        one_shape(M, M, 1, N, M, 1, 0);                 /* one group, one block, one candidate, no proposals */
        one_shape(3 * M, 5 * M, 7, N, M, 4, 25);
        one_shape(2 * M, 33 * M, 3, N, M, 2, 9);        /* bit rows that end inside a word */
    }
    puts("oracle sanitizer driver: clean");
    return 0;
}
