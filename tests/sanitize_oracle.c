/*
 * Driver for a sanitizer build of the fp64 oracle: compiles oracle/mcf_oracle.c into this
 * translation unit (so the very same loops run under -fsanitize=address,undefined) and calls
 * every entry point on small cases that touch the edges of its indexing: distinct extents,
 * a K-contiguous B handed over by strides, padded rows, N = 0, selected rows, the
 * intermediate row and the chain of three GEMMs.  Results are checked against a flat
 * brute-force sum written here.  Exit status 0 = every case matched and no sanitizer report.
 * Test infrastructure only (run by tests/test_oracle_sanitized.py).
 */
#include <stdio.h>
#include <string.h>

#include "../oracle/mcf_oracle.c"

static double val(int t, int64_t i) { return (double)((int)((i * 7 + t * 3) % 9) - 4); }

static int check_plain(int64_t b, int64_t M, int64_t K, int64_t N, int64_t L, int b_kcontig, int64_t pad)
{
    /* A [b,M,K+pad], B [b,K,N+pad] or [b,N,K+pad], D [b,N,L+pad]: padded rows, exact extents */
    const int64_t sa[3] = {M * (K + pad), K + pad, 1};
    int64_t sb[3];
    if (b_kcontig) { sb[0] = N * (K + pad); sb[1] = 1; sb[2] = K + pad; }
    else { sb[0] = K * (N + pad); sb[1] = N + pad; sb[2] = 1; }
    const int64_t sd[3] = {N * (L + pad), L + pad, 1};
    const int64_t na = b * sa[0], nb = b * sb[0], nd = b * sd[0];
    double *A = malloc(sizeof(double) * (size_t)(na > 0 ? na : 1));
    double *B = malloc(sizeof(double) * (size_t)(nb > 0 ? nb : 1));
    double *D = malloc(sizeof(double) * (size_t)(nd > 0 ? nd : 1));
    double *E = malloc(sizeof(double) * (size_t)(b * M * L > 0 ? b * M * L : 1));
    for (int64_t i = 0; i < na; ++i) A[i] = val(1, i);
    for (int64_t i = 0; i < nb; ++i) B[i] = val(2, i);
    for (int64_t i = 0; i < nd; ++i) D[i] = val(3, i);
    mcf_oracle_chain(b, M, K, N, L, A, sa, B, sb, D, sd, 0, 1.0, E);
    int bad = 0;
    for (int64_t x = 0; x < b; ++x)
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < L; ++j) {
                double s = 0.0;
                for (int64_t n = 0; n < N; ++n) {
                    double c = 0.0;
                    for (int64_t k = 0; k < K; ++k)
                        c += A[x * sa[0] + i * sa[1] + k] * B[x * sb[0] + k * sb[1] + n * sb[2]];
                    s += c * D[x * sd[0] + n * sd[1] + j];
                }
                if (E[(x * M + i) * L + j] != s) bad = 1;
            }
    /* selected rows: the last row of the last batch and the first row of the first */
    if (b > 0 && M > 0) {
        const int64_t bi[4] = {b - 1, M - 1, 0, 0};
        double *R = malloc(sizeof(double) * (size_t)(2 * L > 0 ? 2 * L : 1));
        mcf_oracle_chain_rows(b, M, K, N, L, A, sa, B, sb, D, sd, 0, 1.0, 2, bi, R);
        for (int64_t j = 0; j < L; ++j)
            if (R[j] != E[((b - 1) * M + M - 1) * L + j] || R[L + j] != E[j]) bad = 1;
        free(R);
    }
    free(A); free(B); free(D); free(E);
    return bad;
}

static int check_softmax_and_chain3(void)
{
    enum { b = 2, M = 3, K = 4, N = 5, L = 2, P = 3 };
    double A[b * M * K], B[b * K * N], D[b * N * L], F[b * L * P], E[b * M * L], G[b * M * P], row[N];
    const int64_t sa[3] = {M * K, K, 1}, sb[3] = {K * N, N, 1}, sd[3] = {N * L, L, 1}, sf[3] = {L * P, P, 1};
    for (int i = 0; i < b * M * K; ++i) A[i] = 0.25 * val(1, i);
    for (int i = 0; i < b * K * N; ++i) B[i] = 0.25 * val(2, i);
    for (int i = 0; i < b * N * L; ++i) D[i] = val(3, i);
    for (int i = 0; i < b * L * P; ++i) F[i] = val(4, i);
    int bad = 0;
    mcf_oracle_chain(b, M, K, N, L, A, sa, B, sb, D, sd, 1, 0.5, E);
    for (int x = 0; x < b; ++x)
        for (int i = 0; i < M; ++i) {
            mcf_oracle_intermediate_row(b, M, K, N, L, A, sa, B, sb, D, sd, 1, 0.5, x, i, row);
            double sum = 0.0;
            for (int n = 0; n < N; ++n) sum += row[n];
            if (fabs(sum - 1.0) > 1e-14) bad = 1;
            for (int j = 0; j < L; ++j) {
                double s = 0.0;
                for (int n = 0; n < N; ++n) s += row[n] * D[x * sd[0] + n * sd[1] + j];
                if (fabs(s - E[(x * M + i) * L + j]) > 1e-14) bad = 1;
            }
        }
    /* causal mask: every offset from "sees nothing" to "sees everything"; the row sums of what a
     * row sees are checked through a D of ones */
    {
        double ones[b * N * L], Ec[b * M * L];
        for (int i = 0; i < b * N * L; ++i) ones[i] = 1.0;
        for (int off = -M - 1; off <= N + 1; ++off) {
            mcf_oracle_chain_causal(b, M, K, N, L, A, sa, B, sb, ones, sd, 0.5, off, Ec);
            for (int x = 0; x < b; ++x)
                for (int i = 0; i < M; ++i)
                    for (int j = 0; j < L; ++j) {
                        const double want = (i + off >= 0) ? 1.0 : 0.0;
                        if (fabs(Ec[(x * M + i) * L + j] - want) > 1e-14) bad = 1;
                    }
        }
    }
    mcf_oracle_chain3(b, M, K, N, L, A, sa, B, sb, D, sd, 1, 0.5, P, F, sf, G);
    for (int x = 0; x < b; ++x)
        for (int i = 0; i < M; ++i)
            for (int q = 0; q < P; ++q) {
                double s = 0.0;
                for (int h = 0; h < L; ++h) s += E[(x * M + i) * L + h] * F[x * sf[0] + h * sf[1] + q];
                if (fabs(s - G[(x * M + i) * P + q]) > 1e-13) bad = 1;
            }
    return bad;
}

int main(void)
{
    int bad = 0;
    bad |= check_plain(2, 3, 4, 5, 2, 0, 0);
    bad |= check_plain(2, 3, 4, 5, 2, 1, 0);   /* B as [b,N,K] through strides          */
    bad |= check_plain(3, 5, 2, 7, 3, 0, 3);   /* padded rows                           */
    bad |= check_plain(3, 5, 2, 7, 3, 1, 3);
    bad |= check_plain(1, 1, 1, 1, 1, 0, 0);
    bad |= check_plain(2, 4, 3, 0, 2, 0, 0);   /* N = 0: E = 0, no row is ever indexed  */
    bad |= check_plain(0, 4, 3, 2, 2, 0, 0);   /* empty batch                           */
    bad |= check_plain(2, 0, 3, 2, 2, 0, 0);   /* no rows                               */
    bad |= check_softmax_and_chain3();
    printf(bad ? "MISMATCH\n" : "sanitized oracle: all cases match\n");
    return bad;
}
