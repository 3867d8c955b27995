/*
 * fp64 CPU oracle for the fused MBCI operator chain of MCFuser (arXiv 2506.22169).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may include, link or call this
 * file; it exists so that the GPU kernels can be compared with a slow, obviously correct
 * statement of what the chain computes.  It shares no code with the HIP path.
 *
 * What is computed (Sec. III-A "GEMM chain C = A x B, E = C x D"; Sec. VI-B1 for the batched
 * form (batch,M,K)x(batch,K,N) then (batch,M,N)x(batch,N,H); Sec. VI-B2 for the
 * self-attention module, which inserts a softmax between the two GEMMs):
 *
 *   no softmax :  C[b,i,n] = sum_k A[b,i,k] * B[b,k,n]
 *                 E[b,i,j] = sum_n C[b,i,n] * D[b,n,j]
 *   softmax    :  S[b,i,n] = scale * sum_k A[b,i,k] * B[b,k,n]
 *                 P[b,i,n] = exp(S[b,i,n] - max_n S[b,i,:]) / sum_n exp(S[b,i,n] - max_n S[b,i,:])
 *                 E[b,i,j] = sum_n P[b,i,n] * D[b,n,j]
 *
 * The fused kernel reaches exactly this result up to rounding order (fusion and tiling only
 * reorder the sums), so the oracle is the definition written out: one full row of C (or S/P)
 * is materialised per (b,i), softmax is the two-pass form (max, then exp and sum), every sum
 * runs in index order in double.  No blocking, no fusion, no BLAS.
 *
 * The paper's H dimension is called L here.  The paper never states a softmax scale, axis or
 * mask: scale is an explicit argument, the axis is n (each row of C), there is no mask.
 *
 * Strides are in elements, {batch, row, col} per tensor, so the attention case passes the key
 * matrix stored [b,N,K] as B with strides {N*K, 1, K}.  E is written packed row-major [b,M,L]
 * (full variant) or [nrows,L] (rows variant).
 *
 * Pins (tests/test_oracle_pins.py): brute-force flat double sum on tiny integer inputs (bit
 * equality), (A.B).D == A.(B.D), identity/zero operands, closed-form softmax cases, numpy
 * float64 matmul/softmax as the library special case.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int64_t batch, M, K, N, L;
    const double *A, *B, *D;
    int64_t sa[3], sb[3], sd[3];
    int softmax;
    double scale;
    int causal;             /* softmax only: row i sees the columns n <= i + causal_offset */
    int64_t causal_offset;
} chain_t;

/* One output row E[b,i,0..L) into out[0..L); crow is scratch of N doubles.
 * With a causal mask (softmax only; not part of the paper: the usual attention convention) row i
 * sees the columns n <= i + causal_offset only: the softmax runs over those columns, the others
 * have P = 0, and a row that sees no column at all is a row of zeros. */
static void chain_row(const chain_t *p, int64_t b, int64_t i, double *crow, double *out)
{
    const double *Ab = p->A + b * p->sa[0] + i * p->sa[1];
    const double *Bb = p->B + b * p->sb[0];
    const double *Db = p->D + b * p->sd[0];

    for (int64_t n = 0; n < p->N; ++n) {
        double s = 0.0;
        for (int64_t k = 0; k < p->K; ++k)
            s += Ab[k * p->sa[2]] * Bb[k * p->sb[1] + n * p->sb[2]];
        crow[n] = s;
    }

    if (p->softmax) {
        int64_t seen = p->N; /* columns this row sees */
        if (p->causal) {
            seen = i + p->causal_offset + 1;
            if (seen < 0) seen = 0;
            if (seen > p->N) seen = p->N;
        }
        double mx = -INFINITY;
        for (int64_t n = 0; n < seen; ++n) {
            crow[n] *= p->scale;
            if (crow[n] > mx) mx = crow[n];
        }
        double den = 0.0;
        for (int64_t n = 0; n < seen; ++n) {
            crow[n] = exp(crow[n] - mx);
            den += crow[n];
        }
        for (int64_t n = 0; n < seen; ++n)
            crow[n] /= den;
        for (int64_t n = seen; n < p->N; ++n)
            crow[n] = 0.0;
    }

    for (int64_t j = 0; j < p->L; ++j) {
        double s = 0.0;
        for (int64_t n = 0; n < p->N; ++n)
            s += crow[n] * Db[n * p->sd[1] + j * p->sd[2]];
        out[j] = s;
    }
}

static void fill(chain_t *p, int64_t batch, int64_t M, int64_t K, int64_t N, int64_t L,
                 const double *A, const int64_t *sa, const double *B, const int64_t *sb,
                 const double *D, const int64_t *sd, int softmax, double scale)
{
    p->batch = batch; p->M = M; p->K = K; p->N = N; p->L = L;
    p->A = A; p->B = B; p->D = D;
    for (int t = 0; t < 3; ++t) { p->sa[t] = sa[t]; p->sb[t] = sb[t]; p->sd[t] = sd[t]; }
    p->softmax = softmax; p->scale = scale;
    p->causal = 0; p->causal_offset = 0;
}

/* Full tensor: E packed [batch, M, L].  Returns the number of threads used. */
int mcf_oracle_chain(int64_t batch, int64_t M, int64_t K, int64_t N, int64_t L,
                     const double *A, const int64_t *sa, const double *B, const int64_t *sb,
                     const double *D, const int64_t *sd, int softmax, double scale, double *E)
{
    chain_t p;
    fill(&p, batch, M, K, N, L, A, sa, B, sb, D, sd, softmax, scale);
    int threads = 1;
    const int64_t rows = batch * M;
#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        threads = omp_get_num_threads();
#endif
        double *crow = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
#pragma omp for schedule(static)
        for (int64_t r = 0; r < rows; ++r)
            chain_row(&p, r / M, r % M, crow, E + r * L);
        free(crow);
    }
    return threads;
}

/* Selected rows: bi holds nrows pairs (b, i); Erows packed [nrows, L]. */
int mcf_oracle_chain_rows(int64_t batch, int64_t M, int64_t K, int64_t N, int64_t L,
                          const double *A, const int64_t *sa, const double *B, const int64_t *sb,
                          const double *D, const int64_t *sd, int softmax, double scale,
                          int64_t nrows, const int64_t *bi, double *Erows)
{
    chain_t p;
    fill(&p, batch, M, K, N, L, A, sa, B, sb, D, sd, softmax, scale);
    int threads = 1;
#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        threads = omp_get_num_threads();
#endif
        double *crow = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
#pragma omp for schedule(static)
        for (int64_t r = 0; r < nrows; ++r)
            chain_row(&p, bi[2 * r], bi[2 * r + 1], crow, Erows + r * L);
        free(crow);
    }
    return threads;
}

/* The softmax'd (or plain) intermediate row itself, for the row-sum / shift-invariance pins:
 * writes P[b,i,0..N) (or C when softmax == 0). */
void mcf_oracle_intermediate_row(int64_t batch, int64_t M, int64_t K, int64_t N, int64_t L,
                                 const double *A, const int64_t *sa, const double *B,
                                 const int64_t *sb, const double *D, const int64_t *sd,
                                 int softmax, double scale, int64_t b, int64_t i, double *row)
{
    chain_t p;
    fill(&p, batch, M, K, N, L, A, sa, B, sb, D, sd, softmax, scale);
    double *out = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    chain_row(&p, b, i, row, out);
    free(out);
}

/*
 * Chain of three GEMMs (Sec. III-A: the tiling analysis carries over to longer chains of
 * compute-intensive operators): G[b,i,p] = sum_h E[b,i,h] * F[b,h,p] with E as above (the
 * softmax, if any, sits between the first two GEMMs).  One row of E is materialised per (b,i)
 * and nothing is rounded.  G packed [batch, M, P].  Returns the number of threads used.
 */
int mcf_oracle_chain3(int64_t batch, int64_t M, int64_t K, int64_t N, int64_t L,
                      const double *A, const int64_t *sa, const double *B, const int64_t *sb,
                      const double *D, const int64_t *sd, int softmax, double scale,
                      int64_t P, const double *F, const int64_t *sf, double *G)
{
    chain_t p;
    fill(&p, batch, M, K, N, L, A, sa, B, sb, D, sd, softmax, scale);
    int threads = 1;
    const int64_t rows = batch * M;
#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        threads = omp_get_num_threads();
#endif
        double *crow = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        double *erow = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
#pragma omp for schedule(static)
        for (int64_t r = 0; r < rows; ++r) {
            const int64_t b = r / M;
            chain_row(&p, b, r % M, crow, erow);
            const double *Fb = F + b * sf[0];
            for (int64_t q = 0; q < P; ++q) {
                double s = 0.0;
                for (int64_t h = 0; h < L; ++h)
                    s += erow[h] * Fb[h * sf[1] + q * sf[2]];
                G[r * P + q] = s;
            }
        }
        free(crow);
        free(erow);
    }
    return threads;
}

/*
 * The softmax chain under a causal mask (not in the paper; the convention of attention
 * kernels): row i of every batch sees the columns n <= i + causal_offset, i.e.
 *   P[b,i,n] = exp(S[b,i,n] - max) / sum   over those n,   P = 0 elsewhere,
 * with causal_offset = 0 the lower triangle and causal_offset = N - M the triangle aligned at
 * the last row and column; a row that sees nothing gives E = 0.  E packed [batch, M, L].
 */
int mcf_oracle_chain_causal(int64_t batch, int64_t M, int64_t K, int64_t N, int64_t L,
                            const double *A, const int64_t *sa, const double *B, const int64_t *sb,
                            const double *D, const int64_t *sd, double scale, int64_t causal_offset,
                            double *E)
{
    chain_t p;
    fill(&p, batch, M, K, N, L, A, sa, B, sb, D, sd, 1, scale);
    p.causal = 1;
    p.causal_offset = causal_offset;
    int threads = 1;
    const int64_t rows = batch * M;
#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        threads = omp_get_num_threads();
#endif
        double *crow = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
#pragma omp for schedule(static)
        for (int64_t r = 0; r < rows; ++r)
            chain_row(&p, r / M, r % M, crow, E + r * L);
        free(crow);
    }
    return threads;
}
