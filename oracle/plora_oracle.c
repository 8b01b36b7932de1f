/*
 * CPU oracle for the packed multi-LoRA linear layer (forward and backward).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header, table or helper with
 * the HIP library; the two meet only in the tests, which feed both the same seeded inputs.
 *
 * What it computes (plain definition, written out; all arithmetic in fp64):
 *
 *   LoRA (paper section 2.1): a frozen weight W in R^{d x k} gets a trainable low-rank update
 *   made of A in R^{d x r} and B in R^{r x k}; merged form W + scale * (A B).  Row-vector
 *   convention, so one token x_t in R^d produces  y_t = x_t W + scale * (x_t A) B.
 *
 *   Packed LoRA (paper section 2.4, appendix C.2): tokens of several adapters are stacked along
 *   the sequence dimension; every token goes through the shared W, and the tokens of segment s
 *   go through the adapter a(s) of that segment only.  Per adapter the arithmetic is exactly
 *   that of ordinary LoRA.
 *
 *   Backward (appendix C.2, the four gradient cases), for upstream gradient dy:
 *     case 2 (input of the B projection):   g_t  = scale_k * dy_t B_k^T
 *     case 4 (input of the A projection):   dx_t = dy_t W^T + g_t A_k^T
 *     case 3 (weight of the A projection):  dA_k = sum over tokens t of adapter k of x_t^T g_t
 *     case 1 (weight of the B projection):  dB_k = scale_k * sum_t (x_t A_k)^T dy_t
 *   W is frozen and gets no gradient.
 *
 * Inputs are float arrays that already hold the rounded values the GPU sees (bf16 or fp32
 * numbers, both exactly representable in float); they are widened to double before any
 * arithmetic.  Outputs are double.  Loops are the definition itself: no blocking, no fusion,
 * no library calls.  OpenMP only spreads independent output rows over threads; every single
 * output element is summed by one thread, in index order, so results do not depend on the
 * thread count.
 *
 * Pins (tests/test_oracle_pins.py): zero B gives the base product exactly; a packed call
 * equals each adapter run alone; merged-weight identity against a numpy fp64 matmul; rank-1
 * closed form; central finite differences of <y, dy> for dx, dA, dB; zero-padded ranks;
 * doubling scale equals doubling B; exact small-integer cases; adapter id -1 and empty
 * segments.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int64_t T;                   /* tokens (rows of x)                                   */
    int64_t D;                   /* input features  d                                    */
    int64_t K;                   /* output features k                                    */
    int32_t n_seg;               /* number of segments                                   */
    int32_t n_adapters;          /* number of adapters                                   */
    const int32_t *seg_off;      /* [n_seg+1], seg_off[0]=0, seg_off[n_seg]=T, monotone  */
    const int32_t *seg_adapter;  /* [n_seg], adapter of each segment, -1 = base only     */
    const int32_t *rank;         /* [n_adapters]                                         */
    const float *scale;          /* [n_adapters], multiplies the low-rank product        */
    const float *x;              /* [T][D]                                               */
    const float *W;              /* [D][K]                                               */
    const float *const *A;       /* A[k] -> [D][rank[k]]                                 */
    const float *const *B;       /* B[k] -> [rank[k]][K]                                 */
} plora_oracle_problem;

enum { ORACLE_OK = 0, ORACLE_BAD_SEGMENTS = 1, ORACLE_BAD_ADAPTER = 2, ORACLE_BAD_ROW = 3,
       ORACLE_BAD_ARG = 4 };

int plora_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Checks that the segment table covers [0, T) with nondecreasing offsets and valid ids. */
int plora_oracle_check(const plora_oracle_problem *p)
{
    if (!p || p->T < 0 || p->D <= 0 || p->K <= 0 || p->n_seg < 0 || p->n_adapters < 0)
        return ORACLE_BAD_ARG;
    if (p->n_seg == 0)
        return p->T == 0 ? ORACLE_OK : ORACLE_BAD_SEGMENTS;
    if (p->seg_off[0] != 0 || p->seg_off[p->n_seg] != p->T)
        return ORACLE_BAD_SEGMENTS;
    for (int32_t s = 0; s < p->n_seg; ++s) {
        if (p->seg_off[s + 1] < p->seg_off[s])
            return ORACLE_BAD_SEGMENTS;
        int32_t k = p->seg_adapter[s];
        if (k < -1 || k >= p->n_adapters)
            return ORACLE_BAD_ADAPTER;
        if (k >= 0 && p->rank[k] <= 0)
            return ORACLE_BAD_ADAPTER;
    }
    return ORACLE_OK;
}

/* Segment that holds token t, found by scanning the table from the front. */
static int32_t segment_of(const plora_oracle_problem *p, int64_t t)
{
    for (int32_t s = 0; s < p->n_seg; ++s)
        if (t >= p->seg_off[s] && t < p->seg_off[s + 1])
            return s;
    return -1;
}

/* h[j] = sum_i x_t[i] * A_k[i][j]   (the low-rank activation of token t) */
static void low_rank_activation(const plora_oracle_problem *p, int64_t t, int32_t k, double *h)
{
    const int32_t r = p->rank[k];
    const float *xt = p->x + t * p->D;
    const float *Ak = p->A[k];
    for (int32_t j = 0; j < r; ++j) {
        double acc = 0.0;
        for (int64_t i = 0; i < p->D; ++i)
            acc += (double)xt[i] * (double)Ak[i * r + j];
        h[j] = acc;
    }
}

/* g[j] = scale_k * sum_n dy_t[n] * B_k[j][n]   (gradient case 2) */
static void low_rank_gradient(const plora_oracle_problem *p, const float *dy, int64_t t,
                              int32_t k, double *g)
{
    const int32_t r = p->rank[k];
    const float *dyt = dy + t * p->K;
    const float *Bk = p->B[k];
    for (int32_t j = 0; j < r; ++j) {
        double acc = 0.0;
        for (int64_t n = 0; n < p->K; ++n)
            acc += (double)dyt[n] * (double)Bk[(int64_t)j * p->K + n];
        g[j] = (double)p->scale[k] * acc;
    }
}

/*
 * Forward for the listed tokens.  For list position q and token t = rows[q]:
 *   h_out[q][0..r) = x_t A_k                 (columns r..h_pitch are set to 0; all 0 if k = -1)
 *   y_out[q][n]    = sum_i x_t[i] W[i][n] + scale_k * sum_j h[j] B_k[j][n]
 * h_out may be NULL.  h_pitch must be at least the largest rank in use.
 */
int plora_oracle_fwd_rows(const plora_oracle_problem *p, int64_t n_rows, const int64_t *rows,
                          int32_t h_pitch, double *h_out, double *y_out)
{
    int rc = plora_oracle_check(p);
    if (rc)
        return rc;
    if (n_rows < 0 || (n_rows > 0 && (!rows || !y_out)))
        return ORACLE_BAD_ARG;
    for (int64_t q = 0; q < n_rows; ++q)
        if (rows[q] < 0 || rows[q] >= p->T)
            return ORACLE_BAD_ROW;
    for (int32_t k = 0; k < p->n_adapters; ++k)
        if (h_out && p->rank[k] > h_pitch)
            return ORACLE_BAD_ARG;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < n_rows; ++q) {
        const int64_t t = rows[q];
        const int32_t s = segment_of(p, t);
        const int32_t k = p->seg_adapter[s];
        const float *xt = p->x + t * p->D;
        double *y = y_out + q * p->K;

        for (int64_t n = 0; n < p->K; ++n)
            y[n] = 0.0;
        for (int64_t i = 0; i < p->D; ++i) {
            const double xi = (double)xt[i];
            const float *Wi = p->W + i * p->K;
            for (int64_t n = 0; n < p->K; ++n)
                y[n] += xi * (double)Wi[n];
        }

        double *h = NULL;
        if (k >= 0) {
            const int32_t r = p->rank[k];
            h = (double *)malloc(sizeof(double) * (size_t)r);
            low_rank_activation(p, t, k, h);
            const float *Bk = p->B[k];
            for (int64_t n = 0; n < p->K; ++n) {
                double acc = 0.0;
                for (int32_t j = 0; j < r; ++j)
                    acc += h[j] * (double)Bk[(int64_t)j * p->K + n];
                y[n] += (double)p->scale[k] * acc;
            }
        }
        if (h_out) {
            double *ho = h_out + q * (int64_t)h_pitch;
            for (int32_t j = 0; j < h_pitch; ++j)
                ho[j] = (k >= 0 && j < p->rank[k]) ? h[j] : 0.0;
        }
        free(h);
    }
    return ORACLE_OK;
}

/*
 * Backward with respect to the layer input, for the listed tokens:
 *   g_out[q][0..r) = scale_k * dy_t B_k^T                          (case 2; may be NULL)
 *   dx_out[q][i]   = sum_n dy_t[n] W[i][n] + sum_j g[j] A_k[i][j]  (case 4)
 */
int plora_oracle_bwd_rows(const plora_oracle_problem *p, const float *dy, int64_t n_rows,
                          const int64_t *rows, int32_t g_pitch, double *g_out, double *dx_out)
{
    int rc = plora_oracle_check(p);
    if (rc)
        return rc;
    if (n_rows < 0 || (n_rows > 0 && (!rows || !dx_out || !dy)))
        return ORACLE_BAD_ARG;
    for (int64_t q = 0; q < n_rows; ++q)
        if (rows[q] < 0 || rows[q] >= p->T)
            return ORACLE_BAD_ROW;
    for (int32_t k = 0; k < p->n_adapters; ++k)
        if (g_out && p->rank[k] > g_pitch)
            return ORACLE_BAD_ARG;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < n_rows; ++q) {
        const int64_t t = rows[q];
        const int32_t s = segment_of(p, t);
        const int32_t k = p->seg_adapter[s];
        const float *dyt = dy + t * p->K;
        double *dx = dx_out + q * p->D;

        for (int64_t i = 0; i < p->D; ++i) {
            const float *Wi = p->W + i * p->K;
            double acc = 0.0;
            for (int64_t n = 0; n < p->K; ++n)
                acc += (double)dyt[n] * (double)Wi[n];
            dx[i] = acc;
        }

        double *g = NULL;
        if (k >= 0) {
            const int32_t r = p->rank[k];
            g = (double *)malloc(sizeof(double) * (size_t)r);
            low_rank_gradient(p, dy, t, k, g);
            const float *Ak = p->A[k];
            for (int64_t i = 0; i < p->D; ++i) {
                double acc = 0.0;
                for (int32_t j = 0; j < r; ++j)
                    acc += g[j] * (double)Ak[i * r + j];
                dx[i] += acc;
            }
        }
        if (g_out) {
            double *go = g_out + q * (int64_t)g_pitch;
            for (int32_t j = 0; j < g_pitch; ++j)
                go[j] = (k >= 0 && j < p->rank[k]) ? g[j] : 0.0;
        }
        free(g);
    }
    return ORACLE_OK;
}

/*
 * Weight gradients of adapter k, summed over every token of every segment that names k,
 * in token order:
 *   dA[i][j] = sum_t x_t[i] * g_t[j]                (case 3),  [D][r_k]
 *   dB[j][n] = scale_k * sum_t h_t[j] * dy_t[n]     (case 1),  [r_k][K]
 * An adapter without tokens gets zeros.
 */
int plora_oracle_grad_adapter(const plora_oracle_problem *p, const float *dy, int32_t k,
                              double *dA, double *dB)
{
    int rc = plora_oracle_check(p);
    if (rc)
        return rc;
    if (k < 0 || k >= p->n_adapters || !dy || !dA || !dB)
        return ORACLE_BAD_ARG;
    const int32_t r = p->rank[k];
    if (r > 256)
        return ORACLE_BAD_ARG;
    const int64_t D = p->D, K = p->K;

    /* tokens of adapter k, in order */
    int64_t n_tok = 0;
    for (int32_t s = 0; s < p->n_seg; ++s)
        if (p->seg_adapter[s] == k)
            n_tok += p->seg_off[s + 1] - p->seg_off[s];
    int64_t *tok = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_tok > 0 ? n_tok : 1));
    int64_t c = 0;
    for (int32_t s = 0; s < p->n_seg; ++s)
        if (p->seg_adapter[s] == k)
            for (int64_t t = p->seg_off[s]; t < p->seg_off[s + 1]; ++t)
                tok[c++] = t;

    double *h = (double *)malloc(sizeof(double) * (size_t)(n_tok > 0 ? n_tok * r : 1));
    double *g = (double *)malloc(sizeof(double) * (size_t)(n_tok > 0 ? n_tok * r : 1));
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < n_tok; ++q) {
        low_rank_activation(p, tok[q], k, h + q * r);
        low_rank_gradient(p, dy, tok[q], k, g + q * r);
    }

    /* Each output element is one sum over the adapter's tokens in token order; the rank index is
     * the innermost loop only so that x and dy are walked once per (column, token). */
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < D; ++i) {
        double *acc = dA + i * r;
        for (int32_t j = 0; j < r; ++j)
            acc[j] = 0.0;
        for (int64_t q = 0; q < n_tok; ++q) {
            const double xv = (double)p->x[tok[q] * D + i];
            for (int32_t j = 0; j < r; ++j)
                acc[j] += xv * g[q * r + j];
        }
    }

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < K; ++n) {
        double acc[256];
        for (int32_t j = 0; j < r; ++j)
            acc[j] = 0.0;
        for (int64_t q = 0; q < n_tok; ++q) {
            const double dv = (double)dy[tok[q] * K + n];
            for (int32_t j = 0; j < r; ++j)
                acc[j] += h[q * r + j] * dv;
        }
        for (int32_t j = 0; j < r; ++j)
            dB[(int64_t)j * K + n] = (double)p->scale[k] * acc[j];
    }

    free(h);
    free(g);
    free(tok);
    return ORACLE_OK;
}
