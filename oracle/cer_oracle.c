/*
 * CPU ORACLE -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * A plain, slow, obviously-correct implementation of what the CER / CSER path computes, written
 * from the paper (Wiedemann, Mueller, Samek: "Compact and Computationally Efficient Representation
 * of Deep Neural Networks").  Only the tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.  It shares no code, header, table or helper with the HIP library.
 *
 * Contents
 *   orc_encode / orc_free / orc_get_*   dense -> CER or CSER arrays      (Section III-A, format steps 1-4)
 *   orc_decode                          CER / CSER arrays -> dense       (Section III-A: M is uniquely
 *                                                                         reconstructible)
 *   orc_dot_cer / orc_dot_cser          group-sum product, fp64 sums     (Appendix A-C, Algorithms 3, 4;
 *                                                                         Section III-B prose steps 1-5;
 *                                                                         Appendix A-A1 for a non-zero
 *                                                                         most-frequent value)
 *   orc_dot_dense                       three-loop product, fp64 sums    (Algorithm 1)
 *   orc_csr_encode_count / orc_dot_csr  CSR comparator                   (Section III-A, Algorithm 2)
 *   orc_min_bits                        8/16/32-bit index width rule     (Section V, index arrays)
 *
 * All index arrays are exchanged as int64 so that the caller never has to know a width; widths are
 * reported separately by orc_min_bits.  Floating-point inputs are fp32 (the paper's element type),
 * every accumulation is fp64.
 *
 * Readings of the paper taken here (the paper is silent or its listing is garbled):
 *   - Omega is ordered by global occurrence count, highest first; equal counts keep the order of
 *     the caller's codebook; codebook values that never occur are left out.
 *   - Omega[0] is the most frequent value whatever it is, stored unshifted; the subtraction of
 *     Omega[0] happens inside the product.
 *   - Within a row, groups are emitted for rank 1, 2, ... ; CER emits an empty group (a repeated
 *     pointer) for an absent rank that is below the highest rank present in the row and nothing
 *     above it; CSER emits present ranks only and records the rank in OmegaI.
 *   - Inside a group column indices ascend.  All indices are 0-based.
 *   - Pointer arrays carry a leading 0: len(OmegaPtr) = groups + 1, len(rowPtr) = m + 1.
 *   - Algorithm 3 multiplies once per group after the inner loop and not at all for an empty group.
 *   - -0.0 is treated as +0.0 when a matrix element is matched against the codebook.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_E_NOT_IN_CODEBOOK (-1)
#define ORC_E_BAD_CODEBOOK (-2)
#define ORC_E_NOMEM (-3)
#define ORC_E_BAD_ARRAYS (-4)

typedef struct {
    int64_t m, n;
    int64_t K;        /* number of values that actually occur */
    int64_t nnz;      /* elements different from Omega[0] */
    int64_t G;        /* number of groups (CER: including empty ones) */
    int cser;
    float *omega;     /* K */
    int64_t *count;   /* K, occurrences of omega[k] */
    int64_t *colI;    /* nnz */
    int64_t *omegaPtr;/* G + 1 */
    int64_t *rowPtr;  /* m + 1 */
    int64_t *omegaI;  /* G (CSER only) */
} orc_matrix;

static float canon(float v) { return v == 0.0f ? 0.0f : v; } /* -0.0 -> +0.0 */

static int same_value(float a, float b) {
    uint32_t ua, ub;
    a = canon(a); b = canon(b);
    memcpy(&ua, &a, 4); memcpy(&ub, &b, 4);
    return ua == ub;
}

/* Section V: indices are unsigned and take the smallest of 8, 16 or 32 bits that holds them. */
int orc_min_bits(int64_t max_value) {
    if (max_value < 0) return 8;
    if (max_value <= 0xFF) return 8;
    if (max_value <= 0xFFFF) return 16;
    return 32;
}

void orc_free(orc_matrix *A) {
    if (!A) return;
    free(A->omega); free(A->count); free(A->colI); free(A->omegaPtr); free(A->rowPtr); free(A->omegaI);
    free(A);
}

/*
 * Section III-A, steps 1-4 of the CER description and the CSER paragraph.
 * W: m x n row-major fp32; codebook: Kc distinct finite values.
 */
int orc_encode(const float *W, int64_t m, int64_t n, const float *codebook, int64_t Kc, int cser,
               orc_matrix **out) {
    int64_t N = m * n;
    *out = NULL;
    for (int64_t a = 0; a < Kc; ++a) {
        if (!isfinite(codebook[a])) return ORC_E_BAD_CODEBOOK;
        for (int64_t b = 0; b < a; ++b)
            if (same_value(codebook[a], codebook[b])) return ORC_E_BAD_CODEBOOK;
    }

    /* symbol of every element, and how often each codebook value occurs (Section III: p_k = #(w_k)/N) */
    int32_t *sym = (int32_t *)malloc((size_t)(N > 0 ? N : 1) * sizeof(int32_t));
    int64_t *cnt = (int64_t *)calloc((size_t)(Kc > 0 ? Kc : 1), sizeof(int64_t));
    if (!sym || !cnt) { free(sym); free(cnt); return ORC_E_NOMEM; }
    for (int64_t i = 0; i < N; ++i) {
        int64_t k = 0;
        while (k < Kc && !same_value(W[i], codebook[k])) ++k;
        if (k == Kc) { free(sym); free(cnt); return ORC_E_NOT_IN_CODEBOOK; }
        sym[i] = (int32_t)k;
        cnt[k] += 1;
    }

    /* step 1: frequency-major order; selection of the largest remaining count, earliest codebook
       position first among equals; values with count 0 are not part of Omega */
    int64_t *order = (int64_t *)malloc((size_t)(Kc > 0 ? Kc : 1) * sizeof(int64_t));
    int64_t *rank_of = (int64_t *)malloc((size_t)(Kc > 0 ? Kc : 1) * sizeof(int64_t));
    char *used = (char *)calloc((size_t)(Kc > 0 ? Kc : 1), 1);
    int64_t K = 0;
    for (;;) {
        int64_t best = -1;
        for (int64_t k = 0; k < Kc; ++k)
            if (!used[k] && cnt[k] > 0 && (best < 0 || cnt[k] > cnt[best])) best = k;
        if (best < 0) break;
        used[best] = 1;
        rank_of[best] = K;
        order[K++] = best;
    }

    orc_matrix *A = (orc_matrix *)calloc(1, sizeof(orc_matrix));
    A->m = m; A->n = n; A->K = K; A->cser = cser;
    A->omega = (float *)malloc((size_t)(K > 0 ? K : 1) * sizeof(float));
    A->count = (int64_t *)malloc((size_t)(K > 0 ? K : 1) * sizeof(int64_t));
    for (int64_t k = 0; k < K; ++k) { A->omega[k] = canon(codebook[order[k]]); A->count[k] = cnt[order[k]]; }
    A->nnz = K > 0 ? N - A->count[0] : 0;

    A->colI = (int64_t *)malloc((size_t)(A->nnz > 0 ? A->nnz : 1) * sizeof(int64_t));
    /* at most K-1 groups per row */
    int64_t gmax = m * (K > 1 ? K - 1 : 0);
    A->omegaPtr = (int64_t *)malloc((size_t)(gmax + 1) * sizeof(int64_t));
    A->omegaI = (int64_t *)malloc((size_t)(gmax + 1) * sizeof(int64_t));
    A->rowPtr = (int64_t *)malloc((size_t)(m + 1) * sizeof(int64_t));

    int64_t nc = 0, ng = 0;
    A->omegaPtr[0] = 0;
    A->rowPtr[0] = 0;
    for (int64_t r = 0; r < m; ++r) {
        const int32_t *s = sym + r * n;
        int64_t kmax = 0; /* highest rank present in this row */
        for (int64_t c = 0; c < n; ++c) {
            int64_t rk = rank_of[s[c]];
            if (rk > kmax) kmax = rk;
        }
        for (int64_t k = 1; k <= kmax; ++k) {
            int64_t before = nc;
            for (int64_t c = 0; c < n; ++c)          /* step 2: ascending column order */
                if (rank_of[s[c]] == k) A->colI[nc++] = c;
            if (cser) {
                if (nc == before) continue;          /* CSER: present values only */
                A->omegaI[ng] = k;
            }
            A->omegaPtr[++ng] = nc;                  /* step 3: an unchanged pointer = value absent */
        }
        A->rowPtr[r + 1] = ng;                       /* step 4: rowPtr points into OmegaPtr */
    }
    A->G = ng;
    if (!cser) { free(A->omegaI); A->omegaI = NULL; }
    free(sym); free(cnt); free(order); free(rank_of); free(used);
    *out = A;
    return ORC_OK;
}

void orc_get_dims(const orc_matrix *A, int64_t *m, int64_t *n, int64_t *K, int64_t *nnz, int64_t *G) {
    *m = A->m; *n = A->n; *K = A->K; *nnz = A->nnz; *G = A->G;
}

void orc_get_arrays(const orc_matrix *A, float *omega, int64_t *count, int64_t *colI,
                    int64_t *omegaPtr, int64_t *rowPtr, int64_t *omegaI) {
    memcpy(omega, A->omega, (size_t)A->K * sizeof(float));
    memcpy(count, A->count, (size_t)A->K * sizeof(int64_t));
    memcpy(colI, A->colI, (size_t)A->nnz * sizeof(int64_t));
    memcpy(omegaPtr, A->omegaPtr, (size_t)(A->G + 1) * sizeof(int64_t));
    memcpy(rowPtr, A->rowPtr, (size_t)(A->m + 1) * sizeof(int64_t));
    if (A->cser && omegaI) memcpy(omegaI, A->omegaI, (size_t)A->G * sizeof(int64_t));
}

/*
 * Decode (Section III-A: the arrays determine M).  Every element starts as Omega[0]; group g of
 * row r overwrites its columns with Omega[rank], rank = position in the row + 1 (CER) or
 * OmegaI[g] (CSER, omegaI != NULL).
 */
int orc_decode(int64_t m, int64_t n, const float *omega, int64_t K, const int64_t *colI,
               const int64_t *omegaPtr, const int64_t *rowPtr, const int64_t *omegaI, float *W) {
    if (K < 1) return m * n == 0 ? ORC_OK : ORC_E_BAD_ARRAYS;
    for (int64_t i = 0; i < m * n; ++i) W[i] = omega[0];
    for (int64_t r = 0; r < m; ++r) {
        for (int64_t g = rowPtr[r]; g < rowPtr[r + 1]; ++g) {
            int64_t rank = omegaI ? omegaI[g] : g - rowPtr[r] + 1;
            if (rank < 1 || rank >= K) return ORC_E_BAD_ARRAYS;
            for (int64_t i = omegaPtr[g]; i < omegaPtr[g + 1]; ++i) {
                if (colI[i] < 0 || colI[i] >= n) return ORC_E_BAD_ARRAYS;
                W[r * n + colI[i]] = omega[rank];
            }
        }
    }
    return ORC_OK;
}

/* Appendix A-A1: constant c_out(l) = Omega[0] * sum_i X[i,l], added to every output of column l. */
static double dominant_offset(const float *omega, const float *X, int64_t n, int64_t L, int64_t l) {
    if (omega[0] == 0.0f) return 0.0;
    double t = 0.0;
    for (int64_t i = 0; i < n; ++i) t += (double)X[i * L + l];
    return (double)omega[0] * t;
}

/*
 * Algorithm 3 (CER) and Algorithm 4 (CSER), in the paper's loop order: input column l, row,
 * group, index.  y' sums the gathered inputs of one group; one multiplication per non-empty
 * group by (Omega[rank] - Omega[0]); rows are independent, so `threads` > 1 only splits the row
 * loop among OpenMP threads.
 * X: n x L row-major fp32; Y: m x L row-major fp64.
 */
static void dot_grouped(int64_t m, int64_t n, const float *omega, const int64_t *colI,
                        const int64_t *omegaPtr, const int64_t *rowPtr, const int64_t *omegaI,
                        const float *X, int64_t L, double *Y, int threads) {
    for (int64_t l = 0; l < L; ++l) {
        double c_out = dominant_offset(omega, X, n, L, l);
#pragma omp parallel for schedule(static) num_threads(threads) if (threads > 1)
        for (int64_t r = 0; r < m; ++r) {
            double y = 0.0;
            for (int64_t g = rowPtr[r]; g < rowPtr[r + 1]; ++g) {
                int64_t w_start = omegaPtr[g], w_end = omegaPtr[g + 1];
                if (w_start == w_end) continue;              /* value absent in this row */
                double y1 = 0.0;
                for (int64_t i = w_start; i < w_end; ++i) y1 += (double)X[colI[i] * L + l];
                int64_t rank = omegaI ? omegaI[g] : g - rowPtr[r] + 1;
                y += y1 * ((double)omega[rank] - (double)omega[0]);
            }
            Y[r * L + l] = y + c_out;
        }
    }
}

void orc_dot_cer(int64_t m, int64_t n, const float *omega, const int64_t *colI,
                 const int64_t *omegaPtr, const int64_t *rowPtr, const float *X, int64_t L,
                 double *Y, int threads) {
    dot_grouped(m, n, omega, colI, omegaPtr, rowPtr, NULL, X, L, Y, threads);
}

void orc_dot_cser(int64_t m, int64_t n, const float *omega, const int64_t *colI,
                  const int64_t *omegaI, const int64_t *omegaPtr, const int64_t *rowPtr,
                  const float *X, int64_t L, double *Y, int threads) {
    dot_grouped(m, n, omega, colI, omegaPtr, rowPtr, omegaI, X, L, Y, threads);
}

/* Algorithm 1: the standard three-loop product, fp64 accumulation. */
void orc_dot_dense(const float *A, int64_t m, int64_t n, const float *X, int64_t L, double *Y,
                   int threads) {
    for (int64_t l = 0; l < L; ++l) {
#pragma omp parallel for schedule(static) num_threads(threads) if (threads > 1)
        for (int64_t r = 0; r < m; ++r) {
            double y = 0.0;
            for (int64_t c = 0; c < n; ++c) y += (double)A[r * n + c] * (double)X[c * L + l];
            Y[r * L + l] = y;
        }
    }
}

/* sum_c |A[r,c]| |X[c,l]| in fp64: the scale of the rounding-error bound used by the parity tests. */
void orc_abs_dot_dense(const float *A, int64_t m, int64_t n, const float *X, int64_t L, double *S,
                       int threads) {
    for (int64_t l = 0; l < L; ++l) {
#pragma omp parallel for schedule(static) num_threads(threads) if (threads > 1)
        for (int64_t r = 0; r < m; ++r) {
            double y = 0.0;
            for (int64_t c = 0; c < n; ++c) y += fabs((double)A[r * n + c]) * fabs((double)X[c * L + l]);
            S[r * L + l] = y;
        }
    }
}

/* CSR (Section III-A): non-zero values in row-major order, their columns, row pointers. */
int64_t orc_csr_encode(const float *W, int64_t m, int64_t n, float *val, int64_t *colI, int64_t *rowPtr) {
    int64_t k = 0;
    rowPtr[0] = 0;
    for (int64_t r = 0; r < m; ++r) {
        for (int64_t c = 0; c < n; ++c) {
            if (W[r * n + c] != 0.0f) {
                if (val) { val[k] = W[r * n + c]; colI[k] = c; }
                ++k;
            }
        }
        rowPtr[r + 1] = k;
    }
    return k;
}

/* Algorithm 2 with the value array indexed by position i. */
void orc_dot_csr(int64_t m, const float *val, const int64_t *colI, const int64_t *rowPtr,
                 const float *X, int64_t L, double *Y) {
    for (int64_t l = 0; l < L; ++l)
        for (int64_t r = 0; r < m; ++r) {
            double y = 0.0;
            for (int64_t i = rowPtr[r]; i < rowPtr[r + 1]; ++i) y += (double)val[i] * (double)X[colI[i] * L + l];
            Y[r * L + l] = y;
        }
}
