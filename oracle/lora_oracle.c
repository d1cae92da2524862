/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.
 *
 * Plain float64 CPU oracle for the heterogeneous-LoRA batching operator
 * (the operator ATMM accelerates, paper section 4.3.1), written from the
 * definitions in the paper and sharing no code with the HIP library:
 *
 *   - LoRA, section 2: the weight update of an adapter is the product of its
 *     two low-rank factors; in unmerged ("bypass") inference the adapter's
 *     result is added onto the base layer's output.
 *   - Unmerged batching, sections 1 and 2: the base-model product is shared by
 *     all requests of a batch, while each request goes through its own adapter.
 *
 * In row-vector form, for token t whose request uses adapter a (rank r_a,
 * scale s_a):
 *
 *       y[t,:] = x[t,:] W + s_a * (x[t,:] A_a) B_a
 *
 * with x [T,K], W [K,N], A_a [K,r_a], B_a [r_a,N], all row-major doubles.
 * A token with adapter id < 0, or whose adapter has rank 0, gets y = x W.
 *
 * One loop nest per token, in the order of the formula; nothing is blocked
 * or fused, and every sum runs over its index in increasing order (where a
 * loop over the output index is innermost, that is only to walk a row-major
 * matrix along its rows; the additions each output element sees are the same).
 * OpenMP only distributes tokens over threads, so every output row is computed
 * by the same sequence of operations regardless of the thread count.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Segment table -> adapter id of every token.  Segment s covers tokens
 * [seg_indptr[s], seg_indptr[s+1]).  Written as the definition: for each
 * token, scan the segments until the one containing it is found.
 * Returns 0, or -1 when the table does not tile [0,T).
 */
int oracle_token_adapter(int32_t T, int32_t S, const int32_t* seg_indptr,
                         const int32_t* seg_adapter, int32_t* tok_adapter)
{
    if (S == 0) return T == 0 ? 0 : -1;
    if (seg_indptr[0] != 0 || seg_indptr[S] != T) return -1;
    for (int32_t s = 0; s < S; ++s)
        if (seg_indptr[s + 1] < seg_indptr[s]) return -1;
    for (int32_t t = 0; t < T; ++t) {
        int32_t found = -2;
        for (int32_t s = 0; s < S; ++s) {
            if (seg_indptr[s] <= t && t < seg_indptr[s + 1]) { found = seg_adapter[s]; break; }
        }
        if (found == -2) return -1;
        tok_adapter[t] = found;
    }
    return 0;
}

static int has_adapter(int32_t a, const int32_t* rank)
{
    return a >= 0 && rank[a] > 0;
}

/*
 * Shrink (first of the two extra products per layer, section 3.2):
 *     v[t,j] = sum_k x[t,k] A_a[k,j]          j < r_a
 * multiplied by s_a when apply_scale != 0.  Entries j >= r_a of a row, and
 * whole rows of tokens without an adapter, are set to 0.
 * rows == NULL means all T tokens; otherwise only tokens rows[0..n_rows) are
 * computed, and row i of v belongs to token rows[i].
 */
void oracle_shrink(int32_t T, int32_t K, const int32_t* tok_adapter,
                   const int32_t* rank, const double* scale,
                   const double* x, const double* const* A,
                   int apply_scale, double* v, int32_t R,
                   const int32_t* rows, int32_t n_rows)
{
    int32_t M = rows ? n_rows : T;
#pragma omp parallel for schedule(dynamic, 4)
    for (int32_t i = 0; i < M; ++i) {
        int32_t t = rows ? rows[i] : i;
        double* vt = v + (size_t)i * R;
        for (int32_t j = 0; j < R; ++j) vt[j] = 0.0;
        int32_t a = tok_adapter[t];
        if (!has_adapter(a, rank)) continue;
        int32_t r = rank[a];
        const double* xt = x + (size_t)t * K;
        const double* Aa = A[a];
        /* v_j accumulates k = 0, 1, ..., K-1 in that order for every j; the
         * k loop is outermost only so that A_a is walked along its rows. */
        for (int32_t k = 0; k < K; ++k)
            for (int32_t j = 0; j < r; ++j) vt[j] += xt[k] * Aa[(size_t)k * r + j];
        if (apply_scale)
            for (int32_t j = 0; j < r; ++j) vt[j] = scale[a] * vt[j];
    }
}

/*
 * Expand-and-add (the second extra product plus the extra addition per layer,
 * section 3.2), from the operator's inputs:
 *     y_out[t,n] = y_in[t,n] + s_a * sum_j (sum_k x[t,k] A_a[k,j]) B_a[j,n]
 * y_in may be NULL (treated as 0).  Row selection as in oracle_shrink; y_in and
 * y_out are indexed by the position i in the selection.
 */
void oracle_expand(int32_t T, int32_t K, int32_t N, const int32_t* tok_adapter,
                   const int32_t* rank, const double* scale,
                   const double* x, const double* const* A, const double* const* B,
                   const double* y_in, double* y_out,
                   const int32_t* rows, int32_t n_rows)
{
    int32_t M = rows ? n_rows : T;
#pragma omp parallel for schedule(dynamic, 4)
    for (int32_t i = 0; i < M; ++i) {
        int32_t t = rows ? rows[i] : i;
        double* yo = y_out + (size_t)i * N;
        for (int32_t n = 0; n < N; ++n) yo[n] = y_in ? y_in[(size_t)i * N + n] : 0.0;
        int32_t a = tok_adapter[t];
        if (!has_adapter(a, rank)) continue;
        int32_t r = rank[a];
        const double* xt = x + (size_t)t * K;
        const double* Aa = A[a];
        const double* Ba = B[a];
        for (int32_t n = 0; n < N; ++n) {
            double delta = 0.0;
            for (int32_t j = 0; j < r; ++j) {
                double vj = 0.0;
                for (int32_t k = 0; k < K; ++k) vj += xt[k] * Aa[(size_t)k * r + j];
                delta += vj * Ba[(size_t)j * N + n];
            }
            yo[n] += scale[a] * delta;
        }
    }
}

/*
 * Same result as oracle_expand, but v is formed once per token instead of once
 * per output column, and the loops walk A_a and B_a along their rows.  Every
 * output element still sees the same sequence of floating-point operations
 * (v_j sums k = 0..K-1 in order, delta_n sums j = 0..r-1 in order), so the two
 * functions agree bit for bit; this one exists so that full-size
 * configurations finish in seconds.  A test checks the bitwise agreement.
 */
void oracle_expand_fast(int32_t T, int32_t K, int32_t N, const int32_t* tok_adapter,
                        const int32_t* rank, const double* scale,
                        const double* x, const double* const* A, const double* const* B,
                        const double* y_in, double* y_out,
                        const int32_t* rows, int32_t n_rows, int32_t max_rank)
{
    int32_t M = rows ? n_rows : T;
#pragma omp parallel
    {
        double* vj = (double*)malloc(sizeof(double) * (size_t)(max_rank > 0 ? max_rank : 1));
        double* delta = (double*)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
#pragma omp for schedule(dynamic, 4)
        for (int32_t i = 0; i < M; ++i) {
            int32_t t = rows ? rows[i] : i;
            double* yo = y_out + (size_t)i * N;
            for (int32_t n = 0; n < N; ++n) yo[n] = y_in ? y_in[(size_t)i * N + n] : 0.0;
            int32_t a = tok_adapter[t];
            if (!has_adapter(a, rank)) continue;
            int32_t r = rank[a];
            const double* xt = x + (size_t)t * K;
            const double* Aa = A[a];
            const double* Ba = B[a];
            for (int32_t j = 0; j < r; ++j) vj[j] = 0.0;
            for (int32_t k = 0; k < K; ++k)
                for (int32_t j = 0; j < r; ++j) vj[j] += xt[k] * Aa[(size_t)k * r + j];
            for (int32_t n = 0; n < N; ++n) delta[n] = 0.0;
            for (int32_t j = 0; j < r; ++j)
                for (int32_t n = 0; n < N; ++n) delta[n] += vj[j] * Ba[(size_t)j * N + n];
            for (int32_t n = 0; n < N; ++n) yo[n] += scale[a] * delta[n];
        }
        free(vj);
        free(delta);
    }
}

/*
 * Base product alone:  y[t,n] = sum_k x[t,k] W[k,n].
 */
void oracle_base(int32_t T, int32_t K, int32_t N, const double* x, const double* W,
                 double* y, const int32_t* rows, int32_t n_rows)
{
    int32_t M = rows ? n_rows : T;
#pragma omp parallel for schedule(dynamic, 4)
    for (int32_t i = 0; i < M; ++i) {
        int32_t t = rows ? rows[i] : i;
        const double* xt = x + (size_t)t * K;
        double* yo = y + (size_t)i * N;
        for (int32_t n = 0; n < N; ++n) yo[n] = 0.0;
        for (int32_t k = 0; k < K; ++k)
            for (int32_t n = 0; n < N; ++n) yo[n] += xt[k] * W[(size_t)k * N + n];
    }
}

/*
 * Whole layer:  y[t,:] = x[t,:] W + s_a (x[t,:] A_a) B_a   (the formula above).
 * The base row is formed first, then the adapter's bypass result is added onto
 * it, as section 2 describes unmerged inference.
 */
void oracle_forward(int32_t T, int32_t K, int32_t N, const int32_t* tok_adapter,
                    const int32_t* rank, const double* scale,
                    const double* x, const double* W,
                    const double* const* A, const double* const* B,
                    double* y, const int32_t* rows, int32_t n_rows, int32_t max_rank)
{
    int32_t M = rows ? n_rows : T;
#pragma omp parallel
    {
        double* vj = (double*)malloc(sizeof(double) * (size_t)(max_rank > 0 ? max_rank : 1));
        double* delta = (double*)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
#pragma omp for schedule(dynamic, 4)
        for (int32_t i = 0; i < M; ++i) {
            int32_t t = rows ? rows[i] : i;
            const double* xt = x + (size_t)t * K;
            double* yo = y + (size_t)i * N;
            for (int32_t n = 0; n < N; ++n) yo[n] = 0.0;
            for (int32_t k = 0; k < K; ++k)
                for (int32_t n = 0; n < N; ++n) yo[n] += xt[k] * W[(size_t)k * N + n];
            int32_t a = tok_adapter[t];
            if (!has_adapter(a, rank)) continue;
            int32_t r = rank[a];
            const double* Aa = A[a];
            const double* Ba = B[a];
            for (int32_t j = 0; j < r; ++j) vj[j] = 0.0;
            for (int32_t k = 0; k < K; ++k)
                for (int32_t j = 0; j < r; ++j) vj[j] += xt[k] * Aa[(size_t)k * r + j];
            for (int32_t n = 0; n < N; ++n) delta[n] = 0.0;
            for (int32_t j = 0; j < r; ++j)
                for (int32_t n = 0; n < N; ++n) delta[n] += vj[j] * Ba[(size_t)j * N + n];
            for (int32_t n = 0; n < N; ++n) yo[n] += scale[a] * delta[n];
        }
        free(vj);
        free(delta);
    }
}
