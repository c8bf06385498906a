/*
 * CPU oracle for the Relaxed Word Mover's Distance.  TEST INFRASTRUCTURE ONLY:
 * it is called by the tests, by the smoke check and by the benchmark's CPU
 * baseline leg, never by the product path, and it shares no code with the HIP
 * library.
 *
 * Everything here is the plain definition from the paper, evaluated in fp64:
 *
 *   c(p,a)    Euclidean distance between the embedding vectors of words p, a
 *             (Sec. III, the "circle" operation: like T1 * T2^T with distances
 *             in place of dot products), from direct coordinate differences.
 *   d12(i,j)  sum over the words p of X1[i] of  x_i[p] * min_{a in X2[j]} c(p,a)
 *             (Sec. III "Solving the RWMD problem": row minima of C_ij, dot
 *             product with F_1,i).
 *   d21(i,j)  the same with the roles swapped (column minima, dot with F_2,j).
 *   D[i][j]   max(d12, d21)   (Sec. III; Sec. IV: D = max(D1, D2^T)).
 *   R         the k smallest entries of a column of D with their row numbers
 *             (Sec. III: top-k smallest distances and their positions).
 *
 * Two evaluations of D are provided:
 *   oracle_rwmd_bruteforce  the definition pair by pair (quadruple loop);
 *   oracle_rwmd_table       the same sums reorganised per query: the distances
 *                           from the query's words to every vocabulary word are
 *                           tabulated once, then each database row reads them.
 * plus the two phases of the linear-complexity method (Sec. IV) on their own,
 * so that each library entry point has an oracle of its own:
 *   oracle_phase1  Z[w][j] = min_{a in X2[j]} c(w,a) for every vocabulary word w;
 *   oracle_phase2  D = X * Z  (sparse rows times dense matrix).
 *
 * Layout conventions (all host memory): E is row-major v x m float32 with leading
 * dimension ld; a histogram set is CSR (row_ptr int64[rows+1], col_idx int32[nnz],
 * val float32[nnz]); D is row-major, database rows x query columns, fp64.
 * Every histogram must have at least one word (the minimum over an empty set is
 * undefined); functions return -1 when they meet an empty one, 0 on success.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#if defined(__x86_64__) && defined(__GNUC__) && !defined(__clang__)
#define ORACLE_CLONES __attribute__((target_clones("avx2", "default")))
#else
#define ORACLE_CLONES
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* c(p,a): Euclidean distance between two rows of E, fp64, direct differences. */
ORACLE_CLONES
static double word_distance(const float* E, int64_t m, int64_t ld, int64_t p, int64_t a)
{
    const float* x = E + p * ld;
    const float* y = E + a * ld;
    double s = 0.0;
    for (int64_t t = 0; t < m; ++t) {
        double d = (double)x[t] - (double)y[t];
        s += d * d;
    }
    return sqrt(s);
}

static int has_empty_row(const int64_t* ptr, int64_t rows)
{
    for (int64_t r = 0; r < rows; ++r)
        if (ptr[r + 1] <= ptr[r]) return 1;
    return 0;
}

/* One pair, both directions, straight from the definition. */
static void pair_bounds(const float* E, int64_t m, int64_t ld,
                        const int32_t* pc, const float* px, int64_t hp,   /* database doc */
                        const int32_t* ac, const float* ay, int64_t ha,   /* query doc    */
                        double* d12, double* d21)
{
    double s12 = 0.0;
    for (int64_t p = 0; p < hp; ++p) {
        double mn = INFINITY;
        for (int64_t a = 0; a < ha; ++a) {
            double c = word_distance(E, m, ld, pc[p], ac[a]);
            if (c < mn) mn = c;
        }
        s12 += (double)px[p] * mn;
    }
    double s21 = 0.0;
    for (int64_t a = 0; a < ha; ++a) {
        double mn = INFINITY;
        for (int64_t p = 0; p < hp; ++p) {
            double c = word_distance(E, m, ld, pc[p], ac[a]);
            if (c < mn) mn = c;
        }
        s21 += (double)ay[a] * mn;
    }
    *d12 = s12;
    *d21 = s21;
}

/*
 * Brute force over all pairs.  D, D12, D21 are n x q row-major fp64; D12 and D21
 * may be NULL.  D12[i][j] is the cost of moving database doc i to query j.
 */
int oracle_rwmd_bruteforce(const float* E, int64_t v, int64_t m, int64_t ld,
                           const int64_t* db_ptr, const int32_t* db_col, const float* db_val, int64_t n,
                           const int64_t* q_ptr, const int32_t* q_col, const float* q_val, int64_t q,
                           double* D, double* D12, double* D21)
{
    (void)v;
    if (has_empty_row(db_ptr, n) || has_empty_row(q_ptr, q)) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t j = 0; j < q; ++j) {
            double a, b;
            pair_bounds(E, m, ld,
                        db_col + db_ptr[i], db_val + db_ptr[i], db_ptr[i + 1] - db_ptr[i],
                        q_col + q_ptr[j], q_val + q_ptr[j], q_ptr[j + 1] - q_ptr[j], &a, &b);
            if (D12) D12[i * q + j] = a;
            if (D21) D21[i * q + j] = b;
            D[i * q + j] = a > b ? a : b;
        }
    }
    return 0;
}

/* Brute force on a list of (i, j) pairs: out[t] = D[pi[t]][pj[t]]. */
int oracle_rwmd_pairs(const float* E, int64_t v, int64_t m, int64_t ld,
                      const int64_t* db_ptr, const int32_t* db_col, const float* db_val, int64_t n,
                      const int64_t* q_ptr, const int32_t* q_col, const float* q_val, int64_t q,
                      const int64_t* pi, const int64_t* pj, int64_t npairs, double* out)
{
    (void)v;
    for (int64_t t = 0; t < npairs; ++t)
        if (pi[t] < 0 || pi[t] >= n || pj[t] < 0 || pj[t] >= q) return -2;
    if (has_empty_row(db_ptr, n) || has_empty_row(q_ptr, q)) return -1;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < npairs; ++t) {
        int64_t i = pi[t], j = pj[t];
        double a, b;
        pair_bounds(E, m, ld,
                    db_col + db_ptr[i], db_val + db_ptr[i], db_ptr[i + 1] - db_ptr[i],
                    q_col + q_ptr[j], q_val + q_ptr[j], q_ptr[j + 1] - q_ptr[j], &a, &b);
        out[t] = a > b ? a : b;
    }
    return 0;
}

/* Row `a` of the table for one query: W[w] = c(w, word) for every vocabulary word w. */
static void table_row(const float* E, int64_t v, int64_t m, int64_t ld, int64_t word, double* W)
{
#pragma omp parallel for schedule(static)
    for (int64_t w = 0; w < v; ++w) W[w] = word_distance(E, m, ld, w, word);
}

/*
 * Per-query table evaluation of the same definition.  For query j the table
 * W[a][w] = c(w, a-th word of the query) is built once for all v words; then for
 * every database doc i:  d12 = sum_p x_p * min_a W[a][p],  d21 = sum_a y_a * min_p W[a][p].
 */
int oracle_rwmd_table(const float* E, int64_t v, int64_t m, int64_t ld,
                      const int64_t* db_ptr, const int32_t* db_col, const float* db_val, int64_t n,
                      const int64_t* q_ptr, const int32_t* q_col, const float* q_val, int64_t q,
                      double* D, double* D12, double* D21)
{
    if (has_empty_row(db_ptr, n) || has_empty_row(q_ptr, q)) return -1;
    int64_t hmax = 0;
    for (int64_t j = 0; j < q; ++j)
        if (q_ptr[j + 1] - q_ptr[j] > hmax) hmax = q_ptr[j + 1] - q_ptr[j];
    double* W = (double*)malloc(sizeof(double) * (size_t)hmax * (size_t)v);
    double* zmin = (double*)malloc(sizeof(double) * (size_t)v);
    if (!W || !zmin) { free(W); free(zmin); return -3; }

    for (int64_t j = 0; j < q; ++j) {
        const int32_t* ac = q_col + q_ptr[j];
        const float* ay = q_val + q_ptr[j];
        const int64_t ha = q_ptr[j + 1] - q_ptr[j];
        for (int64_t a = 0; a < ha; ++a) table_row(E, v, m, ld, ac[a], W + a * v);
#pragma omp parallel for schedule(static)
        for (int64_t w = 0; w < v; ++w) {
            double mn = INFINITY;
            for (int64_t a = 0; a < ha; ++a)
                if (W[a * v + w] < mn) mn = W[a * v + w];
            zmin[w] = mn;
        }
#pragma omp parallel for schedule(dynamic, 64)
        for (int64_t i = 0; i < n; ++i) {
            const int32_t* pc = db_col + db_ptr[i];
            const float* px = db_val + db_ptr[i];
            const int64_t hp = db_ptr[i + 1] - db_ptr[i];
            double s12 = 0.0;
            for (int64_t p = 0; p < hp; ++p) s12 += (double)px[p] * zmin[pc[p]];
            double s21 = 0.0;
            for (int64_t a = 0; a < ha; ++a) {
                const double* Wa = W + a * v;
                double mn = INFINITY;
                for (int64_t p = 0; p < hp; ++p)
                    if (Wa[pc[p]] < mn) mn = Wa[pc[p]];
                s21 += (double)ay[a] * mn;
            }
            if (D12) D12[i * q + j] = s12;
            if (D21) D21[i * q + j] = s21;
            D[i * q + j] = s12 > s21 ? s12 : s21;
        }
    }
    free(W);
    free(zmin);
    return 0;
}

/* First phase alone (Sec. IV): Z is v x q row-major fp64. */
int oracle_phase1(const float* E, int64_t v, int64_t m, int64_t ld,
                  const int64_t* q_ptr, const int32_t* q_col, int64_t q, double* Z)
{
    if (has_empty_row(q_ptr, q)) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t w = 0; w < v; ++w) {
        for (int64_t j = 0; j < q; ++j) {
            double mn = INFINITY;
            for (int64_t t = q_ptr[j]; t < q_ptr[j + 1]; ++t) {
                double c = word_distance(E, m, ld, w, q_col[t]);
                if (c < mn) mn = c;
            }
            Z[w * q + j] = mn;
        }
    }
    return 0;
}

/* Second phase alone (Sec. IV): D (rows x ncols) = X (rows x v, CSR) * Z (v x ncols), fp64. */
int oracle_phase2(const int64_t* ptr, const int32_t* col, const float* val, int64_t rows,
                  const double* Z, int64_t ncols, double* D)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t j = 0; j < ncols; ++j) {
            double s = 0.0;
            for (int64_t t = ptr[i]; t < ptr[i + 1]; ++t) s += (double)val[t] * Z[(int64_t)col[t] * ncols + j];
            D[i * ncols + j] = s;
        }
    }
    return 0;
}

/*
 * Top-k per query column of D (n x q row-major): the k smallest values of column j
 * ordered by (distance, row index) ascending.  idx and dist are q x k.  Requires k <= n.
 */
int oracle_topk(const double* D, int64_t n, int64_t q, int64_t k, int64_t* idx, double* dist)
{
    if (k < 1 || k > n) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < q; ++j) {
        int64_t* bi = idx + j * k;
        double* bd = dist + j * k;
        int64_t cnt = 0;
        for (int64_t i = 0; i < n; ++i) {
            double d = D[i * q + j];
            if (cnt == k && !(d < bd[k - 1])) continue;   /* rows come in increasing i: ties lose */
            int64_t pos = cnt < k ? cnt : k - 1;
            while (pos > 0 && d < bd[pos - 1]) {
                bd[pos] = bd[pos - 1];
                bi[pos] = bi[pos - 1];
                --pos;
            }
            bd[pos] = d;
            bi[pos] = i;
            if (cnt < k) ++cnt;
        }
    }
    return 0;
}
