/* CPU oracle for the exact k-nearest-neighbour graph and its backward pass.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file; it exists so
 * that the HIP library can be compared, element by element, with a plain definition.  It
 * shares no code, header, table or helper with the HIP path.
 *
 * What the binned search of the paper (Section 3, Algorithm 2) reaches is the exact K nearest
 * neighbours of every point inside its own row split: the search only stops once the best-K
 * radius is certified against everything unsearched (Algorithm 2, termination test), so the
 * result has a plain definition, written out here as a brute-force scan:
 *
 *   - slot 0 of every row is the query itself at squared distance 0 (Algorithm 2, the
 *     initialisation of neighbors[v][0]); the query is excluded from the scan (the u = v test);
 *   - slots 1..K-1 are the K-1 smallest pairs (d2(v,u), u), u != v, u in v's row split,
 *     ordered by d2 ascending and, among equal d2, by lower index u (the paper's buffer is
 *     unordered and its ties depend on bin order; this build fixes one answer);
 *   - d2 uses ALL coordinates (Algorithm 2 caches and uses every one of the n_c coordinates),
 *     as a left-to-right float32 sum of float32 squares of float32 differences, every
 *     operation rounded individually (no fused multiply-add): compile with -ffp-contract=off;
 *   - searches never cross a row split (Section 3, first paragraph);
 *   - a row split with m < K points leaves slots m..K-1 as (index -1, distance 0); -1 is the
 *     padding value the paper's package uses elsewhere (Algorithm 3).
 *
 * Direction flags (Algorithm 2, inputs useDir and dir[]): with flags given, a point whose flag
 * is 0 or 2 issues no query (its output row is all padding: index -1, distance 0, slot 0
 * included), and a point whose flag is 1 or 2 is never anybody's neighbour; any other value
 * means both roles.  A querying point is still its own slot 0 whatever its flag.
 *
 * Backward (Section 3, last paragraph: gradients of the returned distances): the derivative
 * of d2(v,u) = sum_c (x[v][c]-x[u][c])^2 with respect to the coordinates, accumulated in
 * double precision.
 *
 * Parallelism: an OpenMP loop over queries (queries are independent; each query's own scan
 * stays sequential and in index order).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_BLOCK 512

/* Squared distances from query q to candidates u0..u0+m-1, each a left-to-right fp32 sum. */
__attribute__((target_clones("avx2", "default")))
static void block_d2(const float* coords, int d, const float* q, int64_t u0, int m, float* out)
{
    for (int i = 0; i < m; ++i) {
        const float* p = coords + (u0 + i) * (int64_t)d;
        float delta = q[0] - p[0];
        float acc = delta * delta;
        for (int c = 1; c < d; ++c) {
            delta = q[c] - p[c];
            float sq = delta * delta;
            acc = acc + sq;
        }
        out[i] = acc;
    }
}

/* strict total order on (d2, index) */
static inline int pair_less(float d2a, int32_t ia, float d2b, int32_t ib)
{
    return (d2a < d2b) || (d2a == d2b && ia < ib);
}

/* One query: scan its row split [s,e), keep the K-1 best others sorted in best_*[0..filled). */
static void one_query(const float* coords, const int32_t* dir, int d, int64_t s, int64_t e, int64_t v, int k,
                      int32_t* out_idx, float* out_d2)
{
    float buf[ORACLE_BLOCK];
    int cap = k - 1;           /* slots for points other than v */
    int filled = 0;
    int32_t* bi = out_idx + 1; /* sorted best list lives directly in output slots 1.. */
    float* bd = out_d2 + 1;
    const float* q = coords + v * (int64_t)d;

    for (int j = 0; j < k; ++j) { out_idx[j] = -1; out_d2[j] = 0.0f; }
    if (dir && (dir[v] == 0 || dir[v] == 2)) return;      /* not a query */
    out_idx[0] = (int32_t)v;
    if (cap == 0) return;

    for (int64_t u0 = s; u0 < e; u0 += ORACLE_BLOCK) {
        int m = (int)((e - u0) < ORACLE_BLOCK ? (e - u0) : ORACLE_BLOCK);
        block_d2(coords, d, q, u0, m, buf);
        for (int i = 0; i < m; ++i) {
            int64_t u = u0 + i;
            if (u == v) continue;
            if (dir && (dir[u] == 1 || dir[u] == 2)) continue;   /* not a neighbour */
            float d2 = buf[i];
            if (filled == cap && !pair_less(d2, (int32_t)u, bd[cap - 1], bi[cap - 1])) continue;
            /* insertion into the sorted list */
            int pos = (filled < cap) ? filled : cap - 1;
            while (pos > 0 && pair_less(d2, (int32_t)u, bd[pos - 1], bi[pos - 1])) {
                bd[pos] = bd[pos - 1];
                bi[pos] = bi[pos - 1];
                --pos;
            }
            bd[pos] = d2;
            bi[pos] = (int32_t)u;
            if (filled < cap) ++filled;
        }
    }
}

static int64_t find_segment(const int32_t* row_splits, int n_segments, int64_t v)
{
    /* linear scan is fine for an oracle; skips empty segments naturally */
    for (int s = 0; s < n_segments; ++s)
        if (v >= row_splits[s] && v < row_splits[s + 1]) return s;
    return -1;
}

/* Full graph.  dir: [n] direction flags or NULL.  out_idx/out_d2 are [n][k] row-major. Returns 0, or -1 on bad arguments. */
int oracle_knn(const float* coords, const int32_t* row_splits, const int32_t* dir, int64_t n, int d,
               int n_segments, int k, int32_t* out_idx, float* out_d2, int n_threads)
{
    if (!coords || !row_splits || !out_idx || !out_d2 || d < 1 || k < 1 || n_segments < 1) return -1;
    if (row_splits[0] != 0 || row_splits[n_segments] != n) return -1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
    for (int s = 0; s < n_segments; ++s) {
        int64_t b = row_splits[s], e = row_splits[s + 1];
        if (e < b) return -1;
#pragma omp parallel for schedule(dynamic, 64)
        for (int64_t v = b; v < e; ++v)
            one_query(coords, dir, d, b, e, v, k, out_idx + v * (int64_t)k, out_d2 + v * (int64_t)k);
    }
    return 0;
}

/* Selected rows only: out_idx/out_d2 are [n_rows][k], row i answering query rows[i]. */
int oracle_knn_rows(const float* coords, const int32_t* row_splits, const int32_t* dir, int64_t n, int d,
                    int n_segments, int k, const int64_t* rows, int64_t n_rows,
                    int32_t* out_idx, float* out_d2, int n_threads)
{
    if (!coords || !row_splits || !rows || !out_idx || !out_d2 || d < 1 || k < 1 || n_segments < 1) return -1;
    if (row_splits[0] != 0 || row_splits[n_segments] != n) return -1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t v = rows[i];
        int64_t s = (v >= 0 && v < n) ? find_segment(row_splits, n_segments, v) : -1;
        if (s < 0) { bad = 1; continue; }
        one_query(coords, dir, d, row_splits[s], row_splits[s + 1], v, k,
                  out_idx + i * (int64_t)k, out_d2 + i * (int64_t)k);
    }
    return bad ? -1 : 0;
}

/* Backward: dL/dx given g = dL/d(d2) on the returned [n][k] distances.
 *   d2(v,u) = sum_c (x[v][c]-x[u][c])^2  =>  d d2 / d x[v][c] = +2 (x[v][c]-x[u][c]),
 *                                            d d2 / d x[u][c] = -2 (x[v][c]-x[u][c]).
 * Entries with idx < 0 (padding) carry no gradient.  Accumulated in double.
 * abs_sum (optional, may be NULL) receives, per element, the sum of the absolute values of
 * the contributions added into it: the natural scale for a tolerance under cancellation. */
int oracle_knn_backward(const float* grad_d2, const int32_t* idx, const float* coords,
                        int64_t n, int d, int k, double* grad_coords, double* abs_sum)
{
    if (!grad_d2 || !idx || !coords || !grad_coords || d < 1 || k < 1) return -1;
    memset(grad_coords, 0, sizeof(double) * (size_t)n * (size_t)d);
    if (abs_sum) memset(abs_sum, 0, sizeof(double) * (size_t)n * (size_t)d);
    for (int64_t v = 0; v < n; ++v) {
        for (int j = 0; j < k; ++j) {
            int32_t u = idx[v * (int64_t)k + j];
            if (u < 0) continue;
            if (u >= n) return -1;
            double g = (double)grad_d2[v * (int64_t)k + j];
            for (int c = 0; c < d; ++c) {
                double diff = (double)coords[v * (int64_t)d + c] - (double)coords[(int64_t)u * d + c];
                double t = 2.0 * g * diff;
                grad_coords[v * (int64_t)d + c] += t;
                grad_coords[(int64_t)u * d + c] -= t;
                if (abs_sum) {
                    abs_sum[v * (int64_t)d + c] += fabs(t);
                    abs_sum[(int64_t)u * d + c] += fabs(t);
                }
            }
        }
    }
    return 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
