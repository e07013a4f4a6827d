/* Driver for the AddressSanitizer + UndefinedBehaviorSanitizer build of the CPU oracle (tests/test_sanitizers_cpu.py).
 * Calls every entry point of oracle/knn_oracle.c and oracle/oc_helper_oracle.c on small inputs that reach their edge
 * paths (empty and short row splits, K above the split size, padding, direction flags, duplicates, rotation and
 * truncation in Algorithm 3) and checks a few invariants; the sanitizers abort on any invalid access or
 * undefined operation. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_knn(const float*, const int32_t*, const int32_t*, int64_t, int, int, int, int32_t*, float*, int);
int oracle_knn_rows(const float*, const int32_t*, const int32_t*, int64_t, int, int, int, const int64_t*, int64_t,
                    int32_t*, float*, int);
int oracle_knn_backward(const float*, const int32_t*, const float*, int64_t, int, int, double*, double*);
int oracle_oc_helper(const int32_t*, const int32_t*, const int32_t*, const int32_t*, int64_t, int64_t, int64_t, int64_t,
                     int64_t, int, int64_t, int32_t*, int32_t*);

static uint32_t state = 12345u;
static float rnd(void) { state = state * 1664525u + 1013904223u; return (float)(state >> 8) / 16777216.0f; }

int main(void)
{
    int failures = 0;
    for (int d = 1; d <= 10; d += 3) {
        for (int k = 1; k <= 70; k += 23) {
            const int32_t rs[6] = {0, 37, 37, 40, 41, 700};          /* an empty split, splits shorter than k */
            const int64_t n = 700;
            float* x = malloc(sizeof(float) * n * d);
            int32_t* dir = malloc(sizeof(int32_t) * n);
            int32_t* idx = malloc(sizeof(int32_t) * n * k);
            float* d2 = malloc(sizeof(float) * n * k);
            for (int64_t i = 0; i < n * d; ++i) x[i] = rnd();
            for (int64_t i = 100 * d; i < 160 * d; ++i) x[i] = x[100 * d + i % d];      /* duplicates */
            for (int64_t i = 0; i < n; ++i) dir[i] = (int32_t)(rnd() * 5.0f) - 1;
            if (oracle_knn(x, rs, NULL, n, d, 5, k, idx, d2, 1) != 0) ++failures;
            for (int64_t v = 0; v < n; ++v) {
                if (idx[v * k] != v || d2[v * k] != 0.0f) ++failures;
                for (int j = 2; j < k; ++j)
                    if (idx[v * k + j] >= 0 && d2[v * k + j] < d2[v * k + j - 1]) ++failures;
            }
            double* g = malloc(sizeof(double) * n * d);
            double* a = malloc(sizeof(double) * n * d);
            float* up = malloc(sizeof(float) * n * k);
            for (int64_t i = 0; i < n * k; ++i) up[i] = rnd() - 0.5f;
            if (oracle_knn_backward(up, idx, x, n, d, k, g, a) != 0) ++failures;
            if (oracle_knn_backward(up, idx, x, n, d, k, g, NULL) != 0) ++failures;
            if (oracle_knn(x, rs, dir, n, d, 5, k, idx, d2, 1) != 0) ++failures;
            const int64_t rows[5] = {0, 36, 37, 40, 699};
            int32_t* ri = malloc(sizeof(int32_t) * 5 * k);
            float* rd = malloc(sizeof(float) * 5 * k);
            if (oracle_knn_rows(x, rs, dir, n, d, 5, k, rows, 5, ri, rd, 1) != 0) ++failures;
            for (int r = 0; r < 5; ++r)
                for (int j = 0; j < k; ++j)
                    if (ri[r * k + j] != idx[rows[r] * k + j]) ++failures;
            const int64_t bad_row[1] = {700};
            if (oracle_knn_rows(x, rs, NULL, n, d, 5, k, bad_row, 1, ri, rd, 1) == 0) ++failures;     /* must be refused */
            free(x); free(dir); free(idx); free(d2); free(g); free(a); free(up); free(ri); free(rd);
        }
    }
    {   /* Algorithm 3: three row splits, objects with more members than n_maxuq, rotation, a walk cut at n_maxrs */
        const int32_t rs[4] = {0, 50, 50, 130};
        const int64_t n_vert = 130, n_unique = 9;
        int32_t asso[130], unique_idx[9], unique_rs[9];
        for (int i = 0; i < 130; ++i) asso[i] = (int32_t)(rnd() * 11.0f) - 1;
        for (int i = 0; i < 9; ++i) { unique_idx[i] = i; unique_rs[i] = i < 4 ? 0 : (i == 4 ? 1 : 2); }
        for (int rot = 1; rot <= 7; rot += 3) {
            for (int n_maxrs = 20; n_maxrs <= 100; n_maxrs += 80) {
                const int n_maxuq = 4;
                int32_t* M = malloc(sizeof(int32_t) * n_maxuq * n_unique);
                int32_t* Mn = malloc(sizeof(int32_t) * n_maxrs * n_unique);
                if (oracle_oc_helper(asso, unique_idx, unique_rs, rs, n_vert, n_unique, 3, n_maxuq, n_maxrs, 1, rot, M, Mn) != 0) ++failures;
                if (oracle_oc_helper(asso, unique_idx, unique_rs, rs, n_vert, n_unique, 3, n_maxuq, n_maxrs, 0, rot, M, NULL) != 0) ++failures;
                for (int i = 0; i < n_maxuq * n_unique; ++i) if (M[i] < -1 || M[i] >= n_vert) ++failures;
                free(M); free(Mn);
            }
        }
    }
    printf("sanitize_oracle_main: failures=%d\n", failures);
    return failures != 0;
}
