/* Driver for the sanitized build of the host side of the C ABI (tests/test_sanitizers_cpu.py): argument validation,
 * bin-count heuristics and workspace layout arithmetic over a grid of sizes including the ends of the accepted
 * ranges.  Every call here returns before anything is enqueued, so it runs without a GPU. */
#include <stdint.h>
#include <stdio.h>
#include "fastgraph.h"

int main(void)
{
    int32_t nb = 0, db = 0;
    size_t bytes = 0;
    int bad = 0;
    const int64_t sizes[] = {0, 1, 7, 64, 65, 4096, 100000, 1000000, 5000000, 2147418112LL, 2147418113LL, 2147483647LL,
                             2147483648LL, -1, (int64_t)1 << 40};
    for (unsigned i = 0; i < sizeof(sizes) / sizeof(sizes[0]); ++i)
        for (int d = 1; d <= 11; ++d)
            for (int k = 0; k <= 130; k += 13)
                for (int s = 0; s <= (1 << 22) + 1; s = s * 64 + 1)
                    for (int mode = -1; mode <= 2; ++mode) {
                        const int64_t n = sizes[i];
                        const fg_status a = fg_auto_n_bins(n, s, k, d, mode, &nb, &db);
                        const fg_status b = fg_workspace_size(n, d, s, k, 0, 0, &bytes);
                        if ((mode == 0 || mode == 1) && (a == FG_OK) != (b == FG_OK)) ++bad;
                        if (a == FG_OK) {
                            if (nb < 1 || db < 2 || db > 5 || db > d) ++bad;
                            if (fg_workspace_size(n, d, s, k, nb, db, &bytes) != FG_OK || (n > 0 && bytes < (size_t)n * 4)) ++bad;
                        }
                        for (int nbx = 1; nbx <= 1024; nbx *= 32)
                            for (int dbx = 0; dbx <= 6; dbx += 2) fg_workspace_size(n, d, s, k, nbx, dbx, &bytes);
                    }
    /* entry points with bad pointers, sizes and workspaces: all must come back with a status, never touch memory */
    fg_binning view;
    char dummy[512];
    void* p = (void*)(((uintptr_t)dummy + 255) & ~(uintptr_t)255);
    if (fg_bin_points(NULL, NULL, 10, 3, 1, 4, 0, 0, p, 256, &view, NULL) != FG_ERR_NULL) ++bad;
    if (fg_bin_points((const float*)p, (const int32_t*)p, 10, 3, 1, 4, 0, 0, p, 16, &view, NULL) != FG_ERR_WORKSPACE) ++bad;
    if (fg_bin_points((const float*)p, (const int32_t*)p, 10, 3, 1, 4, 0, 0, (char*)p + 4, 1 << 20, &view, NULL) != FG_ERR_WORKSPACE) ++bad;
    if (fg_binned_select_knn((const float*)p, (const int32_t*)p, 10, 12, 1, 4, 0, 0, (int32_t*)p, (float*)p, p, 256, NULL) != FG_ERR_UNSUPPORTED) ++bad;
    if (fg_binned_select_knn_static((const float*)p, (const int32_t*)p, 3000000, 3, 1, 16, 0, 0, (int32_t*)p, (float*)p, NULL) != FG_ERR_WORKSPACE) ++bad;
    if (fg_query_binned(NULL, (const int32_t*)p, 10, 3, 1, 4, (int32_t*)p, (float*)p, NULL, NULL, NULL) != FG_ERR_NULL) ++bad;
    if (fg_knn_backward((const float*)p, (const int32_t*)p, (const float*)p, (const int32_t*)p, 10, 3, 1, 4, (float*)p, p, 16, NULL) != FG_ERR_WORKSPACE) ++bad;
    if (fg_oc_helper_workspace_size(-1, 4, &bytes) != FG_ERR_BAD_SHAPE) ++bad;
    if (fg_status_string(FG_ERR_LAUNCH) == NULL || fg_status_string((fg_status)99) == NULL) ++bad;
    printf("sanitize_abi_main: bad=%d\n", bad);
    return bad != 0;
}
