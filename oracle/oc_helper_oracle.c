/* CPU oracle for the object-condensation index matrices (paper Section 5, Algorithm 3).
 *
 * TEST INFRASTRUCTURE ONLY; shares no code with the HIP path.
 *
 * For every object candidate k (unique_idx[k], living in row split unique_rs_asso[k]) the
 * algorithm walks the vertices of that row split and lists, in M, the vertices associated with
 * the object and, in M_not, the vertices that are not.  The steps, in the paper's order:
 *   1. window = [rs[split], rs[split+1]), clipped to n_vert and to at most n_maxrs vertices;
 *   2. the walk starts `tid` vertices into the window and wraps round to the window's start
 *      (the paper's thread index inside its launch block; here tid = k mod rot_block, with
 *      rot_block given by the caller, because the paper does not state its block size);
 *      when start + tid is already past the window the walk is simply the window in order;
 *   3. every vertex i of the walk with asso_idx[i] == object id is appended to M's row k until
 *      the row holds n_maxuq entries; the rest of the row is -1;
 *   4. if calc_m_not: the same walk appends every vertex with asso_idx[i] != object id to
 *      M_not's row k (capacity n_maxrs, never exceeded because the window is), rest -1.
 * Storage follows the paper's index macro: entry `fill` of row k lives at fill * n_unique + k.
 *
 * Reading taken where the listing is off by one: it tests `fill > n_maxuq` after writing, which
 * would write one entry past a row of n_maxuq entries; here a row stops at n_maxuq entries.
 */
#include <stdint.h>

static void walk(const int32_t* asso_idx, int64_t start, int64_t end, int64_t tid, int32_t uq, int want_equal,
                 int32_t* out, int64_t k, int64_t n_unique, int64_t capacity)
{
    int64_t fill = 0;
    for (int64_t i = start + tid; i < end && fill < capacity; ++i)
        if ((asso_idx[i] == uq) == (want_equal != 0)) { out[fill * n_unique + k] = (int32_t)i; ++fill; }
    for (int64_t i = start; i < start + tid && fill < capacity; ++i)
        if (i < end && (asso_idx[i] == uq) == (want_equal != 0)) { out[fill * n_unique + k] = (int32_t)i; ++fill; }
    for (; fill < capacity; ++fill) out[fill * n_unique + k] = -1;
}

int oracle_oc_helper(const int32_t* asso_idx, const int32_t* unique_idx, const int32_t* unique_rs_asso,
                     const int32_t* rs, int64_t n_vert, int64_t n_unique, int64_t n_splits,
                     int64_t n_maxuq, int64_t n_maxrs, int calc_m_not, int64_t rot_block,
                     int32_t* M, int32_t* M_not)
{
    if (!asso_idx || !unique_idx || !unique_rs_asso || !rs || !M || rot_block < 1) return -1;
    if (calc_m_not && !M_not) return -1;
    for (int64_t k = 0; k < n_unique; ++k) {
        int32_t uq = unique_idx[k];
        int64_t split = unique_rs_asso[k];
        if (split < 0 || split >= n_splits) return -1;
        int64_t start = rs[split], end = rs[split + 1];
        if (end > n_vert) end = n_vert;
        if (end - start > n_maxrs) end = start + n_maxrs;
        int64_t tid = k % rot_block;
        walk(asso_idx, start, end, tid, uq, 1, M, k, n_unique, n_maxuq);
        if (calc_m_not) walk(asso_idx, start, end, tid, uq, 0, M_not, k, n_unique, n_maxrs);
    }
    return 0;
}
