/* fastgraph.h -- C ABI of the MI355X-native binned exact k-nearest-neighbour graph build.
 *
 * The operations follow the problem statement of FastGraph (arXiv 2511.10442), Section 3
 * "Optimized K-Nearest Neighbor Algorithm": points of a ragged batch (row splits) are
 * partitioned into a regular grid of bins, sorted by bin, and every point searches shells of
 * neighbouring bins of growing radius until its K best squared distances are certified
 * against everything unsearched (Algorithm 1, Algorithm 2); gradients of the returned squared
 * distances flow back to the coordinates (Section 3, last paragraph).
 *
 * Conventions for every entry point
 *   - Every array pointer is a DEVICE pointer unless the comment says "host".
 *   - The caller owns every buffer.  The library allocates no device memory, keeps no global
 *     state, never synchronises the stream and never throws.  Inputs are never modified.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it; outputs are valid once the stream has reached that point.
 *   - `workspace` is device memory of at least fg_workspace_size() bytes, 256-byte aligned.
 *     Its contents are scratch: undefined on entry, undefined after the call except for the
 *     arrays an fg_binning view points into (valid until the workspace is reused).
 *   - Every call returns an fg_status; on any status other than FG_OK nothing was enqueued.
 *   - Preconditions that cannot be checked without a device round trip are documented, not
 *     checked: row_splits[0] = 0, row_splits[S] = n, non-decreasing; all coordinates finite.
 *   - n <= FG_MAX_N (indices are int32, and the launch arithmetic keeps a margin below 2^31).
 *     n_segments <= FG_MAX_SEGMENTS.  2 <= d <= 10.  1 <= k <= 128.
 */
#ifndef FASTGRAPH_H
#define FASTGRAPH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FG_OK = 0,
    FG_ERR_NULL = 1,        /* a required pointer is NULL */
    FG_ERR_BAD_SHAPE = 2,   /* n < 0, n > FG_MAX_N, n_segments < 1 or > FG_MAX_SEGMENTS, k < 1, n_bins/d_bin out of
                               range, too many bins */
    FG_ERR_UNSUPPORTED = 3, /* d outside 2..10, k > 128, d_bin outside 2..5 */
    FG_ERR_WORKSPACE = 4,   /* workspace too small or not 256-byte aligned */
    FG_ERR_LAUNCH = 5,      /* the HIP runtime reported an error at launch */
    FG_STATUS_INT_RANGE = 0x7fffffff   /* not a status: makes every non-negative int a valid value of the type on
                                          both sides of the boundary (C callers pass plain ints) */
} fg_status;

/* Largest values accepted. */
#define FG_MAX_N 2147418112       /* 2^31 - 2^16 points */
#define FG_MAX_SEGMENTS (1 << 22)
#define FG_MAX_D 10
#define FG_MIN_D 2
#define FG_MAX_K 128
#define FG_MIN_D_BIN 2
#define FG_MAX_D_BIN 5
#define FG_MAX_TOTAL_BINS (1 << 28) /* n_segments * n_bins^d_bin */

/* Human-readable name of a status (host pointer to a static string). */
const char* fg_status_string(fg_status status);

/* Bins per dimension and number of binning dimensions (Section 3, the equation
 *   n_bins = (32 * n_elems / K)^(1/d_max), n_elems = mean points per row split,
 * its clamp to the range 5..30, and the paragraph limiting binning to the first <= 5 dimensions).
 *   mode 0: the paper's heuristic as printed: d_bin = min(d, 5), value truncated, clamped to [5,30].
 *   mode 1: tuned for MI355X: same functional form with this build's own constant, binning
 *           dimensions and upper clamp (a finer grid; the paper notes the value is hardware
 *           specific and user-adjustable).
 * The choice never changes the result of the search, only its speed.
 * n_bins, d_bin: host out.  Pure host arithmetic; touches no device. */
fg_status fg_auto_n_bins(int64_t n, int32_t n_segments, int32_t k, int32_t d, int32_t mode,
                         int32_t* n_bins, int32_t* d_bin);

/* Bytes of workspace needed by fg_bin_points / fg_binned_select_knn / fg_knn_backward for this
 * problem (n_bins <= 0 or d_bin <= 0: the values fg_auto_n_bins mode 1 would choose).
 * bytes: host out.  O(n * (d + 5) + n_segments * n_bins^d_bin) words: a few words per point beyond
 * the input (the Abstract's claim of a negligible memory overhead). */
fg_status fg_workspace_size(int64_t n, int32_t d, int32_t n_segments, int32_t k,
                            int32_t n_bins, int32_t d_bin, size_t* bytes);

/* Result of the binning stage: device pointers into the caller's workspace. */
typedef struct {
    const int32_t* bin_idx;    /* [n]  flat cell of each point, ORIGINAL order; segment s owns cells [s*T, (s+1)*T);
                                  inside a segment the cells are numbered row-major over the grid, last binning
                                  dimension fastest (the flattening of Algorithm 1).  A cell is a bin, or, with
                                  sub_bins > 1, one of the sub_bins equal slices every bin is cut into along the last
                                  binning dimension (that dimension then counts n_bins * sub_bins cells; bin b of the
                                  plain numbering is cells [b*sub_bins, (b+1)*sub_bins)) */
    const int32_t* bin_bounds; /* [n_segments*T + 1] exclusive prefix of cell populations: cell c holds
                                  sorted positions [bin_bounds[c], bin_bounds[c+1]) */
    const float* sorted_points;/* [n][record_floats] the points in bin order, one record each: the d coordinates, then
                                  the original row index (an int32 stored in the float's 4 bytes), then zeros.  The
                                  index fields, read in order, are the permutation sorted position -> original row */
    const float* seg_geom;     /* [n_segments][d_bin][4]: lower box edge, cells per unit length (0 if the
                                  segment has zero extent in that dimension), cell width, rounding slack */
    int64_t cells_per_segment; /* T = n_bins^d_bin * sub_bins */
    int32_t n_bins;            /* bins per binning dimension actually used */
    int32_t d_bin;             /* binning dimensions actually used (the first d_bin coordinates) */
    int32_t sub_bins;          /* slices per bin along the last binning dimension: 1, 2 or 4, chosen by fg_bin_points
                                  (the search prunes by slice inside the runs of bins it scans; the result does not
                                  depend on it) */
    int32_t record_floats;     /* floats per record of sorted_points: d + 1 rounded up to a multiple of 4 */
    void* scratch;             /* opaque: scratch of the query stage inside the workspace.  Its first int32 holds, after
                                  fg_query_binned, the number of queries the tile kernel handed to the list kernel (a
                                  diagnostic; nothing else in it is meant to be read) */
} fg_binning;

/* Options of the query stage; none changes the result.  A NULL pointer means all defaults. */
typedef struct {
    const int32_t* dir;        /* [n] direction flags in ORIGINAL row order (see fg_binned_select_knn_dir), or NULL */
    int32_t algo;              /* 0: tile kernel + list kernel (default); 1: the one-lane-per-query shell walk for
                                  every query (slower; kept for cross-checking); 2: as 0, with the tile kernel's
                                  flattened scan on every tile instead of the uneven ones only (for tests) */
    int32_t defer_lanes;       /* after shell 1 a wavefront of the tile kernel goes on to the next shell only while
                                  more than this many of its 64 queries are unfinished, the rest go to the list
                                  kernel; 0..64, negative: the default (64 for d <= 5, 6 beyond) */
} fg_query_options;

/* Spatial partition + counting sort (Section 3, second paragraph: bins per row split, points ordered by bin,
 * cumulative bin boundaries; Algorithm 2 inputs binIdx, binBounds, binCounts, binWidths; bins numbered
 * row-major as in Algorithm 1).
 * Per row split: bounding box over the first d_bin coordinates; bin of a point in dimension c =
 * min(n_bins-1, floor((x_c - lo_c) * n_bins / (hi_c - lo_c))), 0 if hi_c == lo_c.
 *   coords      [n][d] row-major float32
 *   row_splits  [n_segments+1] int32
 *   k_hint      the K of the search that will follow (only the automatic bin count depends on it)
 *   n_bins      bins per dimension, <= 0: auto (mode 1);  d_bin likewise
 *   view        host out: where the results live inside `workspace`
 * The order of points inside one bin is unspecified.  n == 0: FG_OK, nothing enqueued. */
fg_status fg_bin_points(const float* coords, const int32_t* row_splits, int64_t n, int32_t d,
                        int32_t n_segments, int32_t k_hint, int32_t n_bins, int32_t d_bin,
                        void* workspace, size_t workspace_bytes, fg_binning* view, void* stream);

/* Exact K nearest neighbours of every point inside its own row split (Algorithm 2;
 * fg_bin_points followed by the shell-expanding query kernel).
 *   out_idx [n][k] int32   slot 0 = the row itself; slots 1.. = the k-1 nearest other points of
 *                          the row split as ORIGINAL row indices, ascending by (squared distance,
 *                          index); -1 where the row split has fewer than k points
 *   out_d2  [n][k] float32 matching squared distances (0 at slot 0 and at padding); each is the
 *                          left-to-right float32 sum over all d coordinates of the float32 squares
 *                          of the float32 differences, every operation rounded on its own
 * Rows are in the caller's original order.  The result is deterministic and independent of
 * n_bins, d_bin, the stream and the run.  k_hint of fg_bin_points is k here. */
fg_status fg_binned_select_knn(const float* coords, const int32_t* row_splits, int64_t n,
                               int32_t d, int32_t n_segments, int32_t k, int32_t n_bins,
                               int32_t d_bin, int32_t* out_idx, float* out_d2,
                               void* workspace, size_t workspace_bytes, void* stream);

/* fg_binned_select_knn for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, result and error behaviour
 * as fg_binned_select_knn, without workspace: the scratch lives in a device array inside the library
 * (FG_STATIC_SCRATCH_BYTES per GPU, held until the process ends).  The call allocates nothing and calls no
 * allocating routine.  A problem whose workspace would be larger returns FG_ERR_WORKSPACE (nothing enqueued):
 * roughly n * (4 d + 40) bytes plus 4 bytes per bin must fit, e.g. 600,000 points of d = 3.  Every call on a GPU
 * uses that GPU's one array: calls that overlap in time on one GPU (different streams, different threads) race and
 * must be serialised by the caller; calls in sequence on one stream are fine.  The array's address is looked up on
 * the first call on each device (with that device current), which should therefore happen outside graph capture. */
#define FG_STATIC_SCRATCH_BYTES (32u << 20)
fg_status fg_binned_select_knn_static(const float* coords, const int32_t* row_splits, int64_t n,
                                      int32_t d, int32_t n_segments, int32_t k, int32_t n_bins,
                                      int32_t d_bin, int32_t* out_idx, float* out_d2, void* stream);

/* Direction-flag variant (Algorithm 2, inputs useDir and dir[]): dir [n] int32, one flag per point:
 *   0  the point can be a neighbour but issues no query
 *   1  the point queries but is nobody's neighbour
 *   2  neither
 *   any other value: both (the plain behaviour)
 * The row of a point that issues no query is all padding (index -1, distance 0, slot 0 included).
 * A querying point is its own slot 0 whatever its flag.  dir == NULL: same as fg_binned_select_knn. */
fg_status fg_binned_select_knn_dir(const float* coords, const int32_t* row_splits, const int32_t* dir,
                                   int64_t n, int32_t d, int32_t n_segments, int32_t k, int32_t n_bins,
                                   int32_t d_bin, int32_t* out_idx, float* out_d2,
                                   void* workspace, size_t workspace_bytes, void* stream);

/* Same as fg_binned_select_knn, and additionally writes, per row, the number of candidate
 * squared distances evaluated for it (Algorithm 2's inner loop trip count) into
 * out_candidates [n] int32 (may not be NULL).  For measurement; slower than the plain call. */
fg_status fg_binned_select_knn_counted(const float* coords, const int32_t* row_splits, int64_t n,
                                       int32_t d, int32_t n_segments, int32_t k, int32_t n_bins,
                                       int32_t d_bin, int32_t* out_idx, float* out_d2,
                                       int32_t* out_candidates,
                                       void* workspace, size_t workspace_bytes, void* stream);

/* Query stage alone on an existing binning (what fg_binned_select_knn runs after
 * fg_bin_points); `view` must come from fg_bin_points on the same coords/row_splits and its
 * workspace must still be intact.  Used to time the query kernel on its own.
 * options: host pointer, may be NULL. */
fg_status fg_query_binned(const fg_binning* view, const int32_t* row_splits, int64_t n, int32_t d,
                          int32_t n_segments, int32_t k, int32_t* out_idx, float* out_d2,
                          int32_t* out_candidates /* may be NULL */, const fg_query_options* options,
                          void* stream);

/* Backward of the squared distances (Section 3, last paragraph):
 *   grad_coords[v][c]  = sum_j grad_d2[v][j] * 2 * (x[v][c] - x[idx[v][j]][c])
 *                      - sum_{(w,j): idx[w][j] = v} grad_d2[w][j] * 2 * (x[w][c] - x[v][c])
 * over entries with 0 <= idx < n (negative = padding; out-of-range entries are ignored).
 *   grad_d2 [n][k] float32, idx [n][k] int32 (as returned by the forward), coords [n][d]
 *   grad_coords [n][d] float32, overwritten (zero-filled by the call, then accumulated with
 *   float32 atomics: the summation order, hence the last bits, may differ between runs).
 *   row_splits [n_segments+1], workspace: optional.  With both given (workspace as for
 *   fg_binned_select_knn with this k and automatic bins) the rows are processed in bin order and
 *   contributions to the same destination are combined in LDS before they reach memory, which
 *   is several times faster; with row_splits == NULL or workspace == NULL every contribution is
 *   one global atomic.  A workspace that is given but too small is FG_ERR_WORKSPACE. */
fg_status fg_knn_backward(const float* grad_d2, const int32_t* idx, const float* coords,
                          const int32_t* row_splits, int64_t n, int32_t d, int32_t n_segments, int32_t k,
                          float* grad_coords, void* workspace, size_t workspace_bytes, void* stream);

/* The same backward on an existing binning (Section 3: the points are sorted by their bins once; the training
 * step that ran the forward on these points has that order already).  `view` must come from fg_bin_points on the
 * same coords, and the workspace it points into must not have been written since, except by fg_query_binned.
 * Its bin order is the row order; nothing is binned again (on 1M points the re-binning is a quarter of
 * fg_knn_backward's time).  Arguments, result and error behaviour as for fg_knn_backward; view == NULL or a view
 * without a row order is FG_ERR_NULL. */
fg_status fg_knn_backward_binned(const fg_binning* view, const float* grad_d2, const int32_t* idx,
                                 const float* coords, int64_t n, int32_t d, int32_t k, float* grad_coords,
                                 void* stream);

/* Object-condensation index matrices (Section 5, Algorithm 3).
 *   asso_idx       [n_vert] int32  object id each vertex is associated with (any value that is no object id,
 *                                  e.g. -1, means none)
 *   unique_idx     [n_unique]      the object ids
 *   unique_rs_asso [n_unique]      row split each object lives in (values outside 0..n_splits-1 are clamped)
 *   rs             [n_splits+1]    row splits
 *   M     [n_maxuq][n_unique] out  entry `fill` of object k at M[fill * n_unique + k] (the paper's index macro):
 *                                  the vertices of the object's row split with asso_idx == unique_idx[k], in walk
 *                                  order, at most n_maxuq of them, then -1
 *   M_not [n_maxrs][n_unique] out  (only if calc_m_not != 0; may be NULL otherwise) the vertices of the walk that
 *                                  are not associated with the object, then -1
 * The walk of object k covers the first min(split size, n_maxrs) vertices of its row split, starting
 * (k mod rot_block) vertices in and wrapping round (in the paper the offset is the thread index inside the launch
 * block, whose size the paper does not state; rot_block = 1 gives plain ascending order).  A row of M stops at
 * n_maxuq entries (the printed listing would write one more).  n_unique == 0: FG_OK, nothing enqueued.
 * workspace: optional device scratch of fg_oc_helper_workspace_size() bytes, 256-byte aligned.  With it the
 * walk is cut into chunks that run in parallel (much faster for long row splits); without it (NULL) one lane
 * walks a whole row split, as in the paper.  Same result either way.
 * Errors: FG_ERR_NULL, FG_ERR_BAD_SHAPE (negative sizes, n_maxuq < 1, n_maxrs < 1, rot_block < 1, n_splits < 1),
 * FG_ERR_WORKSPACE (given but too small or misaligned). */
fg_status fg_oc_helper_workspace_size(int64_t n_unique, int32_t n_maxrs, size_t* bytes /* host out */);
fg_status fg_oc_helper(const int32_t* asso_idx, const int32_t* unique_idx, const int32_t* unique_rs_asso,
                       const int32_t* rs, int64_t n_vert, int64_t n_unique, int32_t n_splits, int32_t n_maxuq,
                       int32_t n_maxrs, int32_t calc_m_not, int32_t rot_block, int32_t* M, int32_t* M_not,
                       void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FASTGRAPH_H */
