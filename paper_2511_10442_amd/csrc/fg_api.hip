// C-ABI entry points: argument validation, workspace layout, stage launches.
#include <math.h>
#include <mutex>
#include "fg_internal.hpp"

// Workspace of fg_binned_select_knn_static: device memory that belongs to the library, one copy per GPU, held
// until the process ends.  In host code this name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[FG_STATIC_SCRATCH_BYTES];

namespace fg {

hipError_t launch_query_d2(const QueryArgs&, int32_t, hipStream_t);
hipError_t launch_query_d3(const QueryArgs&, int32_t, hipStream_t);
hipError_t launch_query_d4(const QueryArgs&, int32_t, hipStream_t);
hipError_t launch_query_d5(const QueryArgs&, int32_t, hipStream_t);
hipError_t launch_query_d6(const QueryArgs&, int32_t, hipStream_t);
hipError_t launch_query_d7(const QueryArgs&, int32_t, hipStream_t);
hipError_t launch_query_d8(const QueryArgs&, int32_t, hipStream_t);
hipError_t launch_query_d9(const QueryArgs&, int32_t, hipStream_t);
hipError_t launch_query_d10(const QueryArgs&, int32_t, hipStream_t);

hipError_t launch_query(const QueryArgs& a, int32_t d, int32_t d_bin, hipStream_t stream)
{
    switch (d) {
        case 2: return launch_query_d2(a, d_bin, stream);
        case 3: return launch_query_d3(a, d_bin, stream);
        case 4: return launch_query_d4(a, d_bin, stream);
        case 5: return launch_query_d5(a, d_bin, stream);
        case 6: return launch_query_d6(a, d_bin, stream);
        case 7: return launch_query_d7(a, d_bin, stream);
        case 8: return launch_query_d8(a, d_bin, stream);
        case 9: return launch_query_d9(a, d_bin, stream);
        case 10: return launch_query_d10(a, d_bin, stream);
        default: return hipErrorInvalidValue;
    }
}

namespace {

constexpr size_t kAlign = 256;

// fg_auto_n_bins mode 1.  The tile kernel is at its best when one shell around the query's bin
// (3 bins per dimension) is enough for most queries, i.e. when the bin width is about the
// radius r_K of the ball that holds K points at the mean density of a row split:
//   r_K = extent * (K / (n_elems * V_d))^(1/d),  V_d = volume of the unit ball in d dimensions,
// so bins per dimension = margin * (n_elems * V_d / K)^(1/d).  Same functional form as
// the paper's heuristic (a power 1/d of n_elems / K), with the constant 32 replaced by V_d and
// the exponent taken over all d coordinates because the distance is.  Binning dimensions: all of
// them up to 5, the first 5 beyond (the paper's limit).
// From d = 6 on a cube of 3 bins per side wastes most of its volume outside the ball, and
// smaller bins searched two shells deep (with box pruning) measured faster.
// Margins measured on uniform data (1e5..1e6 points, K = 10..100) and on the clustered
// configurations.  For d <= 5 the bin width is ~1.1 r_K: finer grids are as fast or faster on
// clustered data and for K >= 40, but for small K a large share of the queries then needs a
// second shell and leaves the tile kernel.  d = 6: ~0.6 r_K (flat between 1.2 and 1.7); d >= 7: ~0.55 r_K
// (1M uniform points, K = 40: d = 8 67 -> 54 ms, d = 10 243 -> 179 ms against 1.6; configuration 4 34 -> 28 ms).
constexpr double kTunedMarginByDim[11] = {0, 0, 0.9, 0.9, 0.9, 0.9, 1.6, 1.85, 1.85, 1.85, 1.85};
constexpr int32_t kTunedMaxBins = 1024;
// Hand-over threshold of the tile kernel (fg_query_options::defer_lanes).  Up to five dimensions every query that
// is not certified after shell 1 goes to the list kernel (64: a wavefront never starts shell 2): the automatic grids
// there are made for one shell, what is left after it are the sparse neighbourhoods, and one query per wavefront
// takes those from where they stand faster than a tile does with most of its lanes idle (1M-point clustered
// workload -6 %, the 100k-point Gaussian mixture -23 %, uniform data -1..-5 %).  From six dimensions on the grids
// are made for two shells and a tile goes on while more than 6 lanes search (always handing over: +19 % at d = 6,
// x2 at d = 8).
constexpr int32_t default_defer_lanes(int32_t d) { return d <= 5 ? 64 : 6; }
constexpr int kScanChunkHost = 256 * 16;   // must match the scan kernels' chunk

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// The query stage's scratch block (fg_binning::scratch): hand-over counter first (the one word documented in the
// header), then the work list, the tile order and an [n] array that the counting sort uses for the ranks inside
// the cells and the query stage afterwards for the tiles' hand-over marks (8 bytes per 64 points).
struct ScratchLayout { size_t work_count, work_list, tile_order, rank, total; };

ScratchLayout scratch_layout(int64_t n)
{
    ScratchLayout S;
    size_t off = 0;
    S.work_count = off; off = align_up(off + sizeof(int32_t));
    S.work_list = off;  off = align_up(off + sizeof(int32_t) * (size_t)n);
    S.tile_order = off; off = align_up(off + sizeof(int32_t) * (size_t)(2 * ((n + 63) / 64) + 128));
    S.rank = off;       off = align_up(off + sizeof(int32_t) * (size_t)n);
    S.total = off;
    return S;
}

struct Layout {
    size_t keys, geom, bin_idx, perm, rec, bounds, partials, scratch, total;
    int64_t total_bins, cells_per_segment;
};

// Slices per bin along the last binning dimension, as a shift.  Bins adjacent in that dimension are adjacent in
// the sorted order, so a query's candidates are runs of whole bins; with every bin cut into slices (and the points
// sorted by slice) a run can end at the slice where the k-th best stops reaching instead of at the bin's end, for
// nothing but a longer boundary table.  Measured with four slices: 1M clustered points, d = 3, K = 32: 10 % fewer
// candidates, query stage -5 %, counting sort +12 us (more distinct cells per block, more counter atomics), and
// the backward pass, whose rows follow the same order, -6 %; 1M uniform points, d = 3..5: -2..-4 %; 5M points of
// strongly skewed density, d = 2: 22.0 -> 15.3 ms; 500k uniform points, d = 8: 24.8 -> 22.3 ms.  The gain stays well
// below the drop in candidates because a wavefront scans a column as long as its longest lane does.  Four slices
// while the table stays within the limit and near the number of points.
int32_t choose_sub_shift(int64_t n, int32_t n_segments, int32_t n_bins, int32_t d_bin)
{
    double cells = (double)n_segments;
    for (int c = 0; c < d_bin; ++c) cells *= n_bins;
    for (int32_t sh = 2; sh > 0; --sh) {
        const double sliced = cells * (1 << sh);
        if (sliced <= (double)FG_MAX_TOTAL_BINS && sliced <= 2.0 * (double)n + 4096.0) return sh;
    }
    return 0;
}

// n_bins, d_bin already resolved and validated
Layout make_layout(int64_t n, int32_t d, int32_t n_segments, int32_t n_bins, int32_t d_bin, int32_t sub_shift)
{
    Layout L;
    int64_t cells = (int64_t)1 << sub_shift;
    for (int c = 0; c < d_bin; ++c) cells *= n_bins;
    L.cells_per_segment = cells;
    L.total_bins = cells * n_segments;
    size_t off = 0;
    L.keys = off;     off = align_up(off + sizeof(uint32_t) * 2 * (size_t)n_segments * d_bin * kKeyStride);
    L.geom = off;     off = align_up(off + sizeof(float) * kGeomStride * (size_t)n_segments * d_bin);
    L.bin_idx = off;  off = align_up(off + sizeof(int32_t) * (size_t)n);
    L.perm = off;     off = align_up(off + sizeof(int32_t) * (size_t)n);      // the backward's own row order only
    L.rec = off;      off = align_up(off + sizeof(float) * 4 * (size_t)rec_vecs(d) * (size_t)n);
    L.bounds = off;   off = align_up(off + sizeof(int32_t) * (size_t)(L.total_bins + 1));
    L.partials = off; off = align_up(off + sizeof(int32_t) * (size_t)((L.total_bins + 1 + kScanChunkHost - 1) / kScanChunkHost));
    L.scratch = off;  off = align_up(off + scratch_layout(n).total);
    L.total = off;
    return L;
}

fg_status check_problem(int64_t n, int32_t d, int32_t n_segments, int32_t k)
{
    // n: launch grids and chunk counts are 32-bit sums of n and a block size; n_segments: offsets into the
    // bounding-box keys and geometry records are 32-bit products of a few hundred and n_segments
    if (n < 0 || n > FG_MAX_N || n_segments < 1 || n_segments > FG_MAX_SEGMENTS || k < 1) return FG_ERR_BAD_SHAPE;
    if (d < FG_MIN_D || d > FG_MAX_D || k > FG_MAX_K) return FG_ERR_UNSUPPORTED;
    return FG_OK;
}

// fills in automatic values, validates explicit ones
fg_status resolve_bins(int64_t n, int32_t d, int32_t n_segments, int32_t k, int32_t* n_bins, int32_t* d_bin)
{
    int32_t auto_n = 0, auto_db = 0;
    fg_status st = fg_auto_n_bins(n, n_segments, k, d, 1, &auto_n, &auto_db);
    if (st != FG_OK) return st;
    if (*d_bin <= 0) {
        *d_bin = auto_db;
        if (*n_bins > 0) {   // explicit n_bins with automatic d_bin: keep the bin table within bounds
            while (*d_bin > FG_MIN_D_BIN && pow((double)*n_bins, *d_bin) * n_segments > (double)FG_MAX_TOTAL_BINS) --*d_bin;
        }
    }
    if (*d_bin < FG_MIN_D_BIN || *d_bin > FG_MAX_D_BIN || *d_bin > d) return FG_ERR_UNSUPPORTED;
    if (*n_bins <= 0) {
        if (*d_bin == auto_db) *n_bins = auto_n;
        else {   // explicit d_bin with automatic n_bins: same occupancy target over d_bin dimensions
            double cells = pow((double)auto_n, auto_db);
            int32_t v = (int32_t)floor(pow(cells, 1.0 / *d_bin) + 1e-9);
            *n_bins = v < 1 ? 1 : v;
        }
    }
    double total = pow((double)*n_bins, *d_bin) * n_segments;
    if (*n_bins < 1 || total > (double)FG_MAX_TOTAL_BINS) return FG_ERR_BAD_SHAPE;
    return FG_OK;
}

}  // namespace
}  // namespace fg

using namespace fg;

static int32_t backward_morton_bits(int64_t n, int32_t d, int32_t n_segments, int32_t k, int32_t* d_bin);

extern "C" {

const char* fg_status_string(fg_status status)
{
    switch (status) {
        case FG_OK: return "FG_OK";
        case FG_ERR_NULL: return "FG_ERR_NULL: a required pointer is NULL";
        case FG_ERR_BAD_SHAPE: return "FG_ERR_BAD_SHAPE: size or bin count out of range";
        case FG_ERR_UNSUPPORTED: return "FG_ERR_UNSUPPORTED: d, k or d_bin outside the supported range";
        case FG_ERR_WORKSPACE: return "FG_ERR_WORKSPACE: workspace too small or misaligned";
        case FG_ERR_LAUNCH: return "FG_ERR_LAUNCH: HIP launch failed";
        default: return "unknown fg_status";
    }
}

fg_status fg_auto_n_bins(int64_t n, int32_t n_segments, int32_t k, int32_t d, int32_t mode,
                         int32_t* n_bins, int32_t* d_bin)
{
    if (!n_bins || !d_bin) return FG_ERR_NULL;
    fg_status st = check_problem(n, d, n_segments, k);
    if (st != FG_OK) return st;
    if (mode != 0 && mode != 1) return FG_ERR_BAD_SHAPE;
    const double n_elems = (double)n / (double)n_segments;
    if (mode == 0) {
        // Section 3: (32 n_elems / K)^(1/d_max), clamped to [5, 30]; at most the first 5 dimensions
        const int32_t db = d < 5 ? d : 5;
        double x = n_elems > 0 ? pow(32.0 * n_elems / (double)k, 1.0 / db) : 0.0;
        int32_t v = (int32_t)floor(x + 1e-9);
        v = v < 5 ? 5 : (v > 30 ? 30 : v);
        while (db > 0 && pow((double)v, db) * n_segments > (double)FG_MAX_TOTAL_BINS && v > 1) --v;
        *n_bins = v;
        *d_bin = db;
        return FG_OK;
    }
    // mode 1: bin width ~ radius of the K-ball at mean density (kTunedMarginByDim, kTunedMaxBins)
    const int32_t db = d < 5 ? d : 5;
    const double unit_ball = pow(M_PI, 0.5 * d) / tgamma(0.5 * d + 1.0);
    const double margin = kTunedMarginByDim[d];
    double x = n_elems > 0 ? margin * pow(n_elems * unit_ball / (double)k, 1.0 / d) : 1.0;
    int32_t v = (int32_t)floor(x + 0.5);
    v = v < 1 ? 1 : (v > kTunedMaxBins ? kTunedMaxBins : v);
    while (pow((double)v, db) * n_segments > (double)FG_MAX_TOTAL_BINS && v > 1) --v;
    *n_bins = v;
    *d_bin = db;
    return FG_OK;
}

fg_status fg_workspace_size(int64_t n, int32_t d, int32_t n_segments, int32_t k,
                            int32_t n_bins, int32_t d_bin, size_t* bytes)
{
    if (!bytes) return FG_ERR_NULL;
    fg_status st = check_problem(n, d, n_segments, k);
    if (st != FG_OK) return st;
    st = resolve_bins(n, d, n_segments, k, &n_bins, &d_bin);
    if (st != FG_OK) return st;
    size_t need = make_layout(n, d, n_segments, n_bins, d_bin, choose_sub_shift(n, n_segments, n_bins, d_bin)).total;
    int32_t db_b = 0;
    const int32_t bits = backward_morton_bits(n, d, n_segments, k, &db_b);   // fg_knn_backward's own grid
    if (bits > 0) {
        const size_t need_b = make_layout(n, d, n_segments, 1 << bits, db_b, 0).total;
        if (need_b > need) need = need_b;
    }
    *bytes = need;
    return FG_OK;
}

// Bits per dimension of the bit-interleaved bin order the backward pass sorts its rows by: the power of two
// nearest to the automatic bin count (the order only has to be spatially coherent, any grid will do).
static int32_t backward_morton_bits(int64_t n, int32_t d, int32_t n_segments, int32_t k, int32_t* d_bin)
{
    int32_t nb = 0;
    if (fg_auto_n_bins(n, n_segments, k, d, 1, &nb, d_bin) != FG_OK) return 0;
    int32_t bits = (int32_t)floor(log2((double)(nb < 2 ? 2 : nb)) + 0.5);
    if (bits < 1) bits = 1;
    while (bits > 1 && (bits * *d_bin > 24 || pow(2.0, bits * *d_bin) * n_segments > (double)FG_MAX_TOTAL_BINS)) --bits;
    return bits;
}

// n_bins, d_bin resolved and validated by the caller
static fg_status bin_points_impl(const float* coords, const int32_t* row_splits, int64_t n, int32_t d,
                                 int32_t n_segments, int32_t n_bins, int32_t d_bin, int32_t morton_bits,
                                 void* workspace, size_t workspace_bytes, fg_binning* view, void* stream)
{
    if (!coords && n > 0) return FG_ERR_NULL;
    if (!row_splits || !workspace) return FG_ERR_NULL;
    const int32_t sub_shift = morton_bits > 0 ? 0 : choose_sub_shift(n, n_segments, n_bins, d_bin);
    const Layout L = make_layout(n, d, n_segments, n_bins, d_bin, sub_shift);
    if (((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < L.total) return FG_ERR_WORKSPACE;
    char* ws = (char*)workspace;
    view->bin_idx = (const int32_t*)(ws + L.bin_idx);
    view->bin_bounds = (const int32_t*)(ws + L.bounds);
    view->sorted_points = (const float*)(ws + L.rec);
    view->seg_geom = (const float*)(ws + L.geom);
    view->record_floats = 4 * rec_vecs(d);
    view->cells_per_segment = L.cells_per_segment;
    view->n_bins = n_bins;
    view->d_bin = d_bin;
    view->sub_bins = 1 << sub_shift;
    view->scratch = ws + L.scratch;
    if (n == 0) return FG_OK;
    hipError_t e = launch_binning(coords, row_splits, (int32_t)n, d, n_segments, n_bins, d_bin, sub_shift, L.total_bins,
                                  (uint32_t*)(ws + L.keys), (float*)(ws + L.geom), (int32_t*)(ws + L.bin_idx),
                                  (int32_t*)(ws + L.scratch + scratch_layout(n).rank), (int32_t*)(ws + L.perm), (float*)(ws + L.rec),
                                  (int32_t*)(ws + L.bounds), (int32_t*)(ws + L.partials), morton_bits,
                                  (hipStream_t)stream);
    return e == hipSuccess ? FG_OK : FG_ERR_LAUNCH;
}

fg_status fg_bin_points(const float* coords, const int32_t* row_splits, int64_t n, int32_t d,
                        int32_t n_segments, int32_t k_hint, int32_t n_bins, int32_t d_bin,
                        void* workspace, size_t workspace_bytes, fg_binning* view, void* stream)
{
    if (!view) return FG_ERR_NULL;
    fg_status st = check_problem(n, d, n_segments, k_hint);
    if (st != FG_OK) return st;
    st = resolve_bins(n, d, n_segments, k_hint, &n_bins, &d_bin);
    if (st != FG_OK) return st;
    return bin_points_impl(coords, row_splits, n, d, n_segments, n_bins, d_bin, 0, workspace, workspace_bytes, view,
                           stream);
}

fg_status fg_query_binned(const fg_binning* view, const int32_t* row_splits, int64_t n, int32_t d,
                          int32_t n_segments, int32_t k, int32_t* out_idx, float* out_d2,
                          int32_t* out_candidates, const fg_query_options* options, void* stream)
{
    if (!view) return FG_ERR_NULL;
    fg_status st = check_problem(n, d, n_segments, k);
    if (st != FG_OK) return st;
    if (n == 0) return FG_OK;
    if (!row_splits || !out_idx || !out_d2 || !view->bin_bounds || !view->sorted_points || !view->seg_geom ||
        !view->scratch)
        return FG_ERR_NULL;
    if (view->d_bin < FG_MIN_D_BIN || view->d_bin > FG_MAX_D_BIN || view->d_bin > d) return FG_ERR_UNSUPPORTED;
    if (view->sub_bins != 1 && view->sub_bins != 2 && view->sub_bins != 4) return FG_ERR_BAD_SHAPE;
    if (view->n_bins < 1 || view->cells_per_segment < 1 ||
        view->cells_per_segment * (int64_t)n_segments > FG_MAX_TOTAL_BINS || view->record_floats != 4 * rec_vecs(d))
        return FG_ERR_BAD_SHAPE;
    QueryArgs a;
    a.rec = reinterpret_cast<const float4*>(view->sorted_points); a.bounds = view->bin_bounds; a.geom = view->seg_geom;
    const ScratchLayout S = scratch_layout(n);
    char* sc = (char*)view->scratch;
    const int32_t* dir = options ? options->dir : nullptr;
    const int32_t defer = (options && options->defer_lanes >= 0) ? options->defer_lanes : default_defer_lanes(d);
    a.row_splits = row_splits; a.dir = dir; a.out_idx = out_idx; a.out_d2 = out_d2; a.out_cand = out_candidates;
    a.n = (int32_t)n; a.d = d; a.n_segments = n_segments; a.k = k;
    a.n_bins = view->n_bins; a.cells_per_segment = (int32_t)view->cells_per_segment;
    a.sub_shift = view->sub_bins == 4 ? 2 : (view->sub_bins == 2 ? 1 : 0);
    a.work_list = (int32_t*)(sc + S.work_list); a.work_count = (int32_t*)(sc + S.work_count);
    a.handed = (uint64_t*)(sc + S.rank);       // the counting sort is done with its ranks
    a.bin_idx = view->bin_idx; a.tile_order = (int32_t*)(sc + S.tile_order);
    a.algo = (options && (options->algo == 1 || options->algo == 2)) ? options->algo : 0;
    a.defer_lanes = defer > 64 ? 64 : defer;
    hipError_t e = launch_query(a, d, view->d_bin, (hipStream_t)stream);
    return e == hipSuccess ? FG_OK : FG_ERR_LAUNCH;
}

static fg_status knn_impl(const float* coords, const int32_t* row_splits, const int32_t* dir, int64_t n, int32_t d, int32_t n_segments,
                          int32_t k, int32_t n_bins, int32_t d_bin, int32_t* out_idx, float* out_d2,
                          int32_t* out_candidates, void* workspace, size_t workspace_bytes, void* stream)
{
    fg_status st = check_problem(n, d, n_segments, k);
    if (st != FG_OK) return st;
    if (n == 0) return FG_OK;
    if (!out_idx || !out_d2) return FG_ERR_NULL;
    fg_binning view;
    st = fg_bin_points(coords, row_splits, n, d, n_segments, k, n_bins, d_bin, workspace, workspace_bytes, &view,
                       stream);
    if (st != FG_OK) return st;
    fg_query_options opt;
    opt.dir = dir;
    opt.algo = 0;
    opt.defer_lanes = -1;
    return fg_query_binned(&view, row_splits, n, d, n_segments, k, out_idx, out_d2, out_candidates, &opt, stream);
}

fg_status fg_binned_select_knn(const float* coords, const int32_t* row_splits, int64_t n,
                               int32_t d, int32_t n_segments, int32_t k, int32_t n_bins,
                               int32_t d_bin, int32_t* out_idx, float* out_d2,
                               void* workspace, size_t workspace_bytes, void* stream)
{
    return knn_impl(coords, row_splits, nullptr, n, d, n_segments, k, n_bins, d_bin, out_idx, out_d2, nullptr, workspace,
                    workspace_bytes, stream);
}

// Address of `scratch` on the current device, looked up once per device.
static fg_status static_scratch_address(void** out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* address[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FG_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(mu);
    if (!address[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return FG_ERR_LAUNCH;
        address[dev] = ptr;
    }
    *out = address[dev];
    return FG_OK;
}

fg_status fg_binned_select_knn_static(const float* coords, const int32_t* row_splits, int64_t n,
                                      int32_t d, int32_t n_segments, int32_t k, int32_t n_bins,
                                      int32_t d_bin, int32_t* out_idx, float* out_d2, void* stream)
{
    fg_status st = check_problem(n, d, n_segments, k);
    if (st != FG_OK) return st;
    if (n == 0) return FG_OK;
    st = resolve_bins(n, d, n_segments, k, &n_bins, &d_bin);
    if (st != FG_OK) return st;
    if (make_layout(n, d, n_segments, n_bins, d_bin, choose_sub_shift(n, n_segments, n_bins, d_bin)).total >
        (size_t)FG_STATIC_SCRATCH_BYTES)
        return FG_ERR_WORKSPACE;
    void* ws = nullptr;
    st = static_scratch_address(&ws);
    if (st != FG_OK) return st;
    return knn_impl(coords, row_splits, nullptr, n, d, n_segments, k, n_bins, d_bin, out_idx, out_d2, nullptr, ws,
                    (size_t)FG_STATIC_SCRATCH_BYTES, stream);
}

fg_status fg_binned_select_knn_dir(const float* coords, const int32_t* row_splits, const int32_t* dir,
                                   int64_t n, int32_t d, int32_t n_segments, int32_t k, int32_t n_bins,
                                   int32_t d_bin, int32_t* out_idx, float* out_d2,
                                   void* workspace, size_t workspace_bytes, void* stream)
{
    return knn_impl(coords, row_splits, dir, n, d, n_segments, k, n_bins, d_bin, out_idx, out_d2, nullptr, workspace,
                    workspace_bytes, stream);
}

fg_status fg_binned_select_knn_counted(const float* coords, const int32_t* row_splits, int64_t n,
                                       int32_t d, int32_t n_segments, int32_t k, int32_t n_bins,
                                       int32_t d_bin, int32_t* out_idx, float* out_d2,
                                       int32_t* out_candidates,
                                       void* workspace, size_t workspace_bytes, void* stream)
{
    if (!out_candidates && n > 0) return FG_ERR_NULL;
    return knn_impl(coords, row_splits, nullptr, n, d, n_segments, k, n_bins, d_bin, out_idx, out_d2, out_candidates,
                    workspace, workspace_bytes, stream);
}

fg_status fg_knn_backward(const float* grad_d2, const int32_t* idx, const float* coords,
                          const int32_t* row_splits, int64_t n, int32_t d, int32_t n_segments, int32_t k,
                          float* grad_coords, void* workspace, size_t workspace_bytes, void* stream)
{
    fg_status st = check_problem(n, d, n_segments < 1 ? 1 : n_segments, k);
    if (st != FG_OK) return st;
    if (n == 0) return FG_OK;
    if (!grad_d2 || !idx || !coords || !grad_coords) return FG_ERR_NULL;
    const int32_t* perm = nullptr;
    const float* coords4 = nullptr;
    if (row_splits && workspace && n_segments >= 1) {
        // bin the points once more to get a spatially coherent row order (the forward's workspace
        // is scratch by contract, so nothing of it is assumed to survive)
        // rows sorted by bit-interleaved bin: 256 consecutive rows then form a compact block in space and
        // share more destinations than a run of bins along the last dimension would
        fg_binning view;
        int32_t db = 0;
        const int32_t bits = backward_morton_bits(n, d, n_segments, k, &db);
        if (bits < 1) return FG_ERR_BAD_SHAPE;
        st = bin_points_impl(coords, row_splits, n, d, n_segments, 1 << bits, db, bits, workspace, workspace_bytes, &view,
                             stream);
        if (st != FG_OK) return st;
        perm = (const int32_t*)((const char*)workspace + make_layout(n, d, n_segments, 1 << bits, db, 0).perm);
        if (d == 3) coords4 = view.sorted_points;    // in this mode: the rows padded to four floats, original order
    }
    hipError_t e = launch_backward(grad_d2, idx, coords, coords4, perm, 1, (int32_t)n, d, k, grad_coords, (hipStream_t)stream);
    return e == hipSuccess ? FG_OK : FG_ERR_LAUNCH;
}

fg_status fg_knn_backward_binned(const fg_binning* view, const float* grad_d2, const int32_t* idx,
                                 const float* coords, int64_t n, int32_t d, int32_t k, float* grad_coords,
                                 void* stream)
{
    if (!view) return FG_ERR_NULL;
    fg_status st = check_problem(n, d, 1, k);
    if (st != FG_OK) return st;
    if (n == 0) return FG_OK;
    if (!grad_d2 || !idx || !coords || !grad_coords || !view->sorted_points) return FG_ERR_NULL;
    if (view->record_floats != 4 * rec_vecs(d)) return FG_ERR_BAD_SHAPE;
    // the forward's bin order (runs of bins along the last binning dimension) is a little less compact than the
    // bit-interleaved order fg_knn_backward makes for itself: +0.01 ms in the kernel against 0.08 ms of binning.
    // The row of sorted position q is the index field of its point record.
    hipError_t e = launch_backward(grad_d2, idx, coords, nullptr, reinterpret_cast<const int32_t*>(view->sorted_points) + d,
                                   view->record_floats, (int32_t)n, d, k, grad_coords, (hipStream_t)stream);
    return e == hipSuccess ? FG_OK : FG_ERR_LAUNCH;
}

fg_status fg_oc_helper_workspace_size(int64_t n_unique, int32_t n_maxrs, size_t* bytes)
{
    if (!bytes) return FG_ERR_NULL;
    if (n_unique < 0 || n_unique >= ((int64_t)1 << 31) || n_maxrs < 1) return FG_ERR_BAD_SHAPE;
    *bytes = align_up(oc_workspace_bytes(n_unique, n_maxrs));
    return FG_OK;
}

fg_status fg_oc_helper(const int32_t* asso_idx, const int32_t* unique_idx, const int32_t* unique_rs_asso,
                       const int32_t* rs, int64_t n_vert, int64_t n_unique, int32_t n_splits, int32_t n_maxuq,
                       int32_t n_maxrs, int32_t calc_m_not, int32_t rot_block, int32_t* M, int32_t* M_not,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    if (n_vert < 0 || n_vert >= ((int64_t)1 << 31) || n_unique < 0 || n_unique >= ((int64_t)1 << 31) || n_splits < 1 ||
        n_maxuq < 1 || n_maxrs < 1 || rot_block < 1)
        return FG_ERR_BAD_SHAPE;
    if (n_unique == 0) return FG_OK;
    if (!asso_idx || !unique_idx || !unique_rs_asso || !rs || !M || (calc_m_not && !M_not)) return FG_ERR_NULL;
    if (workspace && (((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < oc_workspace_bytes(n_unique, n_maxrs)))
        return FG_ERR_WORKSPACE;
    hipError_t e = launch_oc_helper(asso_idx, unique_idx, unique_rs_asso, rs, (int32_t)n_vert, (int32_t)n_unique, n_splits,
                                    n_maxuq, n_maxrs, calc_m_not ? 1 : 0, rot_block, M, M_not, (int32_t*)workspace,
                                    (hipStream_t)stream);
    return e == hipSuccess ? FG_OK : FG_ERR_LAUNCH;
}

}  // extern "C"
