// One translation unit per coordinate count: compile with -DFG_QUERY_D=<2..10>.
// (Compile-time specialisation per dimension, as in the paper's Section 3: loops over
// coordinates and binning dimensions unroll and per-dimension state stays in registers.)
#include "fg_query_launch.hpp"

#ifndef FG_QUERY_D
#error "define FG_QUERY_D"
#endif

#define FG_CAT2(a, b) a##b
#define FG_CAT(a, b) FG_CAT2(a, b)

namespace fg {
hipError_t FG_CAT(launch_query_d, FG_QUERY_D)(const QueryArgs& a, int32_t d_bin, hipStream_t stream)
{
    return dispatch_query_dbin<FG_QUERY_D>(a, d_bin, stream);
}
}  // namespace fg
