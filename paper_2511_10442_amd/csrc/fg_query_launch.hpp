// Host-side launch of the query stage: picks the kernel variant for (d, d_bin, K).
#pragma once
#include "fg_query.hpp"
#include "fg_query_tile.hpp"
#include "fg_query_list.hpp"

namespace fg {

static __global__ void k_reset_counter(int32_t* c) { if (threadIdx.x == 0) *c = 0; }

template <typename K>
static void allow_lds(K kernel, size_t bytes)
{
    if (bytes > 48 * 1024) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <int D, int DB, bool COUNT>
static hipError_t launch_query_impl(const QueryArgs& a, hipStream_t stream)
{
    const int grid = (a.n + kQueryBlock - 1) / kQueryBlock;
    const size_t heap_bytes = (size_t)(a.k > 1 ? a.k - 1 : 1) * kQueryBlock * sizeof(uint64_t);
    if (a.algo == 1) {
        allow_lds(k_query_shell<D, DB, COUNT>, heap_bytes);
        hipLaunchKernelGGL((k_query_shell<D, DB, COUNT>), dim3(grid), dim3(kQueryBlock), heap_bytes, stream, a);
        return hipGetLastError();
    }
    allow_lds(k_query_list<D, DB, COUNT>, heap_bytes);
    hipLaunchKernelGGL(k_reset_counter, dim3(1), dim3(64), 0, stream, a.work_count);
    const int32_t cap = a.k - 1;
    if (cap <= 16) {
        const size_t lds = tile_sorted_lds_bytes<16, D>();
        hipLaunchKernelGGL((k_query_tile_sorted<D, DB, 16, COUNT>), dim3(grid), dim3(kQueryBlock), lds, stream, a);
    } else if (cap <= 32) {
        const size_t lds = tile_sorted_lds_bytes<32, D>();
        hipLaunchKernelGGL((k_query_tile_sorted<D, DB, 32, COUNT>), dim3(grid), dim3(kQueryBlock), lds, stream, a);
    } else if (cap <= 48) {
        const size_t lds = tile_sorted_lds_bytes<48, D>();
        hipLaunchKernelGGL((k_query_tile_sorted<D, DB, 48, COUNT>), dim3(grid), dim3(kQueryBlock), lds, stream, a);
    } else if (cap <= 64) {
        const size_t lds = tile_sorted_lds_bytes<64, D>();
        hipLaunchKernelGGL((k_query_tile_sorted<D, DB, 64, COUNT>), dim3(grid), dim3(kQueryBlock), lds, stream, a);
    } else if (cap <= 96) {
        const size_t lds = tile_sorted_lds_bytes<96, D>();
        hipLaunchKernelGGL((k_query_tile_sorted<D, DB, 96, COUNT>), dim3(grid), dim3(kQueryBlock), lds, stream, a);
    } else {
        const size_t lds = tile_sorted_lds_bytes<128, D>();
        hipLaunchKernelGGL((k_query_tile_sorted<D, DB, 128, COUNT>), dim3(grid), dim3(kQueryBlock), lds, stream, a);
    }
    if (cap <= 64) {   // one query per wavefront
        const int list_grid = a.n < 8192 ? a.n : 8192;
        hipLaunchKernelGGL((k_query_list_wave<D, DB, COUNT>), dim3(list_grid), dim3(kQueryBlock), 0, stream, a);
    } else {
        const int list_grid = grid < 4096 ? grid : 4096;
        hipLaunchKernelGGL((k_query_list<D, DB, COUNT>), dim3(list_grid), dim3(kQueryBlock), heap_bytes, stream, a);
    }
    return hipGetLastError();
}

template <int D, int DB>
static hipError_t launch_query_shell(const QueryArgs& a, hipStream_t stream)
{
    return a.out_cand ? launch_query_impl<D, DB, true>(a, stream) : launch_query_impl<D, DB, false>(a, stream);
}

template <int D>
static hipError_t dispatch_query_dbin(const QueryArgs& a, int32_t d_bin, hipStream_t stream)
{
    switch (d_bin) {
        case 2: return launch_query_shell<D, 2>(a, stream);
        case 3: if constexpr (D >= 3) return launch_query_shell<D, 3>(a, stream); break;
        case 4: if constexpr (D >= 4) return launch_query_shell<D, 4>(a, stream); break;
        case 5: if constexpr (D >= 5) return launch_query_shell<D, 5>(a, stream); break;
        default: break;
    }
    return hipErrorInvalidValue;
}

}  // namespace fg
