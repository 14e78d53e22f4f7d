// moe_permute: per-replica token lists of one rank (a stable counting sort of the pairs
// routed to that rank by local slot), built by one workgroup with wavefront ballots.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_utils.h"
#include "metro.h"

namespace metro {
namespace {

constexpr int kThreads = kListThreads;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxSpr = kListMaxSpr;

__global__ __launch_bounds__(kThreads) void permute_kernel(const int32_t* __restrict__ pair_slot, int n, int rank,
                                                           int spr, int32_t* __restrict__ group_offsets,
                                                           int32_t* __restrict__ perm_pair,
                                                           int32_t* __restrict__ pair_row,
                                                           int32_t* __restrict__ n_pairs) {
    __shared__ int s_hist[kWaves * kMaxSpr];
    __shared__ int s_cnt[kMaxSpr];
    __shared__ int s_off[kMaxSpr + 1];
    const int lo = rank * spr;
    auto key_of = [&](int p) {
        const int l = pair_slot[p] - lo;
        return (l >= 0 && l < spr) ? l : -1;
    };
    build_token_lists(key_of, nullptr, n, spr, s_hist, s_cnt, s_off, group_offsets, perm_pair, pair_row, n_pairs);
}

}  // namespace
}  // namespace metro

extern "C" int moe_permute(const int32_t* pair_slot, int T, int k, int rank, int spr, int32_t* group_offsets,
                           int32_t* perm_pair, int32_t* pair_row, int32_t* n_pairs, void* stream) {
    using namespace metro;
    if (!group_offsets || !n_pairs) return METRO_ERR_INVALID_ARG;
    if (T < 0 || k < 1 || rank < 0 || spr < 1) return METRO_ERR_INVALID_ARG;
    if ((!pair_slot || !perm_pair || !pair_row) && T > 0) return METRO_ERR_INVALID_ARG;
    if (spr > kMaxSpr || rank >= 64 || (int64_t)T * k >= (1 << 24)) return METRO_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(permute_kernel, dim3(1), dim3(kThreads), 0, (hipStream_t)stream, pair_slot, T * k, rank,
                       spr, group_offsets, perm_pair, pair_row, n_pairs);
    return hipGetLastError() == hipSuccess ? METRO_OK : METRO_ERR_HIP;
}
