// Routing kernels for gfx950: the METRO greedy solve (Alg. 1, Sec. 4.3 of arxiv 2512.09277)
// and the token-balanced baseline (Sec. 2.3 / Sec. 6.1).  One workgroup solves one layer;
// every table lives in LDS.
//
// The paper's kernel runs Alg. 1 with one thread per expert and test-and-set locks on one
// SM; the order in which experts are served is whatever the lock races give.  Here the order
// is fixed (ascending expert id, ties to the lowest rank), which removes the locks and lets
// most of the serial chain collapse:
//   - an active expert with a single replica has no choice; its effect on the load L[g] seen
//     by a later expert e is a prefix popcount of a per-rank bitmap of such experts below e;
//   - only active experts with >= 2 replicas (at most S - N of them) form a serial chain, and
//     each step is an argmin over <= G lanes, done with ballots over the bits of the load.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_utils.h"
#include "metro.h"

namespace metro {
namespace {

constexpr int kMaxN = 512;
constexpr int kMaxG = 64;
constexpr int kMaxSpr = 64;
constexpr int kMaxS = 2048;   // G*spr
constexpr int kWords = kMaxN / 64;
constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kNoSlot = 0x7fffffff;

struct RouteArgs {
    const int32_t* ids;
    const int32_t* slot_to_expert;
    int T, k, N, G, spr;
    int vec4;  // 1 when every layer's id and pair_slot run is 16-byte aligned and T*k % 4 == 0
    int32_t* pair_slot;
    int32_t* expert_slot;
    int32_t* rank_active;
    uint64_t* rank_bitmap;
    int32_t* err_flag;
    // token lists of one rank, emitted by the same workgroup after pair_slot (single-layer calls only)
    int list_rank;            // < 0: no lists
    int32_t* group_offsets;
    int32_t* perm_pair;
    int32_t* pair_row;
    int32_t* n_pairs;
};

__device__ __forceinline__ uint64_t join64(uint32_t lo, uint32_t hi) { return ((uint64_t)hi << 32) | lo; }

__device__ __forceinline__ void set_bit64(uint32_t* lo, uint32_t* hi, int idx, int bit) {
    if (bit < 32) atomicOr(&lo[idx], 1u << bit);
    else atomicOr(&hi[idx], 1u << (bit - 32));
}

// Ranks hosting each expert (matrix A, one 64-bit row per expert) from slot_to_expert.
__device__ __forceinline__ void build_host_masks(const int32_t* s2e, int N, int S, int spr, uint32_t* host_lo,
                                                 uint32_t* host_hi, int* err) {
    for (int s = threadIdx.x; s < S; s += blockDim.x) {
        const int e = s2e[s];
        if (e < -1 || e >= N) atomicOr(err, METRO_FLAG_BAD_PLACEMENT);
        else if (e >= 0) set_bit64(host_lo, host_hi, e, s / spr);
    }
}

// ------------------------------------------------------------------------------------------ METRO
constexpr int kIdCache = 8;      // int4 loads of ids a thread keeps in registers between the two passes

__global__ __launch_bounds__(kThreads) void metro_route_kernel(RouteArgs a) {
    __shared__ int s_active[kMaxN];
    __shared__ uint32_t s_host_lo[kMaxN], s_host_hi[kMaxN];
    __shared__ int s_rank[kMaxN];                  // chosen rank g* of every active expert
    __shared__ int s_slot[kMaxN];                  // chosen slot
    __shared__ uint32_t s_forced_lo[kWords][kMaxG], s_forced_hi[kWords][kMaxG];
    __shared__ uint32_t s_multi_lo[kWords], s_multi_hi[kWords];
    __shared__ uint32_t s_bm_lo[kMaxG], s_bm_hi[kMaxG];
    __shared__ int s_err;
    __shared__ int s_list_hist[kWaves * kListMaxSpr], s_list_cnt[kListMaxSpr], s_list_off[kListMaxSpr + 1];

    const int layer = blockIdx.x;
    const int N = a.N, G = a.G, spr = a.spr, S = G * spr;
    const int n_pairs = a.T * a.k;
    const int32_t* ids = a.ids + (size_t)layer * n_pairs;
    const int32_t* s2e = a.slot_to_expert + (size_t)layer * S;
    int32_t* pair_slot = a.pair_slot + (size_t)layer * n_pairs;
    const int tid = threadIdx.x;

    // The global loads go out first, so that their latency overlaps the LDS set-up; the ids stay in
    // registers for the emit pass (batches beyond kIdCache*4*1024 pairs re-read the rest).
    const int4* v = reinterpret_cast<const int4*>(ids);
    const int n4 = a.vec4 ? n_pairs / 4 : 0;
    int4 idc[kIdCache];
#pragma unroll
    for (int c = 0; c < kIdCache; ++c) {
        idc[c] = make_int4(-1, -1, -1, -1);
        const int i = tid + c * kThreads;
        if (i < n4) idc[c] = v[i];
    }
    int se[kMaxS / kThreads];
#pragma unroll
    for (int j = 0; j < kMaxS / kThreads; ++j) {
        const int sl = tid + j * kThreads;
        se[j] = sl < S ? s2e[sl] : -1;
    }

    for (int e = tid; e < kMaxN; e += kThreads) {
        s_active[e] = 0;
        s_host_lo[e] = 0;
        s_host_hi[e] = 0;
        s_rank[e] = -1;
        s_slot[e] = kNoSlot;
    }
    for (int i = tid; i < kWords * kMaxG; i += kThreads) {
        (&s_forced_lo[0][0])[i] = 0;
        (&s_forced_hi[0][0])[i] = 0;
    }
    if (tid < kWords) { s_multi_lo[tid] = 0; s_multi_hi[tid] = 0; }
    if (tid < kMaxG) { s_bm_lo[tid] = 0; s_bm_hi[tid] = 0; }
    if (tid == 0) s_err = 0;
    __syncthreads();

    // Ranks hosting each expert (matrix A) and T[i] > 0 for every expert.
#pragma unroll
    for (int j = 0; j < kMaxS / kThreads; ++j) {
        const int sl = tid + j * kThreads;
        if (sl < S) {
            if (se[j] < -1 || se[j] >= N) { atomicOr(&s_err, METRO_FLAG_BAD_PLACEMENT); se[j] = -1; }
            else if (se[j] >= 0) set_bit64(s_host_lo, s_host_hi, se[j], sl / spr);
        }
    }
    auto mark = [&](int id) {
        if (id < -1 || id >= N) atomicOr(&s_err, METRO_FLAG_BAD_ID);
        else if (id >= 0) s_active[id] = 1;
    };
#pragma unroll
    for (int c = 0; c < kIdCache; ++c) {
        mark(idc[c].x); mark(idc[c].y); mark(idc[c].z); mark(idc[c].w);   // padding (-1) where not loaded
    }
    for (int i = tid + kIdCache * kThreads; i < n4; i += kThreads) {
        const int4 q = v[i];
        mark(q.x); mark(q.y); mark(q.z); mark(q.w);
    }
    if (!a.vec4)
        for (int i = tid; i < n_pairs; i += kThreads) mark(ids[i]);
    __syncthreads();

    // Split the active experts: single replica (forced) or several (the serial chain).
    for (int e = tid; e < N; e += kThreads) {
        if (!s_active[e]) continue;
        const uint64_t host = join64(s_host_lo[e], s_host_hi[e]);
        const int r = __popcll(host);
        if (r == 0) {
            atomicOr(&s_err, METRO_FLAG_NO_REPLICA);
        } else if (r == 1) {
            const int g = __ffsll((unsigned long long)host) - 1;
            s_rank[e] = g;
            set_bit64(&s_forced_lo[e >> 6][0], &s_forced_hi[e >> 6][0], g, e & 63);
        } else {
            set_bit64(s_multi_lo, s_multi_hi, e >> 6, e & 63);
        }
    }
    __syncthreads();

    // The chain: wave 0, lane g keeps L[g].  Load of rank g when expert e is served =
    //   L (all experts of lower words) + forced experts of this word below e + chain picks of this word.
    // Per 64-expert word the lanes first fetch the host masks of the word's experts (lane b <-> expert
    // 64w+b), so that the serial loop reads them with readlane instead of waiting for LDS each step.
    if (tid < kWave) {
        const int g = tid;
        int L = 0;
        int load_bits = 1;
        while ((1 << load_bits) <= spr) ++load_bits;   // L[g] <= spr always
        const int n_words = (N + 63) >> 6;
        for (int w = 0; w < n_words; ++w) {
            const uint64_t forced = g < G ? join64(s_forced_lo[w][g], s_forced_hi[w][g]) : 0ull;
            const int my_e = min((w << 6) + g, kMaxN - 1);
            const uint32_t hl = s_host_lo[my_e], hh = s_host_hi[my_e];
            uint64_t multi = join64(__builtin_amdgcn_readfirstlane(s_multi_lo[w]),
                                    __builtin_amdgcn_readfirstlane(s_multi_hi[w]));
            int picked = 0;
            uint32_t best_of = 0xffffffffu;              // lane b: rank chosen for expert 64w+b
            while (multi) {
                const int b = __ffsll((unsigned long long)multi) - 1;
                multi &= multi - 1;
                uint64_t cand = join64(__builtin_amdgcn_readlane(hl, b), __builtin_amdgcn_readlane(hh, b));
                const int cur = L + __popcll(forced & ((1ull << b) - 1ull)) + picked;
                for (int bit = load_bits - 1; bit >= 0; --bit) {     // keep the candidates with the smallest load
                    const uint64_t zero_here = __ballot(((cur >> bit) & 1) == 0) & cand;
                    if (zero_here) cand = zero_here;
                }
                const int best = __ffsll((unsigned long long)cand) - 1;   // lowest rank among them
                if (g == best) ++picked;
                if (g == b) best_of = best;
            }
            if (best_of != 0xffffffffu) s_rank[(w << 6) + g] = (int)best_of;
            L += __popcll(forced) + picked;
        }
    }
    __syncthreads();

    // y[i][g*] = 1 -> the lowest slot of expert i on rank g*.
#pragma unroll
    for (int j = 0; j < kMaxS / kThreads; ++j) {
        const int sl = tid + j * kThreads;
        const int e = se[j];
        if (sl < S && e >= 0 && s_active[e] && s_rank[e] == sl / spr) atomicMin(&s_slot[e], sl);
    }
    __syncthreads();
    for (int e = tid; e < N; e += kThreads) {
        int slot = s_slot[e];
        if (slot == kNoSlot) slot = -1;
        s_slot[e] = slot;
        a.expert_slot[(size_t)layer * N + e] = slot;
        if (slot >= 0) set_bit64(s_bm_lo, s_bm_hi, slot / spr, slot % spr);
    }
    __syncthreads();
    if (tid < G) {
        const uint64_t bm = join64(s_bm_lo[tid], s_bm_hi[tid]);
        a.rank_bitmap[(size_t)layer * G + tid] = bm;
        a.rank_active[(size_t)layer * G + tid] = __popcll(bm);
    }
    if (tid == 0) a.err_flag[layer] = s_err;

    // x from y: every pair of expert i goes to its activated replica.
    auto slot_of = [&](int id) { return (id >= 0 && id < N) ? s_slot[id] : -1; };
    int4* o = reinterpret_cast<int4*>(pair_slot);
#pragma unroll
    for (int c = 0; c < kIdCache; ++c) {
        const int i = tid + c * kThreads;
        if (i < n4) o[i] = make_int4(slot_of(idc[c].x), slot_of(idc[c].y), slot_of(idc[c].z), slot_of(idc[c].w));
    }
    for (int i = tid + kIdCache * kThreads; i < n4; i += kThreads) {
        const int4 q = v[i];
        o[i] = make_int4(slot_of(q.x), slot_of(q.y), slot_of(q.z), slot_of(q.w));
    }
    if (!a.vec4)
        for (int i = tid; i < n_pairs; i += kThreads) pair_slot[i] = slot_of(ids[i]);
    // "Route tokens" (Sec. 4.3) in the same launch: the token lists of one rank.  A pair's slot is looked up from
    // the table in LDS again (the ids come back from the cache), so nothing written above has to be re-read.
    if (a.list_rank >= 0) {                         // uniform
        const int lo = a.list_rank * spr;
        auto key_of = [&](int p) {
            const int id = ids[p];
            const int l = ((id >= 0 && id < N) ? s_slot[id] : -1) - lo;
            return (l >= 0 && l < spr) ? l : -1;
        };
        build_token_lists(key_of, nullptr, n_pairs, spr, s_list_hist, s_list_cnt, s_list_off, a.group_offsets,
                          a.perm_pair, a.pair_row, a.n_pairs);
    }
}

// ------------------------------------------------------------------------------------------ token-balanced
__global__ __launch_bounds__(kThreads) void token_balanced_kernel(RouteArgs a) {
    __shared__ int s_hist[kWaves * kMaxN];          // per-wave occurrence bases
    __shared__ int s_cnt[kMaxN];                    // T[i]
    __shared__ uint32_t s_host_lo[kMaxN], s_host_hi[kMaxN];
    __shared__ int s_base[kMaxN + 1];               // CSR of replicas per expert
    __shared__ int s_repl[kMaxS];                   // replica slots, ascending slot id within an expert
    __shared__ int s_s2e[kMaxS];
    __shared__ uint32_t s_bm_lo[kMaxG], s_bm_hi[kMaxG];
    __shared__ int s_wave_sum[kWaves];
    __shared__ int s_err;

    const int layer = blockIdx.x;
    const int N = a.N, G = a.G, spr = a.spr, S = G * spr;
    const int n_pairs = a.T * a.k;
    const int32_t* ids = a.ids + (size_t)layer * n_pairs;
    const int32_t* s2e = a.slot_to_expert + (size_t)layer * S;
    int32_t* pair_slot = a.pair_slot + (size_t)layer * n_pairs;
    const int tid = threadIdx.x;

    OrderedCounter oc;
    oc.init(n_pairs, N, s_hist, s_cnt);
    for (int e = tid; e < kMaxN; e += kThreads) { s_host_lo[e] = 0; s_host_hi[e] = 0; }
    if (tid < kMaxG) { s_bm_lo[tid] = 0; s_bm_hi[tid] = 0; }
    if (tid == 0) s_err = 0;
    for (int s = tid; s < S; s += kThreads) {
        const int e = s2e[s];
        s_s2e[s] = (e >= 0 && e < N) ? e : -1;
    }
    __syncthreads();

    build_host_masks(s2e, N, S, spr, s_host_lo, s_host_hi, &s_err);
    auto key_of = [&](int p) {
        const int id = ids[p];
        if (id < -1 || id >= N) { atomicOr(&s_err, METRO_FLAG_BAD_ID); return -1; }
        return id;
    };
    int keys[OrderedCounter::kCached];
    oc.load_keys(key_of, keys);
    oc.histogram(key_of, keys);
    __syncthreads();
    oc.prefix();                                     // s_cnt[e] = T[e]

    // Exclusive scan of replica counts r_e = popcount(host[e]) over experts -> s_base.
    {
        int r = 0;
        if (tid < N) r = __popcll(join64(s_host_lo[tid], s_host_hi[tid]));
        int incl = r;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int up = __shfl_up(incl, d);
            if (lane_id() >= d) incl += up;
        }
        if (lane_id() == kWave - 1) s_wave_sum[wave_id()] = incl;
        __syncthreads();
        int before = 0;
        for (int w = 0; w < wave_id(); ++w) before += s_wave_sum[w];
        if (tid < N) s_base[tid] = before + incl - r;
        if (tid == N - 1) s_base[N] = before + incl;
    }
    __syncthreads();

    // Replica lists: the lowest slot of an expert on each hosting rank, ranks ascending
    // (= ascending slot id).  A replica is activated iff its index is below T[e].
    for (int s = tid; s < S; s += kThreads) {
        const int e = s_s2e[s];
        if (e < 0) continue;
        const int g = s / spr;
        bool primary = true;
        for (int q = g * spr; q < s; ++q) primary = primary && s_s2e[q] != e;
        if (!primary) continue;
        const uint64_t host = join64(s_host_lo[e], s_host_hi[e]);
        const int j = __popcll(host & ((1ull << g) - 1ull));
        s_repl[s_base[e] + j] = s;
        if (j < s_cnt[e]) set_bit64(s_bm_lo, s_bm_hi, g, s - g * spr);
    }
    for (int e = tid; e < N; e += kThreads)
        if (s_cnt[e] > 0 && s_base[e + 1] == s_base[e]) atomicOr(&s_err, METRO_FLAG_NO_REPLICA);
    __syncthreads();

    // q-th pair of expert e -> replica q mod r_e.  The slots of the wave's register-cached chunks are kept for
    // the token lists (their items map to lanes the same way there).
    const int lo = a.list_rank * spr;
    auto local = [&](int slot) {
        const int l = slot - lo;
        return (a.list_rank >= 0 && l >= 0 && l < spr) ? l : -1;
    };
    int list_keys[OrderedCounter::kCached];
#pragma unroll
    for (int c = 0; c < OrderedCounter::kCached; ++c) list_keys[c] = -1;
    oc.number(
        [&](int p) {
            const int id = ids[p];
            return (id < 0 || id >= N) ? -1 : id;
        },
        keys, [&](int p, int e, int occ, auto cached) {
            int slot = -1;
            if (e >= 0) {
                const int r = s_base[e + 1] - s_base[e];
                if (r > 0) slot = s_repl[s_base[e] + occ % r];
            }
            pair_slot[p] = slot;
            constexpr int c = decltype(cached)::value;
            if constexpr (c >= 0) list_keys[c] = local(slot);
        });
    if (tid < G) {
        const uint64_t bm = join64(s_bm_lo[tid], s_bm_hi[tid]);
        a.rank_bitmap[(size_t)layer * G + tid] = bm;
        a.rank_active[(size_t)layer * G + tid] = __popcll(bm);
    }
    __syncthreads();
    if (tid == 0) a.err_flag[layer] = s_err;
    // "Route tokens" (Sec. 4.3) in the same launch.  The occurrence tables are free again and the token lists reuse
    // them.  Pairs beyond the register-cached chunks (batches of more than 8192 pairs) are read back from
    // pair_slot: the fence pushes this workgroup's stores past the CU's L1, the loads go around it.
    if (a.list_rank >= 0) {                         // uniform
        __threadfence();
        __syncthreads();
        auto key_of = [&](int p) {
            return local(__hip_atomic_load(pair_slot + p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        };
        build_token_lists(key_of, list_keys, n_pairs, spr, s_hist, s_cnt, s_base, a.group_offsets, a.perm_pair,
                          a.pair_row, a.n_pairs);
    }
}

int check_route_args(const void* ids, const void* s2e, int L, int T, int k, int N, int G, int spr,
                     const void* pair_slot, const void* rank_active, const void* rank_bitmap,
                     const void* err_flag) {
    if (!s2e || !rank_active || !rank_bitmap || !err_flag) return METRO_ERR_INVALID_ARG;
    if (L < 1 || T < 0 || k < 1 || N < 1 || G < 1 || spr < 1 || k > N) return METRO_ERR_INVALID_ARG;
    if ((!ids || !pair_slot) && T > 0) return METRO_ERR_INVALID_ARG;   // an empty batch has no id tensor
    if (N > kMaxN || G > kMaxG || spr > kMaxSpr || G * spr > kMaxS || (int64_t)T * k >= (1 << 24))
        return METRO_ERR_UNSUPPORTED;
    return METRO_OK;
}

RouteArgs pack(const int32_t* ids, const int32_t* s2e, int T, int k, int N, int G, int spr, int32_t* pair_slot,
               int32_t* expert_slot, int32_t* rank_active, uint64_t* rank_bitmap, int32_t* err_flag) {
    RouteArgs a;
    a.ids = ids;
    a.slot_to_expert = s2e;
    a.T = T; a.k = k; a.N = N; a.G = G; a.spr = spr;
    const bool aligned = (((uintptr_t)ids | (uintptr_t)pair_slot) & 15) == 0 && ((int64_t)T * k) % 4 == 0;
    a.vec4 = aligned ? 1 : 0;
    a.pair_slot = pair_slot;
    a.expert_slot = expert_slot;
    a.rank_active = rank_active;
    a.rank_bitmap = rank_bitmap;
    a.err_flag = err_flag;
    a.list_rank = -1;
    a.group_offsets = a.perm_pair = a.pair_row = a.n_pairs = nullptr;
    return a;
}

int add_lists(RouteArgs& a, int rank, int32_t* group_offsets, int32_t* perm_pair, int32_t* pair_row, int32_t* n_pairs) {
    if (!group_offsets || !n_pairs || rank < 0 || rank >= a.G) return METRO_ERR_INVALID_ARG;
    if ((!perm_pair || !pair_row) && a.T > 0) return METRO_ERR_INVALID_ARG;
    a.list_rank = rank;
    a.group_offsets = group_offsets;
    a.perm_pair = perm_pair;
    a.pair_row = pair_row;
    a.n_pairs = n_pairs;
    return METRO_OK;
}

}  // namespace
}  // namespace metro

extern "C" int metro_route(const int32_t* topk_ids, const int32_t* slot_to_expert, int L, int T, int k, int N,
                           int G, int spr, int32_t* pair_slot, int32_t* expert_slot, int32_t* rank_active,
                           uint64_t* rank_bitmap, int32_t* err_flag, void* stream) {
    using namespace metro;
    int rc = check_route_args(topk_ids, slot_to_expert, L, T, k, N, G, spr, pair_slot, rank_active, rank_bitmap,
                              err_flag);
    if (rc != METRO_OK) return rc;
    if (!expert_slot) return METRO_ERR_INVALID_ARG;
    RouteArgs a = pack(topk_ids, slot_to_expert, T, k, N, G, spr, pair_slot, expert_slot, rank_active,
                       rank_bitmap, err_flag);
    hipLaunchKernelGGL(metro_route_kernel, dim3(L), dim3(kThreads), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? METRO_OK : METRO_ERR_HIP;
}

extern "C" int metro_route_token_balanced(const int32_t* topk_ids, const int32_t* slot_to_expert, int L, int T,
                                          int k, int N, int G, int spr, int32_t* pair_slot,
                                          int32_t* rank_active, uint64_t* rank_bitmap, int32_t* err_flag,
                                          void* stream) {
    using namespace metro;
    int rc = check_route_args(topk_ids, slot_to_expert, L, T, k, N, G, spr, pair_slot, rank_active, rank_bitmap,
                              err_flag);
    if (rc != METRO_OK) return rc;
    RouteArgs a = pack(topk_ids, slot_to_expert, T, k, N, G, spr, pair_slot, nullptr, rank_active, rank_bitmap,
                       err_flag);
    hipLaunchKernelGGL(token_balanced_kernel, dim3(L), dim3(kThreads), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? METRO_OK : METRO_ERR_HIP;
}

extern "C" int metro_route_permute(const int32_t* topk_ids, const int32_t* slot_to_expert, int T, int k, int N, int G,
                                   int spr, int rank, int32_t* pair_slot, int32_t* expert_slot, int32_t* rank_active,
                                   uint64_t* rank_bitmap, int32_t* err_flag, int32_t* group_offsets,
                                   int32_t* perm_pair, int32_t* pair_row, int32_t* n_pairs, void* stream) {
    using namespace metro;
    int rc = check_route_args(topk_ids, slot_to_expert, 1, T, k, N, G, spr, pair_slot, rank_active, rank_bitmap,
                              err_flag);
    if (rc != METRO_OK) return rc;
    if (!expert_slot) return METRO_ERR_INVALID_ARG;
    RouteArgs a = pack(topk_ids, slot_to_expert, T, k, N, G, spr, pair_slot, expert_slot, rank_active,
                       rank_bitmap, err_flag);
    rc = add_lists(a, rank, group_offsets, perm_pair, pair_row, n_pairs);
    if (rc != METRO_OK) return rc;
    hipLaunchKernelGGL(metro_route_kernel, dim3(1), dim3(kThreads), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? METRO_OK : METRO_ERR_HIP;
}

extern "C" int metro_route_token_balanced_permute(const int32_t* topk_ids, const int32_t* slot_to_expert, int T, int k,
                                                  int N, int G, int spr, int rank, int32_t* pair_slot,
                                                  int32_t* rank_active, uint64_t* rank_bitmap, int32_t* err_flag,
                                                  int32_t* group_offsets, int32_t* perm_pair, int32_t* pair_row,
                                                  int32_t* n_pairs, void* stream) {
    using namespace metro;
    int rc = check_route_args(topk_ids, slot_to_expert, 1, T, k, N, G, spr, pair_slot, rank_active, rank_bitmap,
                              err_flag);
    if (rc != METRO_OK) return rc;
    RouteArgs a = pack(topk_ids, slot_to_expert, T, k, N, G, spr, pair_slot, nullptr, rank_active, rank_bitmap,
                       err_flag);
    rc = add_lists(a, rank, group_offsets, perm_pair, pair_row, n_pairs);
    if (rc != METRO_OK) return rc;
    hipLaunchKernelGGL(token_balanced_kernel, dim3(1), dim3(kThreads), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? METRO_OK : METRO_ERR_HIP;
}
