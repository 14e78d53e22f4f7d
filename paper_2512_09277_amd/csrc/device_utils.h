// Wavefront-level helpers shared by the gfx950 kernels (64-wide waves).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace metro {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }
__device__ __forceinline__ uint64_t lanes_below() { return (1ull << lane_id()) - 1ull; }

// For the lanes with `valid`, the number of lower lanes holding the same key; `total` receives the
// number of lanes holding it.  Keys are < 2^bits.  One ballot per key bit: the lanes that agree with
// mine on every bit are the lanes with my key (no loop over the distinct keys of the wave).
__device__ __forceinline__ int wave_rank_by_key(int key, bool valid, int bits, int& total) {
    uint64_t same = __ballot(valid);
    for (int b = 0; b < bits; ++b) {
        const bool mine = (key >> b) & 1;
        const uint64_t set = __ballot(mine);
        same &= mine ? set : ~set;
    }
    total = __popcll(same);
    return __popcll(same & lanes_below());
}

// Stable occurrence numbering of n items by key, in item order, by one workgroup.
//   hist: LDS, [n_waves][n_keys] ints.  tot: LDS, [n_keys] ints.
// After pass 1 + prefix, hist[w][key] = items with that key owned by lower waves, tot[key] = all.
// Each wave owns a contiguous run of 64-item chunks, so item order = (wave, chunk, lane).
struct OrderedCounter {
    int n, n_keys, key_bits, chunks_per_wave;
    int* hist;
    int* tot;

    __device__ __forceinline__ void init(int n_, int n_keys_, int* hist_, int* tot_) {
        n = n_;
        n_keys = n_keys_;
        key_bits = 32 - __clz(max(n_keys_ - 1, 1));              // keys are < 2^key_bits
        hist = hist_;
        tot = tot_;
        const int n_waves = blockDim.x >> 6;
        const int chunks = (n + kWave - 1) / kWave;
        chunks_per_wave = (chunks + n_waves - 1) / n_waves;
        for (int i = threadIdx.x; i < n_waves * n_keys; i += blockDim.x) hist[i] = 0;
    }

    static constexpr int kCached = 8;   // chunks per wave whose keys stay in registers between the passes

    // Keys of this wave's first kCached chunks, fetched with independent loads (one round trip for
    // all of them).  key_of(item) -> key in [0, n_keys) or -1 to leave the item out.
    template <typename KeyFn>
    __device__ __forceinline__ void load_keys(KeyFn key_of, int (&keys)[kCached]) const {
        const int first = wave_id() * chunks_per_wave;
#pragma unroll
        for (int c = 0; c < kCached; ++c) {
            const int item = (first + c) * kWave + lane_id();
            keys[c] = (c < chunks_per_wave && item < n) ? key_of(item) : -1;
        }
    }

    // Per-wave histogram.  Call between barriers.
    template <typename KeyFn>
    __device__ __forceinline__ void histogram(KeyFn key_of, const int (&keys)[kCached]) {
        int* mine = hist + wave_id() * n_keys;
        const int first = wave_id() * chunks_per_wave;
#pragma unroll
        for (int c = 0; c < kCached; ++c)
            if (keys[c] >= 0) atomicAdd(&mine[keys[c]], 1);
        for (int c = first + kCached; c < first + chunks_per_wave; ++c) {
            const int item = c * kWave + lane_id();
            if (item < n) {
                const int key = key_of(item);
                if (key >= 0) atomicAdd(&mine[key], 1);
            }
        }
    }

    // Turns per-wave counts into per-wave bases and totals.  Call between barriers.
    __device__ __forceinline__ void prefix() {
        const int n_waves = blockDim.x >> 6;
        for (int key = threadIdx.x; key < n_keys; key += blockDim.x) {
            int running = 0;
            for (int w = 0; w < n_waves; ++w) {
                const int c = hist[w * n_keys + key];
                hist[w * n_keys + key] = running;
                running += c;
            }
            tot[key] = running;
        }
    }

    // emit(item, key, occ, cached) for every item: occ = number of earlier items with the same key
    // (key = -1: occ undefined); cached = index of the item's chunk among the wave's register-cached chunks
    // (a compile-time constant there), or -1.  Call between barriers.
    template <typename KeyFn, typename EmitFn>
    __device__ __forceinline__ void number(KeyFn key_of, const int (&keys)[kCached], EmitFn emit) {
        int* mine = hist + wave_id() * n_keys;
        const int first = wave_id() * chunks_per_wave;
        auto one_chunk = [&](int c, int key, bool in_range, auto cached) {
            const bool valid = key >= 0;
            int total;
            const int rank = wave_rank_by_key(key, valid, key_bits, total);
            int occ = 0;
            if (valid) occ = mine[key] + rank;
            // the wave executes in lockstep: every read of mine[] above precedes the update below
            if (valid && rank == total - 1) mine[key] = occ + 1;
            if (in_range) emit(c * kWave + lane_id(), key, occ, cached);
        };
        number_cached(one_chunk, keys, first, std::make_integer_sequence<int, kCached>{});
        for (int c = first + kCached; c < first + chunks_per_wave; ++c) {
            const int item = c * kWave + lane_id();
            const bool in_range = item < n;
            one_chunk(c, in_range ? key_of(item) : -1, in_range, std::integral_constant<int, -1>{});
        }
    }

    template <typename ChunkFn, int... Cs>
    __device__ __forceinline__ void number_cached(ChunkFn& one_chunk, const int (&keys)[kCached], int first,
                                                  std::integer_sequence<int, Cs...>) {
        // chunk index Cs is a compile-time constant, so a caller may keep per-chunk values in registers
        ((Cs < chunks_per_wave                                        // uniform per wave
              ? one_chunk(first + Cs, keys[Cs], (first + Cs) * kWave + lane_id() < n, std::integral_constant<int, Cs>{})
              : (void)0),
         ...);
    }
};

// Per-replica token lists of one rank (a stable counting sort of the pairs by local slot), by one workgroup of
// 1024 threads; shared by moe_permute and the routing calls that emit the lists themselves.
//   key_of(p): local slot of pair p on the rank, or -1.  preset: the keys of the wave's register-cached chunks
//   if the caller already holds them (else nullptr: they are fetched with key_of).
//   s_hist [16 * 64], s_cnt [64], s_off [65]: LDS.
constexpr int kListThreads = 1024;
constexpr int kListMaxSpr = 64;
template <typename KeyFn>
__device__ __forceinline__ void build_token_lists(KeyFn key_of, const int* preset, int n, int spr, int* s_hist,
                                                  int* s_cnt, int* s_off, int32_t* __restrict__ group_offsets,
                                                  int32_t* __restrict__ perm_pair, int32_t* __restrict__ pair_row,
                                                  int32_t* __restrict__ n_pairs) {
    OrderedCounter oc;
    oc.init(n, spr, s_hist, s_cnt);
    int keys[OrderedCounter::kCached];
    if (preset) {
#pragma unroll
        for (int c = 0; c < OrderedCounter::kCached; ++c) keys[c] = preset[c];
    } else {
        oc.load_keys(key_of, keys);
    }
    __syncthreads();
    oc.histogram(key_of, keys);
    __syncthreads();
    oc.prefix();
    __syncthreads();
    if (threadIdx.x < kWave) {                          // exclusive scan of the slot counts
        const int c = (int)threadIdx.x < spr ? s_cnt[threadIdx.x] : 0;
        int incl = c;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int up = __shfl_up(incl, d);
            if (lane_id() >= d) incl += up;
        }
        if ((int)threadIdx.x < spr) {
            s_off[threadIdx.x] = incl - c;
            group_offsets[threadIdx.x] = incl - c;
        }
        if ((int)threadIdx.x == spr - 1) {
            s_off[spr] = incl;
            group_offsets[spr] = incl;
            *n_pairs = incl;
        }
    }
    __syncthreads();
    oc.number(key_of, keys, [&](int p, int l, int occ, auto) {
        int row = -1;
        if (l >= 0) {
            row = s_off[l] + occ;
            perm_pair[row] = p;
        }
        pair_row[p] = row;
    });
}

}  // namespace metro
