// moe_gate_topk for gfx950: router logits + top-k + gating weights on the full (gathered) token set,
// the step that produces the global top-k ids the routing solve consumes (Sec. 4.3 of arxiv
// 2512.09277: every rank runs top-k over all tokens).
//
//   logit[t][e] = x[t] . w_gate[e]        ids[t] = k largest logits (descending, ties to the lower id)
//   w[t][j]     = softmax over the k selected logits          cnt[e] = pairs that selected expert e
//
// The logits are a small dense contraction ([T,H] x [H,N], 3.8 GFLOP at T=1024, H=7168, N=256) whose
// operands total 18 MB: neither the matrix cores nor HBM is the limit, launch latency and the number
// of busy CUs are.  Launches:
//   1. gate_logits_mfma_kernel: 64 tokens x 64 experts x one K chunk per workgroup (split-K so that
//      ~512 workgroups exist at any batch size); both operands go straight from global memory into
//      the MFMA operand layout; fp32 partial sums land in the workspace, part[chunk][t][e];
//   2. gate_topk_kernel: one wave per token sums the chunks in a fixed order (deterministic), picks the
//      top-k by k rounds of a wave-wide arg-max over (logit, -id) and forms the softmax weights;
//   3. (only when the caller wants expert_count) gate_count_kernel: pairs per expert, one workgroup.
// Shapes the MFMA kernel does not take (fp32, N not a multiple of 64, H not a multiple of 32) use a
// plain one-wave-per-logit kernel in fp32.
#include <hip/hip_runtime.h>
#include <float.h>
#include <stdint.h>

#include <type_traits>

#include "device_utils.h"
#include "host_utils.h"
#include "metro.h"

namespace metro {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kMaxN = 512;
constexpr int kTokTile = 16;              // tokens of one matrix-instruction sub-tile
constexpr int kMinChunkSteps = 2;           // K steps of 32 a wave gets at least

struct GateArgs {
    const void* x;
    const void* w_gate;
    float* part;              // [n_chunks][T][N]
    int T, H, N, ldw;
    int steps_per_chunk;      // K steps of 32 per chunk
};

// One workgroup: 16*MT tokens x 64 experts x one K chunk; its four waves split the chunk's K steps and
// meet through LDS, so one partial tile leaves the workgroup.  (Splitting K over workgroups only would
// need four times the chunks for the same number of waves, and the partial sums -- written here, read
// by the top-k kernel -- would outweigh the operands.)
// Lane (r16, q) supplies the 8 elements k = kk + q*8 .. +8 of expert row r16 of a block (A operand) and of
// token row r16 of a sub-tile (B operand); D[i][j]: i = expert 4*q + v of the block, j = token r16.
constexpr int kExpTile = 64, kNB = kExpTile / 16;

template <int MT>
__global__ __launch_bounds__(kThreads, 2) void gate_logits_mfma_kernel(GateArgs a) {
    __shared__ floatx4 xch[3][kNB * MT][kWave];                   // sums of waves 1..3
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int r16 = lane & 15, q = lane >> 4;
    // K chunk fastest in launch order: workgroup i runs on XCD i mod 8, so with a multiple of 8 chunks
    // every XCD (own L2) streams its own K range of x and w_gate instead of all eight fetching everything.
    const int chunk = blockIdx.x, t0 = blockIdx.y * (16 * MT), e0 = blockIdx.z * kExpTile;
    const int n_steps = a.H / 32;
    const int c_begin = chunk * a.steps_per_chunk, c_end = min(c_begin + a.steps_per_chunk, n_steps);
    const int per_wave = (c_end - c_begin + 3) / 4;
    const int s_begin = min(c_begin + wv * per_wave, c_end), s_end = min(s_begin + per_wave, c_end);
    const char* xp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int tok = min(t0 + mt * 16 + r16, a.T - 1);         // rows past the batch repeat the last token
        xp[mt] = reinterpret_cast<const char*>(a.x) + ((size_t)tok * a.H + q * 8) * 2;
    }
    const char* wp = reinterpret_cast<const char*>(a.w_gate) + ((size_t)(e0 + r16) * a.ldw + q * 8) * 2;
    const size_t blk = (size_t)16 * a.ldw * 2;                    // bytes between 16-row blocks

    floatx4 acc[kNB][MT];
#pragma unroll
    for (int b = 0; b < kNB; ++b)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[b][mt] = floatx4{0.f, 0.f, 0.f, 0.f};
    // U steps at a time: all their loads are issued before the first matrix instruction (the scheduling
    // barrier keeps the compiler from sinking each load next to its use, which would leave one or two
    // loads in flight per wave).
    auto steps = [&](auto U, int s) {
        constexpr int n = decltype(U)::value;
        bf16x8 xb[n][MT], wa[n][kNB];
#pragma unroll
        for (int u = 0; u < n; ++u) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xb[u][mt] = *reinterpret_cast<const bf16x8*>(xp[mt] + (size_t)(s + u) * 64);
#pragma unroll
            for (int b = 0; b < kNB; ++b) wa[u][b] = *reinterpret_cast<const bf16x8*>(wp + b * blk + (size_t)(s + u) * 64);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < n; ++u)
#pragma unroll
            for (int b = 0; b < kNB; ++b)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[b][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[u][b], xb[u][mt], acc[b][mt], 0, 0, 0);
    };
    int s = s_begin;
    for (; s + 3 <= s_end; s += 3) steps(std::integral_constant<int, 3>{}, s);
    for (; s < s_end; ++s) steps(std::integral_constant<int, 1>{}, s);

    if (wv > 0) {
#pragma unroll
        for (int b = 0; b < kNB; ++b)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xch[wv - 1][b * MT + mt][lane] = acc[b][mt];
    }
    __syncthreads();
    if (wv == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int t = t0 + mt * 16 + r16;
            float* out = a.part + ((size_t)chunk * a.T + min(t, a.T - 1)) * a.N + e0 + q * 4;
#pragma unroll
            for (int b = 0; b < kNB; ++b) {
                floatx4 sum = acc[b][mt];
#pragma unroll
                for (int o = 0; o < 3; ++o) sum += xch[o][b * MT + mt][lane];     // waves in a fixed order
                if (t < a.T) *reinterpret_cast<floatx4*>(out + b * 16) = sum;
            }
        }
    }
}

// Large batches: one workgroup = 128 tokens x 128 experts x one K chunk, both operands staged through
// LDS.  Global loads are fully coalesced (8 lanes read the 128 contiguous bytes a row contributes to a
// K step of 64: a wave instruction covers 8 whole cache lines instead of 16 half lines), each operand
// byte enters the CU once per workgroup, and the 2 x 2 waves (64 x 64 each, 16 accumulator tiles) read
// their fragments from LDS in operand layout.  Double-buffered: the loads of step s + 1 are in flight
// while step s is multiplied.
constexpr int kBigTile = 128, kBigBK = 64;
constexpr int kBigRow = kBigBK * 2 + 16;                         // LDS bytes per staged row (+16 spreads the banks)
constexpr int kBigBuf = 2 * kBigTile * kBigRow;                  // x tile + w tile of one step
constexpr int kBigLds = 2 * kBigBuf;

__global__ __launch_bounds__(kThreads, 2) void gate_logits_lds_kernel(GateArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r16 = lane & 15, q = lane >> 4;
    const int chunk = blockIdx.x, t0 = blockIdx.y * kBigTile, e0 = blockIdx.z * kBigTile;
    const int n_steps = a.H / kBigBK;                             // the host takes this path only if H % 64 == 0
    const int s_begin = chunk * a.steps_per_chunk, s_end = min(s_begin + a.steps_per_chunk, n_steps);
    const int last = s_end - 1;

    // staging: thread (row, piece) copies 16 bytes of rows row, row + 32, row + 64, row + 96 of both tiles
    const int srow = tid >> 3, piece = tid & 7;
    const char* xg[4];
    const char* wg[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int tok = min(t0 + p * 32 + srow, a.T - 1);         // rows past the batch repeat the last token
        xg[p] = reinterpret_cast<const char*>(a.x) + ((size_t)tok * a.H) * 2 + piece * 16;
        wg[p] = reinterpret_cast<const char*>(a.w_gate) + ((size_t)(e0 + p * 32 + srow) * a.ldw) * 2 + piece * 16;
    }
    const int st_off = srow * kBigRow + piece * 16;
    // Three register sets: the loads of steps s + 1 .. s + 3 are in flight while step s is multiplied
    // (one workgroup per CU at most at these sizes, so the prefetch distance is all the latency hiding
    // there is).  Loads are unconditional -- past the chunk they re-read its last step -- so that the
    // compiler counts outstanding loads exactly.
    u32x4 xr[3][4], wr[3][4];
    auto load = [&](int set, int s) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            xr[set][p] = *reinterpret_cast<const u32x4*>(xg[p] + (size_t)s * (kBigBK * 2));
            wr[set][p] = *reinterpret_cast<const u32x4*>(wg[p] + (size_t)s * (kBigBK * 2));
        }
    };
    auto park = [&](int set, int buf) {
        char* base = lds + buf * kBigBuf + st_off;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            *reinterpret_cast<u32x4*>(base + p * 32 * kBigRow) = xr[set][p];
            *reinterpret_cast<u32x4*>(base + kBigTile * kBigRow + p * 32 * kBigRow) = wr[set][p];
        }
    };

    const int ty = wv >> 1, tx = wv & 1;                          // wave: tokens [64 ty, +64), experts [64 tx, +64)
    const int rd = r16 * kBigRow + q * 16;
    floatx4 acc[4][4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) acc[b][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

    // step U of a period of 6 (register set U % 3, LDS buffer U % 2 known at compile time)
    auto step = [&](auto Uc, int s) {
        constexpr int U = decltype(Uc)::value;
        load(U % 3, min(s + 3, last));                            // set U % 3 was parked one step ago
        const char* xt = lds + (U % 2) * kBigBuf + ty * 64 * kBigRow + rd;
        const char* wt = lds + (U % 2) * kBigBuf + kBigTile * kBigRow + tx * 64 * kBigRow + rd;
#pragma unroll
        for (int j = 0; j < kBigBK / 32; ++j) {
            bf16x8 xb[4], wa[4];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) xb[mt] = *reinterpret_cast<const bf16x8*>(xt + mt * 16 * kBigRow + j * 64);
#pragma unroll
            for (int b = 0; b < 4; ++b) wa[b] = *reinterpret_cast<const bf16x8*>(wt + b * 16 * kBigRow + j * 64);
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
                    acc[b][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[b], xb[mt], acc[b][mt], 0, 0, 0);
        }
        park((U + 1) % 3, (U + 1) % 2);                           // step s + 1, loaded two steps ago
        __syncthreads();
    };
    load(0, min(s_begin, last));
    load(1, min(s_begin + 1, last));
    load(2, min(s_begin + 2, last));
    park(0, 0);
    __syncthreads();
    int s = s_begin;
    for (; s + 6 <= s_end; s += 6) {
        step(std::integral_constant<int, 0>{}, s);
        step(std::integral_constant<int, 1>{}, s + 1);
        step(std::integral_constant<int, 2>{}, s + 2);
        step(std::integral_constant<int, 3>{}, s + 3);
        step(std::integral_constant<int, 4>{}, s + 4);
        step(std::integral_constant<int, 5>{}, s + 5);
    }
    // tail: at most five steps; once one is past the end nothing after it is tested
    (void)((s + 0 < s_end && (step(std::integral_constant<int, 0>{}, s + 0), true)) &&
           (s + 1 < s_end && (step(std::integral_constant<int, 1>{}, s + 1), true)) &&
           (s + 2 < s_end && (step(std::integral_constant<int, 2>{}, s + 2), true)) &&
           (s + 3 < s_end && (step(std::integral_constant<int, 3>{}, s + 3), true)) &&
           (s + 4 < s_end && (step(std::integral_constant<int, 4>{}, s + 4), true)));
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        const int t = t0 + ty * 64 + mt * 16 + r16;
        if (t < a.T) {
            float* out = a.part + ((size_t)chunk * a.T + t) * a.N + e0 + tx * 64 + q * 4;
#pragma unroll
            for (int b = 0; b < 4; ++b) *reinterpret_cast<floatx4*>(out + b * 16) = acc[b][mt];
        }
    }
}

template <typename T>
__device__ __forceinline__ float elem_f32(const void* p, size_t i);
template <>
__device__ __forceinline__ float elem_f32<float>(const void* p, size_t i) { return ((const float*)p)[i]; }
template <>
__device__ __forceinline__ float elem_f32<__bf16>(const void* p, size_t i) { return (float)((const __bf16*)p)[i]; }

// Any shape, fp32 arithmetic: one wave per logit, a single chunk.
template <typename T>
__global__ __launch_bounds__(kThreads) void gate_logits_general_kernel(GateArgs a) {
    const int t = blockIdx.x;
    const int e = blockIdx.y * (kThreads / kWave) + wave_id();
    if (e >= a.N) return;
    float acc = 0.f;
    for (int h = lane_id(); h < a.H; h += kWave)
        acc = fmaf(elem_f32<T>(a.x, (size_t)t * a.H + h), elem_f32<T>(a.w_gate, (size_t)e * a.ldw + h), acc);
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) acc += __shfl_xor(acc, d);
    if (lane_id() == 0) a.part[(size_t)t * a.N + e] = acc;
}

struct Cand {
    float v;
    int id;
};
__device__ __forceinline__ bool better(const Cand& a, const Cand& b) { return a.v > b.v || (a.v == b.v && a.id < b.id); }

// One wave per token.  Lane l holds the logits of experts l, l + 64, ... (kPerLane = ceil(N / 64) of them).
// Tokens at or past *n_valid (a padded batch) get ids -1 and weights 0.
template <int kPerLane>
__global__ __launch_bounds__(kThreads) void gate_topk_kernel(const float* __restrict__ part, int n_chunks, int T, int N,
                                                              int k, const int32_t* __restrict__ n_valid,
                                                              int32_t* __restrict__ ids, float* __restrict__ w) {
    const int t = blockIdx.x * (kThreads / kWave) + wave_id();
    if (t >= T) return;                                          // uniform per wave
    const int l = lane_id();
    if (n_valid && t >= min(max(*n_valid, 0), T)) {              // padded token (uniform per wave)
        if (l < k) {
            ids[(size_t)t * k + l] = -1;
            w[(size_t)t * k + l] = 0.f;
        }
        return;
    }
    // Chunk sums in ascending chunk order (fixed, so the result is deterministic); the loads of a batch
    // of chunks x all of the lane's experts are issued together, only the additions are sequential.
    float v[kPerLane];
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) v[j] = 0.f;
    const float* row = part + (size_t)t * N + l;
    const size_t chunk_stride = (size_t)T * N;
    constexpr int kBatch = kPerLane <= 4 ? 8 : 4;
    for (int c0 = 0; c0 < n_chunks; c0 += kBatch) {
        float p[kBatch][kPerLane];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int c = min(c0 + u, n_chunks - 1);             // past the end: re-read, not added
#pragma unroll
            for (int j = 0; j < kPerLane; ++j)
                p[u][j] = (j * kWave + l < N) ? row[c * chunk_stride + j * kWave] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
            if (c0 + u < n_chunks) {
#pragma unroll
                for (int j = 0; j < kPerLane; ++j) v[j] += p[u][j];
            }
    }
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) {
        if (v[j] != v[j]) v[j] = -FLT_MAX;                       // NaN sorts below every number
        if (j * kWave + l >= N) v[j] = -INFINITY;                // experts past N never win
    }
    uint32_t taken = 0;                                          // bit j: v[j] already selected
#pragma unroll
    for (int j = 0; j < kPerLane; ++j)
        if (j * kWave + l >= N) taken |= 1u << j;
    float my_v = 0.f;
    int my_id = 0;
    for (int r = 0; r < k; ++r) {
        Cand best{-INFINITY, 0x7fffffff};
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            const Cand c{v[j], j * kWave + l};
            if (!((taken >> j) & 1u) && better(c, best)) best = c;
        }
#pragma unroll
        for (int d = kWave / 2; d > 0; d >>= 1) {
            const Cand o{__shfl_xor(best.v, d), __shfl_xor(best.id, d)};
            if (better(o, best)) best = o;
        }
        if ((best.id & (kWave - 1)) == l) taken |= 1u << (best.id >> 6);   // k <= N: a real expert
        if (l == r) {
            my_v = best.v;
            my_id = best.id;
        }
    }
    // lanes 0..k-1 hold the selection in descending order; softmax over it
    const float top = __shfl(my_v, 0);
    const float ex = l < k ? expf(my_v - top) : 0.f;
    float sum = ex;
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) sum += __shfl_xor(sum, d);
    if (l < k) {
        ids[(size_t)t * k + l] = my_id;
        w[(size_t)t * k + l] = ex / sum;
    }
}

// T[i] of Sec. 4.1: pairs per expert, one workgroup, LDS histogram over the ids just written (padded pairs,
// id -1, count nothing).  A launch of its own because every way of folding it into the top-k kernel measured
// slower at T = 1024: device-scope atomics from every token's wave onto the same few cache lines serialise
// across the eight L2s (~10 us, more than the rest of the top-k kernel), and per-workgroup histograms added up
// by the last workgroup to finish need a device-scope fence in every workgroup, which invalidates that XCD's
// L2 under the workgroups still reading their partial sums (top-k kernel 10.7 -> 33.8 us).
constexpr int kCountThreads = 1024;
__global__ __launch_bounds__(kCountThreads) void gate_count_kernel(const int32_t* __restrict__ ids, int n_pairs, int N,
                                                                   int32_t* __restrict__ cnt) {
    __shared__ int hist[kMaxN];
    for (int e = threadIdx.x; e < N; e += kCountThreads) hist[e] = 0;
    __syncthreads();
    for (int p = threadIdx.x; p < n_pairs; p += kCountThreads) {
        const int e = ids[p];
        if (e >= 0 && e < N) atomicAdd(&hist[e], 1);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < N; e += kCountThreads) cnt[e] = hist[e];
}

inline bool gate_mfma_shape(int H, int N, int dtype) {
    return dtype == METRO_DTYPE_BF16 && H % 32 == 0 && N % kExpTile == 0 && N <= kMaxN;
}

// The LDS-staged kernel takes batches of at least 1024 tokens when N % 128 == 0 and H % 64 == 0 (measured
// against the direct kernel at N = 256, H = 7168: 17.0 vs 18.7 us at T = 1024, 28 vs 56 us at T = 4096;
// below that the direct kernel's smaller workgroups win).
inline bool gate_big(int T, int H, int N) { return T >= 1024 && N % kBigTile == 0 && H % kBigBK == 0; }

// Tokens per workgroup: 64 (four sub-tiles) unless the batch is a single sub-tile.
inline int gate_tok_tile(int T) { return T > kTokTile ? 4 * kTokTile : kTokTile; }

// K chunks: enough workgroups for two per CU (~512), each chunk at least kMinChunkSteps steps per wave.
inline int gate_steps_per_chunk(int T, int H, int N) {
    if (gate_big(T, H, N)) {                    // steps of 64; ~8 chunks (one K range per XCD), >= 4 steps each
        const int n_steps = H / kBigBK;
        const int tiles = ((T + kBigTile - 1) / kBigTile) * (N / kBigTile);
        const int want = tiles * 8 < 256 ? 16 : 8;               // at least one workgroup per CU
        int chunks = n_steps / 4 >= want ? want : n_steps / 4 >= 8 ? 8 : n_steps / 4 > 0 ? n_steps / 4 : 1;
        return (n_steps + chunks - 1) / chunks;
    }
    const int n_steps = H / 32, tile = gate_tok_tile(T);
    const int tiles = ((T + tile - 1) / tile) * (N / kExpTile);
    int chunks = (512 + tiles - 1) / tiles;
    const int max_chunks = n_steps / (4 * kMinChunkSteps) > 0 ? n_steps / (4 * kMinChunkSteps) : 1;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks >= 8) chunks = chunks / 8 * 8;                      // one K range (or two, ...) per XCD
    if (chunks < 1) chunks = 1;
    return (n_steps + chunks - 1) / chunks;
}
inline int gate_chunks(int T, int H, int N, int dtype) {
    if (!gate_mfma_shape(H, N, dtype)) return 1;
    const int spc = gate_steps_per_chunk(T, H, N);
    const int n_steps = gate_big(T, H, N) ? H / kBigBK : H / 32;
    return (n_steps + spc - 1) / spc;
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace
}  // namespace metro

extern "C" size_t moe_gate_topk_workspace_bytes(int T, int H, int N, int dtype) {
    using namespace metro;
    if (T < 0 || H < 1 || N < 1) return 0;
    if (T == 0) return 256;                                       // an empty batch has no partial sums
    return align256((size_t)gate_chunks(T, H, N, dtype) * T * N * sizeof(float)) + 256;
}

extern "C" int moe_gate_topk(const void* x, const void* w_gate, int ldw, int T, int H, int N, int k, int dtype,
                             const int32_t* n_valid, int32_t* topk_ids, float* topk_w, int32_t* expert_count,
                             void* ws, size_t ws_bytes, void* stream) {
    using namespace metro;
    if (T < 0 || H < 1 || N < 1 || k < 1 || k > N) return METRO_ERR_INVALID_ARG;
    if (dtype != METRO_DTYPE_BF16 && dtype != METRO_DTYPE_F32) return METRO_ERR_UNSUPPORTED;
    if (N > kMaxN || k > kWave || (int64_t)T * k >= (1 << 24)) return METRO_ERR_UNSUPPORTED;
    if (ldw < H) return METRO_ERR_INVALID_ARG;
    if (T == 0) {                                                 // no token: every expert counts zero pairs
        if (expert_count) {
            hipLaunchKernelGGL(gate_count_kernel, dim3(1), dim3(kCountThreads), 0, (hipStream_t)stream,
                               (const int32_t*)nullptr, 0, N, expert_count);
            if (hipGetLastError() != hipSuccess) return METRO_ERR_HIP;
        }
        return METRO_OK;
    }
    if (!x || !w_gate || !topk_ids || !topk_w || !ws) return METRO_ERR_INVALID_ARG;
    if (((uintptr_t)ws & 255) != 0) return METRO_ERR_INVALID_ARG;
    if (ws_bytes < moe_gate_topk_workspace_bytes(T, H, N, dtype)) return METRO_ERR_WORKSPACE;
    const bool mfma = gate_mfma_shape(H, N, dtype) && ldw % 8 == 0 &&
                      (((uintptr_t)x | (uintptr_t)w_gate) & 15) == 0;
    hipStream_t st = (hipStream_t)stream;
    GateArgs a;
    a.x = x;
    a.w_gate = w_gate;
    a.part = (float*)ws;
    a.T = T; a.H = H; a.N = N; a.ldw = ldw;
    int n_chunks = 1;
    if (mfma) {
        a.steps_per_chunk = gate_steps_per_chunk(T, H, N);
        n_chunks = gate_chunks(T, H, N, dtype);
        if (gate_big(T, H, N)) {
            static PerDeviceOnce lds_ok;                          // opt in to > 64 KB of dynamic LDS, once per device
            if (lds_ok.run([] {
                    return hipFuncSetAttribute((const void*)gate_logits_lds_kernel,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, kBigLds);
                }) != METRO_OK)
                return METRO_ERR_HIP;
            const dim3 grid(n_chunks, (T + kBigTile - 1) / kBigTile, N / kBigTile);
            hipLaunchKernelGGL(gate_logits_lds_kernel, grid, dim3(kThreads), kBigLds, st, a);
        } else {
        const int tile = gate_tok_tile(T);
        const dim3 grid(n_chunks, (T + tile - 1) / tile, N / kExpTile);
        if (tile == kTokTile)
            hipLaunchKernelGGL(gate_logits_mfma_kernel<1>, grid, dim3(kThreads), 0, st, a);
        else
            hipLaunchKernelGGL(gate_logits_mfma_kernel<4>, grid, dim3(kThreads), 0, st, a);
        }
    }
    if (!mfma) {
        a.steps_per_chunk = 0;
        n_chunks = 1;
        const dim3 grid(T, (N + kThreads / kWave - 1) / (kThreads / kWave));
        if (dtype == METRO_DTYPE_F32)
            hipLaunchKernelGGL(gate_logits_general_kernel<float>, grid, dim3(kThreads), 0, st, a);
        else
            hipLaunchKernelGGL(gate_logits_general_kernel<__bf16>, grid, dim3(kThreads), 0, st, a);
    }
    if (hipGetLastError() != hipSuccess) return METRO_ERR_HIP;
    const int per = kThreads / kWave;
    const dim3 tgrid((T + per - 1) / per);
    const float* part = (const float*)ws;
    auto topk = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, tgrid, dim3(kThreads), 0, st, part, n_chunks, T, N, k, n_valid, topk_ids, topk_w);
    };
    if (N <= 64) topk(gate_topk_kernel<1>);
    else if (N <= 128) topk(gate_topk_kernel<2>);
    else if (N <= 256) topk(gate_topk_kernel<4>);
    else topk(gate_topk_kernel<8>);
    if (expert_count)
        hipLaunchKernelGGL(gate_count_kernel, dim3(1), dim3(kCountThreads), 0, st, (const int32_t*)topk_ids, T * k, N,
                           expert_count);
    return hipGetLastError() == hipSuccess ? METRO_OK : METRO_ERR_HIP;
}
