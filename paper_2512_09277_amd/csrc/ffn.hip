// moe_grouped_ffn for gfx950: SwiGLU expert FFN over one rank's per-slot token lists.
//
// Decode is HBM-bound: runtime follows the bytes of the activated experts' weights (Sec. 3.2 of
// arxiv 2512.09277).  Every activated weight row is streamed from HBM once, with 128-bit loads that
// land directly in the matrix-core operand layout (16 rows x 64 contiguous bytes per instruction);
// the small, heavily reused activations are staged through LDS.  Work is cut into tiles of one
// slot's rows (at most 128; 32 on the smallest shapes):
//   stream tiles (<= 32 rows at large shapes, the bulk of the bytes): per wave 2 x 16 weight rows, K steps of 128,
//       loads issued two steps ahead so that ~128 KB per CU are in flight at 2 waves per SIMD;
//   wide tiles (33..128 rows at large shapes, the few popular experts): per wave 4 x 16 weight rows, K steps of 64,
//       so that each activation fragment read from LDS feeds four MFMAs and the matrix cores,
//       not LDS, bound the tile; they are listed first so that they spread over the chip early.
//   gate/up: a wave owns gate rows and the matching up rows, so silu(gate)*up is formed in
//            registers and written once as bf16;   down: same structure over K = I.
// A slot with no rows produces no tile and its weights are never touched.  There is no planning pass:
// every workgroup finds its (tile, column tile) from group_offsets itself.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "device_utils.h"
#include "host_utils.h"
#include "metro.h"

namespace metro {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kMaxSpr = 64;
constexpr int kWideRows = 128;              // rows of a full wide tile
constexpr int kStreamRows = 128;            // largest remainder that may become a stream tile

struct Tile {
    int slot, row0, rows, col;              // rows [row0, row0 + rows) of a slot x column tile `col`
};

// Upper bound of the tile count (the launch grid; workgroups past the real count exit after locating
// nothing): cap / tile_rows full tiles, and per slot one remainder -- or two tiles where one-tile slots
// are cut finer (each at least half a tile).
inline int max_tiles(int cap, int spr, int tile_rows, bool finer_singles) {
    return (finer_singles ? 2 : 1) * spr + cap / tile_rows;
}

// ------------------------------------------------------------------------------------------ work items
// A slot of m rows gives m / tile_rows full tiles and one tile for the remainder; a tile is wide if it has
// more than `stream_rows` rows.  Tile order: full tiles, then the remainders by rows descending
// (ties: lower slot first); the first n_wide of them are the wide ones.  Work item = (tile, column
// tile), tile-major, wide items first, `ntw` column tiles per wide tile and `nts` per stream tile.
// Every workgroup derives its own item from group_offsets (65 integers, one memory round trip, a few
// hundred scalar-ish instructions): no planning kernel, no list in memory.  Each wave computes the
// same result with lane = local slot; everything returned is uniform.
struct Item {
    Tile tile;
    bool valid, wide;
};

__device__ __forceinline__ Item locate_item(const int32_t* __restrict__ group_offsets, int spr, int cap,
                                            int tile_rows, int single_rows, int stream_rows, int ntw, int nts,
                                            int id) {
    const int l = lane_id();
    int begin = 0, m = 0;
    if (l < spr) {                              // offsets that are not a partition of [0, cap] are clamped
        begin = min(max(group_offsets[l], 0), cap);
        m = min(max(group_offsets[l + 1], begin), cap) - begin;
    }
    // one-tile slots may be cut finer than the slots that re-read their weights once per tile
    const int th = (single_rows > 0 && m <= tile_rows) ? single_rows : tile_rows;
    const int full = m / th, part = m % th;
    int incl = full;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d);
        if (l >= d) incl += up;
    }
    const int n_full = __builtin_amdgcn_readlane(incl, kWave - 1);
    int rank = 0;                               // remainders: more rows first, then lower slot
#pragma unroll
    for (int j = 0; j < kWave; ++j) {
        const int pj = __builtin_amdgcn_readlane(part, j);
        rank += (pj > part || (pj == part && j < l)) ? 1 : 0;
    }
    const int n_part_wide = __popcll(__ballot(part > stream_rows));
    const int n_part = __popcll(__ballot(part > 0));
    // stream_rows >= 128: no wide class at all, full tiles take the stream path too
    const int n_wide = stream_rows >= tile_rows ? 0 : n_full + n_part_wide;
    const int n_stream = n_full + n_part - n_wide;
    const int wide_items = n_wide * ntw, n_items = wide_items + n_stream * nts;

    Item it;
    it.valid = id < n_items;
    it.wide = id < wide_items;
    it.tile = Tile{0, 0, 0, 0};
    if (!it.valid) return it;
    const int nt = it.wide ? ntw : nts, r = it.wide ? id : id - wide_items;
    const int tl = r / nt;
    const int ti = it.wide ? tl : n_wide + tl;
    it.tile.col = r - tl * nt;
    if (ti < n_full) {
        const uint64_t owner = __ballot(incl - full <= ti && ti < incl);      // exactly one lane
        const int o = __ffsll((unsigned long long)owner) - 1;
        const int first = __builtin_amdgcn_readlane(incl - full, o);
        it.tile.slot = o;
        const int th_o = __builtin_amdgcn_readlane(th, o);
        it.tile.row0 = __builtin_amdgcn_readlane(begin, o) + (ti - first) * th_o;
        it.tile.rows = th_o;
    } else {
        const uint64_t owner = __ballot(part > 0 && n_full + rank == ti);     // exactly one lane
        const int o = __ffsll((unsigned long long)owner) - 1;
        it.tile.slot = o;
        it.tile.row0 = __builtin_amdgcn_readlane(begin + full * th, o);
        it.tile.rows = __builtin_amdgcn_readlane(part, o);
    }
    it.valid = it.tile.rows > 0;                // always true here; keeps a broken invariant from indexing row -1
    return it;
}

// ------------------------------------------------------------------------------------------ MFMA path
struct FfnArgs {
    const __bf16* src;        // gate/up: x[T,H]; down: act[cap,I]
    const int32_t* perm_pair; // gate/up only
    const __bf16* w;          // gate/up: w13[spr,2I,H]; down: w2[spr,H,I]
    __bf16* dst;              // gate/up: act[cap,I]; down: y_perm[cap,H]
    const int32_t* group_offsets;
    int T, k, spr, H, I;
    int ldw;                  // elements between consecutive weight rows (>= K)
    int tile_rows;            // rows of a full tile (<= 128)
    int single_rows;          // > 0: slots of at most tile_rows rows are cut into tiles of this many rows
    int bk256;                // <= 32-row tiles take K steps of 256 with one step of prefetch
    int stream_rows;          // tiles with more rows are wide
    int ntw, nts;             // column tiles per wide / stream tile
};

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
    const uint32_t ra = ua + 0x7fffu + ((ua >> 16) & 1u);       // round to nearest even
    const uint32_t rb = ub + 0x7fffu + ((ub >> 16) & 1u);
    // NaN stays a (quiet) NaN: the rounding add could carry its mantissa into Inf or -0
    ua = (a != a) ? (ua | 0x00400000u) : ra;
    ub = (b != b) ? (ub | 0x00400000u) : rb;
    return (ua >> 16) | (ub & 0xffff0000u);
}

__device__ __forceinline__ float silu(float g) { return g / (1.0f + __expf(-g)); }

// D[i][j] of block b, sub-tile mt: i = output column 4*q + v of the block, j = tile row r16.
template <bool kGateUp, int NB, int MT>
__device__ __forceinline__ void store_tile(const FfnArgs& a, const Tile& t, const floatx4 (&acc)[NB][MT], int col0,
                                           int n_out, int mt_count, int r16, int q) {
    const int H = a.H, I = a.I;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int row = mt * 16 + r16;
        if (mt < mt_count && row < t.rows) {
            if (kGateUp) {
#pragma unroll
                for (int b = 0; b < NB / 2; ++b) {
                    const int col = col0 + b * 16;
                    if (col < n_out) {
                        const floatx4 g = acc[b][mt], u = acc[b + NB / 2][mt];
                        u32x2 o;
                        o.x = pack_bf16x2(silu(g[0]) * u[0], silu(g[1]) * u[1]);
                        o.y = pack_bf16x2(silu(g[2]) * u[2], silu(g[3]) * u[3]);
                        *reinterpret_cast<u32x2*>(a.dst + (size_t)(t.row0 + row) * I + col + q * 4) = o;
                    }
                }
            } else {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const int col = col0 + b * 16;
                    if (col < n_out) {
                        u32x2 o;
                        o.x = pack_bf16x2(acc[b][mt][0], acc[b][mt][1]);
                        o.y = pack_bf16x2(acc[b][mt][2], acc[b][mt][3]);
                        *reinterpret_cast<u32x2*>(a.dst + (size_t)(t.row0 + row) * H + col + q * 4) = o;
                    }
                }
            }
        }
    }
}

// do_step(U, s) for U = 0..n-1 with compile-time U (buffer indices), s = s0 + U.
template <int... Us, typename F>
__device__ __forceinline__ void run_steps(std::integer_sequence<int, Us...>, F& f, int s0) {
    (f(std::integral_constant<int, Us>{}, s0 + Us), ...);
}
template <int... Us, typename F>
__device__ __forceinline__ void run_steps_tail(std::integer_sequence<int, Us...>, F& f, int s0, int n_steps) {
    // short-circuit: once a step is past the end nothing after it is tested, the paths join only at the end
    (void)((s0 + Us < n_steps && (f(std::integral_constant<int, Us>{}, s0 + Us), true)) && ...);
}

// One tile x one column tile.
//   NB    16-row weight blocks per wave (gate/up: NB/2 gate blocks + the matching up blocks)
//   MT    16-row activation sub-tiles (tile rows <= 16*MT)
//   BK    K elements per step;  DEPTH  steps the loads run ahead
// Lane (r16, q) of a wave supplies, for MFMA j of a step, the 8 elements k = j*32 + q*8 .. +8 of
// weight row r16 (A operand) and of tile row r16 (B operand): one load instruction reads 64
// contiguous bytes of each of 16 rows.  D[i][j]: i = weight row 4*q + v, j = tile row r16.
template <bool kGateUp, int NB, int MT, int BK, int DEPTH>
__device__ __forceinline__ void ffn_tile(const FfnArgs& a, const Tile t, const int nt, char* lds) {
    constexpr int NJ = BK / 32;                 // MFMAs per block per step
    constexpr int NW = DEPTH + 1;               // weight register buffers
    constexpr int kLdsRow = BK * 2 + 16;        // bytes per staged row (+16 spreads the banks)
    constexpr int kChunks = BK * 2 / 16;        // 16-byte chunks per staged row
    constexpr int kRowsPerPass = kThreads / kChunks;
    constexpr int NP = (MT * 16 + kRowsPerPass - 1) / kRowsPerPass;   // staging loads per thread
    constexpr int kPeriod = (DEPTH == 1) ? 2 : (DEPTH == 2) ? 6 : 12; // lcm(NW, DEPTH, 2)
    static_assert(DEPTH >= 1 && DEPTH <= 3, "prefetch distance");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);        // wave index, kept in a scalar register
    const int r16 = lane & 15, q = lane >> 4;
    const int H = a.H, I = a.I;
    const int K = kGateUp ? H : I;
    const int n_steps = K / BK;
    const int mt_count = (t.rows + 15) >> 4;
    const int n_out = kGateUp ? I : H;          // output columns of this stage
    const int cols_per_wave = kGateUp ? NB * 8 : NB * 16;
    const int col0 = nt * 4 * cols_per_wave + wv * cols_per_wave;     // first output column of the wave

    // Addresses are a uniform base (scalar registers) plus a 32-bit per-lane offset, which keeps the
    // vector registers for data in flight.  Weight row of block b: gate/up pairs block b (gate) with
    // block b + NB/2 (up).
    const char* wslot = reinterpret_cast<const char*>(a.w) + (size_t)t.slot * (kGateUp ? 2 * I : H) * a.ldw * 2;
    const uint32_t w_lane = (uint32_t)(r16 * a.ldw + q * 8) * 2u;
    const char* pw[NB];                                               // uniform: first row of block b
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        int col = kGateUp ? col0 + (b % (NB / 2)) * 16 : col0 + b * 16;
        col = col < n_out ? col : n_out - 16;   // a block past the last column repeats the last block
        const int row = (kGateUp && b >= NB / 2) ? I + col : col;
        pw[b] = wslot + (size_t)row * a.ldw * 2;
    }

    // activation staging: thread (frow, fchunk) copies 16 bytes of rows frow, frow + kRowsPerPass, ...
    // (the host only takes this path while every activation byte offset fits 32 bits)
    const int frow = tid / kChunks, fchunk = tid % kChunks;
    const char* xbase = reinterpret_cast<const char*>(a.src);
    uint32_t x_lane[NP];
#pragma unroll
    for (int pz = 0; pz < NP; ++pz) {
        int row = pz * kRowsPerPass + frow;
        row = row < t.rows ? row : t.rows - 1;  // rows past the tile repeat its last row
        const uint32_t src_row = kGateUp ? (uint32_t)min(max(a.perm_pair[t.row0 + row] / a.k, 0), a.T - 1)
                                         : (uint32_t)(t.row0 + row);
        x_lane[pz] = src_row * (uint32_t)(K * 2) + fchunk * 16;
    }
    const int wr_off = frow * kLdsRow + fchunk * 16;
    const int rd_off = r16 * kLdsRow + q * 16;
    constexpr int kLdsBuf = NP * kRowsPerPass * kLdsRow;   // staged rows past 16*MT are never read

    floatx4 acc[NB][MT];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[b][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

    u32x4 w[NW][NB * NJ];
    u32x4 xr[DEPTH][NP];

    auto load_w = [&](int buf, int step) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                w[buf][b * NJ + j] = *reinterpret_cast<const u32x4*>(pw[b] + (size_t)step * (BK * 2) + w_lane + j * 64);
    };
    auto load_x = [&](int set, int step) {
#pragma unroll
        for (int pz = 0; pz < NP; ++pz)
            xr[set][pz] = *reinterpret_cast<const u32x4*>(xbase + (size_t)step * (BK * 2) + x_lane[pz]);
    };
    auto park_x = [&](int set, int buf) {
#pragma unroll
        for (int pz = 0; pz < NP; ++pz)
            *reinterpret_cast<u32x4*>(lds + buf * kLdsBuf + wr_off + pz * kRowsPerPass * kLdsRow) = xr[set][pz];
    };

    // Every load below is unconditional (past the last step the index is clamped, which re-reads
    // the last step): the compiler can then count outstanding loads exactly and waits only for
    // the ones a step consumes, instead of draining the queue at every branch join.
    const int last = n_steps - 1;
    // (the weight addresses need only the tile, the activation addresses also need perm_pair: the
    // weight loads go out first so that they overlap that extra round trip)
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) load_w(d, min(d, last));
    load_x(0, 0);
#pragma unroll
    for (int d = 1; d < DEPTH; ++d) load_x(d % DEPTH, min(d, last));
    park_x(0, 0);
    __syncthreads();

    // One K step with compile-time buffer indices u (= step s mod kPeriod).
    auto do_step = [&](auto U, const int s) {
        constexpr int u = decltype(U)::value;
        // Loads retire in issue order: the activations go first so that waiting for them (to park
        // them one step later) never waits for the younger weight loads.
        const int ps = min(s + DEPTH, last);                          // past the end: re-read the last step
        load_x(u % DEPTH, ps);
        load_w((u + DEPTH) % NW, ps);
        const char* cur = lds + (u % 2) * kLdsBuf + rd_off;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (mt < mt_count) {
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const bf16x8 xb = *reinterpret_cast<const bf16x8*>(cur + mt * 16 * kLdsRow + j * 64);
#pragma unroll
                    for (int b = 0; b < NB; ++b)
                        acc[b][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8, w[u % NW][b * NJ + j]), xb, acc[b][mt], 0, 0, 0);
                }
            }
        }
        // activations of the next step were loaded DEPTH-1 steps ago (set (u+1) % DEPTH)
        park_x((u + 1) % DEPTH, (u + 1) % 2);
        __syncthreads();
    };

    int s0 = 0;
    for (; s0 + kPeriod <= n_steps; s0 += kPeriod) run_steps(std::make_integer_sequence<int, kPeriod>{}, do_step, s0);
    run_steps_tail(std::make_integer_sequence<int, kPeriod - 1>{}, do_step, s0, n_steps);
    store_tile<kGateUp, NB, MT>(a, t, acc, col0, n_out, mt_count, r16, q);
}

constexpr int kLdsStream = 2 * 64 * (128 * 2 + 16);
constexpr int kLdsWide = 2 * 128 * (64 * 2 + 16);
constexpr int kLdsBytes = kLdsWide > kLdsStream ? kLdsWide : kLdsStream;

template <bool kGateUp>
__global__ __launch_bounds__(kThreads, 2) void ffn_mfma_kernel(FfnArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    // Work items = (tile, column tile), wide items first: a wide workgroup lives several times longer
    // than a stream one, so it has to start early for the stream items to fill in around it.
    // (Measured alternatives that lost: spreading the wide items through the launch order,
    // alternating wide and stream items, and per-XCD work queues.)  Everything here is uniform per
    // workgroup.
    const Item it = locate_item(a.group_offsets, a.spr, a.T * a.k, a.tile_rows, a.single_rows, a.stream_rows, a.ntw, a.nts, blockIdx.x);
    if (!it.valid) return;
    const Tile t = it.tile;
    // partial wide tiles stage only the rows they have; with half the accumulators the 64-row variant
    // also affords a second K step of weights in flight (token-balanced rank: gate/up 401 -> 390 us)
    if (it.wide && t.rows <= 64) ffn_tile<kGateUp, 4, 4, 64, 2>(a, t, t.col, lds);
    else if (it.wide && t.rows <= 96) ffn_tile<kGateUp, 4, 6, 64, 1>(a, t, t.col, lds);
    else if (it.wide) ffn_tile<kGateUp, 4, 8, 64, 1>(a, t, t.col, lds);
    else if (t.rows <= 32 && a.bk256) {
        if (t.rows <= 16) ffn_tile<kGateUp, 2, 1, 256, 1>(a, t, t.col, lds);
        else ffn_tile<kGateUp, 2, 2, 256, 1>(a, t, t.col, lds);
    }
    else if (t.rows <= 16) ffn_tile<kGateUp, 2, 1, 128, 2>(a, t, t.col, lds);
    else if (t.rows <= 32) ffn_tile<kGateUp, 2, 2, 128, 2>(a, t, t.col, lds);
    else if (t.rows <= 64) ffn_tile<kGateUp, 2, 4, 128, 2>(a, t, t.col, lds);
    else ffn_tile<kGateUp, 2, 8, 64, 3>(a, t, t.col, lds);
}

// ------------------------------------------------------------------------------------------ general path
// Any shape, fp32 or bf16 storage, fp32 arithmetic on the vector ALUs (the matrix-core path needs bf16 and
// H, I multiples of 128).  One workgroup = 16 rows of one slot x 64 output columns; both operands go through LDS
// in K steps of 32 (the loads of the next step in flight in registers meanwhile), so a weight element is
// fetched once per 16 rows and an activation element once per 64 columns (not once per output element); a
// thread owns 4 outputs of one row and adds its products in ascending k with fused multiply-adds.
template <typename T>
__device__ __forceinline__ float to_f32(T v);
template <>
__device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ float to_f32<__bf16>(__bf16 v) { return (float)v; }

template <typename T>
__device__ __forceinline__ T from_f32(float v);
template <>
__device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ __bf16 from_f32<__bf16>(float v) {
    const uint16_t bits = (uint16_t)(pack_bf16x2(v, 0.f) & 0xffffu);
    return __builtin_bit_cast(__bf16, bits);
}

constexpr int kGenRows = 16, kGenCols = 64, kGenK = 32;

// Row tile `b` (counted over the slots' tiles of 16 rows, slot by slot) -> slot, first row, rows; rows = 0 past
// the last tile.  One thread walks the <= 64 slots, the result reaches the workgroup through LDS.
__device__ __forceinline__ void general_locate(const int32_t* __restrict__ group_offsets, int spr, int cap, int b,
                                               int* s_tile) {
    if (threadIdx.x == 0) {
        int slot = 0, row0 = 0, rows = 0;
        for (int l = 0; l < spr; ++l) {
            const int begin = min(max(group_offsets[l], 0), cap);
            const int m = min(max(group_offsets[l + 1], begin), cap) - begin;
            const int nt = (m + kGenRows - 1) / kGenRows;
            if (b < nt) {
                slot = l;
                row0 = begin + b * kGenRows;
                rows = min(kGenRows, m - b * kGenRows);
                break;
            }
            b -= nt;
        }
        s_tile[0] = slot;
        s_tile[1] = row0;
        s_tile[2] = rows;
    }
    __syncthreads();
}

template <typename T>
__global__ __launch_bounds__(kThreads) void general_gate_up_kernel(const T* __restrict__ x,
                                                                   const int32_t* __restrict__ perm_pair,
                                                                   const int32_t* __restrict__ group_offsets, int Tn,
                                                                   int k, int spr, int H, int I,
                                                                   const T* __restrict__ w13, int ldw,
                                                                   float* __restrict__ act) {
    __shared__ float xs[kGenRows][kGenK + 1], wg[kGenCols][kGenK + 1], wu[kGenCols][kGenK + 1];
    __shared__ int s_tile[3], s_tok[kGenRows];
    general_locate(group_offsets, spr, Tn * k, blockIdx.x, s_tile);
    const int slot = s_tile[0], row0 = s_tile[1], rows = s_tile[2];
    if (rows == 0) return;                                           // uniform
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    const int col0 = blockIdx.y * kGenCols;
    if (tid < kGenRows) s_tok[tid] = min(max(perm_pair[row0 + min(tid, rows - 1)] / k, 0), Tn - 1);
    __syncthreads();
    const T* wslot = w13 + (size_t)slot * 2 * I * ldw;
    float g[4] = {0.f, 0.f, 0.f, 0.f}, u[4] = {0.f, 0.f, 0.f, 0.f};
    // the global loads of step s + 1 are in flight (in registers) while step s is multiplied out of LDS
    constexpr int NX = kGenRows * kGenK / kThreads, NW = kGenCols * kGenK / kThreads;
    float rx[NX], rg[NW], ru[NW];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int j = 0; j < NX; ++j) {
            const int e = tid + j * kThreads, r = e / kGenK, kk = e % kGenK;
            rx[j] = (r < rows && k0 + kk < H) ? to_f32<T>(x[(size_t)s_tok[r] * H + k0 + kk]) : 0.f;
        }
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            const int e = tid + j * kThreads, c = e / kGenK, kk = e % kGenK;
            const bool in = col0 + c < I && k0 + kk < H;
            const size_t at = (size_t)(col0 + c) * ldw + k0 + kk;
            rg[j] = in ? to_f32<T>(wslot[at]) : 0.f;
            ru[j] = in ? to_f32<T>(wslot[(size_t)I * ldw + at]) : 0.f;
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < H; k0 += kGenK) {
#pragma unroll
        for (int j = 0; j < NX; ++j) {
            const int e = tid + j * kThreads;
            xs[e / kGenK][e % kGenK] = rx[j];
        }
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            const int e = tid + j * kThreads;
            wg[e / kGenK][e % kGenK] = rg[j];
            wu[e / kGenK][e % kGenK] = ru[j];
        }
        __syncthreads();
        if (k0 + kGenK < H) fetch(k0 + kGenK);                       // uniform
#pragma unroll 8
        for (int kk = 0; kk < kGenK; ++kk) {
            const float xv = xs[ty][kk];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                g[c] = fmaf(xv, wg[tx + 16 * c][kk], g[c]);
                u[c] = fmaf(xv, wu[tx + 16 * c][kk], u[c]);
            }
        }
        __syncthreads();
    }
    if (ty < rows) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int col = col0 + tx + 16 * c;
            if (col < I) act[(size_t)(row0 + ty) * I + col] = g[c] / (1.0f + expf(-g[c])) * u[c];
        }
    }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void general_down_kernel(const float* __restrict__ act,
                                                                const int32_t* __restrict__ group_offsets, int cap,
                                                                int spr, int H, int I, const T* __restrict__ w2, int ldw,
                                                                T* __restrict__ y) {
    __shared__ float as[kGenRows][kGenK + 1], ws[kGenCols][kGenK + 1];
    __shared__ int s_tile[3];
    general_locate(group_offsets, spr, cap, blockIdx.x, s_tile);
    const int slot = s_tile[0], row0 = s_tile[1], rows = s_tile[2];
    if (rows == 0) return;                                           // uniform
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    const int col0 = blockIdx.y * kGenCols;
    const T* wslot = w2 + (size_t)slot * H * ldw;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    constexpr int NX = kGenRows * kGenK / kThreads, NW = kGenCols * kGenK / kThreads;
    float ra[NX], rw[NW];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int j = 0; j < NX; ++j) {
            const int e = tid + j * kThreads, r = e / kGenK, kk = e % kGenK;
            ra[j] = (r < rows && k0 + kk < I) ? act[(size_t)(row0 + r) * I + k0 + kk] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            const int e = tid + j * kThreads, c = e / kGenK, kk = e % kGenK;
            rw[j] = (col0 + c < H && k0 + kk < I) ? to_f32<T>(wslot[(size_t)(col0 + c) * ldw + k0 + kk]) : 0.f;
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < I; k0 += kGenK) {
#pragma unroll
        for (int j = 0; j < NX; ++j) {
            const int e = tid + j * kThreads;
            as[e / kGenK][e % kGenK] = ra[j];
        }
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            const int e = tid + j * kThreads;
            ws[e / kGenK][e % kGenK] = rw[j];
        }
        __syncthreads();
        if (k0 + kGenK < I) fetch(k0 + kGenK);                       // uniform
#pragma unroll 8
        for (int kk = 0; kk < kGenK; ++kk) {
            const float av = as[ty][kk];
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = fmaf(av, ws[tx + 16 * c][kk], acc[c]);
        }
        __syncthreads();
    }
    if (ty < rows) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int col = col0 + tx + 16 * c;
            if (col < H) y[(size_t)(row0 + ty) * H + col] = from_f32<T>(acc[c]);
        }
    }
}

// Row tiles of the general path: every slot may end with a partial tile.
inline int general_row_tiles(int cap, int spr) { return cap / kGenRows + spr; }

inline bool mfma_shape(int H, int I, int dtype) {
    return dtype == METRO_DTYPE_BF16 && H % 128 == 0 && I % 128 == 0;
}

inline bool mfma_fits(int T, int k, int H, int I);
inline bool use_mfma(int T, int k, int H, int I, int dtype) { return mfma_shape(H, I, dtype) && mfma_fits(T, k, H, I); }

// The MFMA kernels address activations with 32-bit byte offsets.
inline bool mfma_fits(int T, int k, int H, int I) {
    return (uint64_t)T * H * 2 < (1ull << 32) && (uint64_t)T * k * I * 2 < (1ull << 32);
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Workspace: the activations between the two stages, act[cap, I] (bf16 on the MFMA path, else f32).
inline char* act_of(void* ws) { return (char*)ws; }

int check_common(const int32_t* group_offsets, int T, int k, int spr, int H, int I, int dtype, const void* ws,
                 size_t ws_bytes) {
    if (!group_offsets || !ws) return METRO_ERR_INVALID_ARG;
    if (T < 0 || k < 1 || spr < 1 || H < 1 || I < 1) return METRO_ERR_INVALID_ARG;
    if (dtype != METRO_DTYPE_BF16 && dtype != METRO_DTYPE_F32) return METRO_ERR_UNSUPPORTED;
    if (spr > kMaxSpr || (int64_t)T * k >= (1 << 24)) return METRO_ERR_UNSUPPORTED;
    if (((uintptr_t)ws & 255) != 0) return METRO_ERR_INVALID_ARG;
    if (ws_bytes < moe_grouped_ffn_workspace_bytes(T, k, spr, H, I, dtype)) return METRO_ERR_WORKSPACE;
    return METRO_OK;
}

int enable_large_lds() {                            // opt in to > 64 KB of dynamic LDS, once per device
    static PerDeviceOnce once;
    return once.run([] {
        hipError_t e = hipFuncSetAttribute((const void*)ffn_mfma_kernel<true>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void*)ffn_mfma_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    kLdsBytes);
        return e;
    });
}

// Remainders of at most this many rows become stream tiles.  A wide workgroup prefetches one step
// ahead, so its K loop runs at about one memory latency per step: at large shapes that hides behind
// the stream items, at small ones (short launches, HBM not saturated) it is the critical path.  Small
// FFNs therefore keep every tile on the deep-prefetch stream path, whose narrower column tile costs
// more activation re-reads -- which is what decides at large shapes, where only <= 32 rows go there.
inline int stream_rows_for(int H, int I) { return (size_t)H * I >= (size_t)4096 * 2048 ? 32 : kStreamRows; }

// Rows of a full tile.  128 amortises a slot's weights over the most rows (one HBM pass per 128 rows).
// The smallest FFNs finish in a few tens of microseconds and are bound by their longest workgroup, not
// by bytes: a 128-row tile spends longer in its matrix instructions than the whole launch should take,
// while re-reading a small slot's weights from L2 is cheap, so they cut groups into 32-row tiles
// (Qwen3-30B-shaped METRO rank: 60 -> 52 us; at 4096 x 1536 the same cut loses, 194 -> 250 us).
inline int tile_rows_for(int H, int I) { return (size_t)H * I < (size_t)2048 * 1024 ? 32 : kWideRows; }

inline int launched() { return hipGetLastError() == hipSuccess ? METRO_OK : METRO_ERR_HIP; }

// Built-in workspace of moe_grouped_ffn_static_ws: one array per GPU, held from the moment the library is
// loaded on that GPU until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address it yields (one per device) is what kernels and copies get.
constexpr size_t kStaticWsBytes = METRO_STATIC_WS_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];

// Device address of `scratch` on the current device, looked up once per device.
int static_ws(void** out) {
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> table[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return METRO_ERR_HIP;
    void* p = table[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return METRO_ERR_HIP;
        table[dev].store(p, std::memory_order_release);      // a racing first call stores the same address
    }
    *out = p;
    return METRO_OK;
}

}  // namespace
}  // namespace metro

extern "C" size_t moe_grouped_ffn_workspace_bytes(int T, int k, int spr, int H, int I, int dtype) {
    using namespace metro;
    if (T < 0 || k < 1 || spr < 1 || H < 1 || I < 1) return 0;
    const size_t cap = (size_t)T * k;
    const size_t act = align256(cap * I * (use_mfma(T, k, H, I, dtype) ? 2 : 4));
    return act + 256;
}

extern "C" int moe_grouped_ffn_gate_up(const void* x, const int32_t* perm_pair, const int32_t* group_offsets, int T,
                                       int k, int spr, int H, int I, int dtype, const void* w13, int ldw13,
                                       void* ws, size_t ws_bytes, void* stream) {
    using namespace metro;
    const int rc = check_common(group_offsets, T, k, spr, H, I, dtype, ws, ws_bytes);
    if (rc != METRO_OK) return rc;
    if (!x || !perm_pair || !w13 || (((uintptr_t)x | (uintptr_t)w13) & 15) != 0) return METRO_ERR_INVALID_ARG;
    if (ldw13 < H || ldw13 % 8 != 0) return METRO_ERR_INVALID_ARG;
    const int cap = T * k;
    if (cap == 0) return METRO_OK;
    hipStream_t st = (hipStream_t)stream;
    char* act = act_of(ws);
    if (!use_mfma(T, k, H, I, dtype)) {
        const dim3 grid(general_row_tiles(cap, spr), (I + kGenCols - 1) / kGenCols);
        if (dtype == METRO_DTYPE_F32)
            hipLaunchKernelGGL(general_gate_up_kernel<float>, grid, dim3(kThreads), 0, st, (const float*)x,
                               perm_pair, group_offsets, T, k, spr, H, I, (const float*)w13, ldw13, (float*)act);
        else
            hipLaunchKernelGGL(general_gate_up_kernel<__bf16>, grid, dim3(kThreads), 0, st, (const __bf16*)x,
                               perm_pair, group_offsets, T, k, spr, H, I, (const __bf16*)w13, ldw13, (float*)act);
        return launched();
    }
    if (enable_large_lds() != METRO_OK) return METRO_ERR_HIP;
    FfnArgs a;
    a.src = (const __bf16*)x;
    a.perm_pair = perm_pair;
    a.w = (const __bf16*)w13;
    a.ldw = ldw13;
    a.dst = (__bf16*)act;
    a.group_offsets = group_offsets;
    a.T = T; a.k = k; a.spr = spr; a.H = H; a.I = I;
    a.stream_rows = stream_rows_for(H, I);
    a.tile_rows = tile_rows_for(H, I);
    // mid shapes (every tile on the stream path, 128-row tiles): a one-tile slot of 65..128 rows is the
    // longest workgroup of a launch that has fewer workgroups than the chip has slots; two 64-row tiles
    // balance it (token-balanced rank of the 4096 x 1536 shape: gate/up 109 -> 101 us; no gain for down)
    a.single_rows = (a.stream_rows >= kWideRows && a.tile_rows == kWideRows) ? 64 : 0;
    a.bk256 = 0;
    a.ntw = I / 128;
    a.nts = I / 64;
    hipLaunchKernelGGL(ffn_mfma_kernel<true>, dim3(max_tiles(cap, spr, a.tile_rows, a.single_rows > 0) * a.nts), dim3(kThreads), kLdsBytes, st, a);
    return launched();
}

extern "C" int moe_grouped_ffn_down(const int32_t* group_offsets, int T, int k, int spr, int H, int I, int dtype,
                                    const void* w2, int ldw2, void* y_perm, void* ws, size_t ws_bytes,
                                    void* stream) {
    using namespace metro;
    const int rc = check_common(group_offsets, T, k, spr, H, I, dtype, ws, ws_bytes);
    if (rc != METRO_OK) return rc;
    if (!w2 || !y_perm || (((uintptr_t)w2 | (uintptr_t)y_perm) & 15) != 0) return METRO_ERR_INVALID_ARG;
    if (ldw2 < I || ldw2 % 8 != 0) return METRO_ERR_INVALID_ARG;
    const int cap = T * k;
    if (cap == 0) return METRO_OK;
    hipStream_t st = (hipStream_t)stream;
    char* act = act_of(ws);
    if (!use_mfma(T, k, H, I, dtype)) {
        const dim3 grid(general_row_tiles(cap, spr), (H + kGenCols - 1) / kGenCols);
        if (dtype == METRO_DTYPE_F32)
            hipLaunchKernelGGL(general_down_kernel<float>, grid, dim3(kThreads), 0, st, (const float*)act,
                               group_offsets, cap, spr, H, I, (const float*)w2, ldw2, (float*)y_perm);
        else
            hipLaunchKernelGGL(general_down_kernel<__bf16>, grid, dim3(kThreads), 0, st, (const float*)act,
                               group_offsets, cap, spr, H, I, (const __bf16*)w2, ldw2, (__bf16*)y_perm);
        return launched();
    }
    if (enable_large_lds() != METRO_OK) return METRO_ERR_HIP;
    FfnArgs a;
    a.src = (const __bf16*)act;
    a.perm_pair = nullptr;
    a.w = (const __bf16*)w2;
    a.ldw = ldw2;
    a.dst = (__bf16*)y_perm;
    a.group_offsets = group_offsets;
    a.T = T; a.k = k; a.spr = spr; a.H = H; a.I = I;
    a.stream_rows = stream_rows_for(H, I);
    a.tile_rows = tile_rows_for(H, I);
    a.single_rows = 0;
    // mid shapes: the full 128-row tiles of a several-tile slot take the wide path in this stage (half
    // the column tiles, each activation fragment feeding four matrix instructions); smaller tiles stay
    // on the stream path (METRO rank of the 4096 x 1536 shape: down 71 -> 60 us; a 113-row one-tile
    // slot on the wide path costs the token-balanced rank 8 us, hence "full tiles only")
    if (a.stream_rows >= kWideRows && a.tile_rows == kWideRows) a.stream_rows = kWideRows - 1;
    // a short K (few steps): half as many barriers for the same bytes in flight (Qwen3-30B-shaped
    // down stage 23.2 -> 20.6 us; no gain on the gate/up stage or at I = 2048)
    a.bk256 = I % 256 == 0 && I <= 1536;
    a.ntw = (H + 255) / 256;
    a.nts = H / 128;
    hipLaunchKernelGGL(ffn_mfma_kernel<false>, dim3(max_tiles(cap, spr, a.tile_rows, a.single_rows > 0) * a.nts), dim3(kThreads), kLdsBytes, st, a);
    return launched();
}

extern "C" int moe_grouped_ffn(const void* x, const int32_t* perm_pair, const int32_t* group_offsets, int T, int k,
                               int spr, int H, int I, int dtype, const void* w13, int ldw13, const void* w2,
                               int ldw2, void* y_perm, void* ws, size_t ws_bytes, void* stream) {
    // all arguments are checked before the first launch
    if (!x || !perm_pair || !w13 || !w2 || !y_perm) return METRO_ERR_INVALID_ARG;
    if ((((uintptr_t)x | (uintptr_t)w13 | (uintptr_t)w2 | (uintptr_t)y_perm) & 15) != 0) return METRO_ERR_INVALID_ARG;
    if (ldw13 < H || ldw2 < I || ldw13 % 8 != 0 || ldw2 % 8 != 0) return METRO_ERR_INVALID_ARG;
    int rc = moe_grouped_ffn_gate_up(x, perm_pair, group_offsets, T, k, spr, H, I, dtype, w13, ldw13, ws, ws_bytes,
                                     stream);
    if (rc == METRO_OK)
        rc = moe_grouped_ffn_down(group_offsets, T, k, spr, H, I, dtype, w2, ldw2, y_perm, ws, ws_bytes, stream);
    return rc;
}

extern "C" size_t moe_grouped_ffn_static_ws_bytes(void) { return metro::kStaticWsBytes; }

extern "C" int moe_grouped_ffn_static_ws(const void* x, const int32_t* perm_pair, const int32_t* group_offsets, int T,
                                         int k, int spr, int H, int I, int dtype, const void* w13, int ldw13,
                                         const void* w2, int ldw2, void* y_perm, void* stream) {
    using namespace metro;
    if (T < 0 || k < 1 || spr < 1 || H < 1 || I < 1) return METRO_ERR_INVALID_ARG;
    if (dtype != METRO_DTYPE_BF16 && dtype != METRO_DTYPE_F32) return METRO_ERR_UNSUPPORTED;
    if (spr > kMaxSpr || (int64_t)T * k >= (1 << 24)) return METRO_ERR_UNSUPPORTED;
    if (moe_grouped_ffn_workspace_bytes(T, k, spr, H, I, dtype) > kStaticWsBytes) return METRO_ERR_TOO_LARGE;
    void* ws = nullptr;
    const int rc = static_ws(&ws);
    if (rc != METRO_OK) return rc;
    // the intermediate activations of rows < n_pairs are written by the first stage before the second reads
    // them, so nothing in the array has to start at zero
    return moe_grouped_ffn(x, perm_pair, group_offsets, T, k, spr, H, I, dtype, w13, ldw13, w2, ldw2, y_perm, ws,
                           kStaticWsBytes, stream);
}
