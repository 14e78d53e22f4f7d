// moe_grouped_ffn for gfx950: SwiGLU expert FFN over one rank's per-slot token lists.
//
// Decode is HBM-bound: runtime follows the bytes of the activated experts' weights (Sec. 3.2 of
// arxiv 2512.09277), so the kernels are built around streaming every activated weight row from
// HBM exactly once with 128-bit loads straight into the matrix-core operand layout, while the
// (small, heavily reused) activations are staged through LDS:
//   plan     : one wave turns group_offsets into a list of work tiles (slot, first row, rows<=128),
//              heaviest first, so that the few wide groups are spread over the chip early;
//   gate/up  : tile x 64 intermediate columns per workgroup; each wave owns 16 gate rows and the
//              16 matching up rows, so silu(gate)*up is formed in registers and written as bf16;
//   down     : tile x 128 output columns per workgroup, same structure over K = I.
// A slot with no rows produces no tile and its weights are never touched.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_utils.h"
#include "metro.h"

namespace metro {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBK = 128;                    // K elements per pipeline step
constexpr int kLdsRow = kBK * 2 + 16;       // bytes per staged activation row (+16: bank spread)
constexpr int kMaxMT = 8;                   // 16-row sub-tiles per work tile
constexpr int kTileRows = kMaxMT * 16;      // 128
constexpr int kLdsBytes = 2 * kTileRows * kLdsRow;
constexpr int kThreads = 256;
constexpr int kMaxSpr = 64;
constexpr size_t kPlanBytes = 256;          // header before the tile list

struct Tile {
    int slot, row0, rows, pad;
};

struct PlanHeader {
    int n_tiles;
};

__host__ __device__ inline int max_tiles(int cap, int spr) { return spr + cap / kTileRows; }

// ------------------------------------------------------------------------------------------ plan
__global__ __launch_bounds__(kWave) void plan_kernel(const int32_t* __restrict__ group_offsets, int spr, int cap,
                                                     int tile_cap, PlanHeader* __restrict__ hdr,
                                                     Tile* __restrict__ tiles) {
    const int l = threadIdx.x;
    int begin = 0, m = 0;
    if (l < spr) {                              // offsets that are not a partition of [0, cap] are clamped
        begin = min(max(group_offsets[l], 0), cap);
        m = min(max(group_offsets[l + 1], begin), cap) - begin;
    }
    const int full = m / kTileRows, part = m % kTileRows;
    int incl = full;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d);
        if (l >= d) incl += up;
    }
    const int n_full = __shfl(incl, kWave - 1);
    int rank = 0;                               // partial tiles: more rows first, then lower slot
    for (int j = 0; j < kWave; ++j) {
        const int pj = __shfl(part, j);
        rank += (pj > part || (pj == part && j < l)) ? 1 : 0;
    }
    const int n_part = __popcll(__ballot(part > 0));
    for (int f = 0; f < full; ++f)
        if (incl - full + f < tile_cap) tiles[incl - full + f] = Tile{l, begin + f * kTileRows, kTileRows, 0};
    if (part > 0 && n_full + rank < tile_cap) tiles[n_full + rank] = Tile{l, begin + full * kTileRows, part, 0};
    if (l == 0) hdr->n_tiles = min(n_full + n_part, tile_cap);
}

// ------------------------------------------------------------------------------------------ MFMA path
struct FfnArgs {
    const __bf16* src;        // gate/up: x[T,H]; down: act[cap,I]
    const int32_t* perm_pair; // gate/up only
    const __bf16* w;          // gate/up: w13[spr,2I,H]; down: w2[spr,H,I]
    __bf16* dst;              // gate/up: act[cap,I]; down: y_perm[cap,H]
    const PlanHeader* hdr;
    const Tile* tiles;
    int T, k, H, I, n_ntiles;
};

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
    ua += 0x7fffu + ((ua >> 16) & 1u);       // round to nearest even
    ub += 0x7fffu + ((ub >> 16) & 1u);
    return (ua >> 16) | (ub & 0xffff0000u);
}

__device__ __forceinline__ float silu(float g) { return g / (1.0f + __expf(-g)); }

template <int MT>
struct Accum {
    floatx4 a[MT], b[MT];
};

// One K step: issue the next step's loads, run this step's MFMAs, park the next activations in LDS.
template <int MT>
__device__ __forceinline__ void k_step(const u32x4 (&w_cur)[8], u32x4 (&w_nxt)[8], const u32x4* pa0, const u32x4* pa1,
                                       const u32x4* (&px)[MT], int step, int n_steps, int mt_count,
                                       const char* lds_cur, char* lds_nxt, int rd_off, int wr_off,
                                       Accum<MT>& acc) {
    const bool more = step + 1 < n_steps;
    u32x4 xr[MT];
    if (more) {
        const int o = (step + 1) * (kBK * 2 / 16);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            w_nxt[j] = pa0[o + j];
            w_nxt[4 + j] = pa1[o + j];
        }
#pragma unroll
        for (int pz = 0; pz < MT; ++pz) xr[pz] = px[pz][o];
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if (mt < mt_count) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bf16x8 xb = *reinterpret_cast<const bf16x8*>(lds_cur + rd_off + mt * 16 * kLdsRow + j * 16);
                acc.a[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w_cur[j]), xb,
                                                                    acc.a[mt], 0, 0, 0);
                acc.b[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w_cur[4 + j]), xb,
                                                                    acc.b[mt], 0, 0, 0);
            }
        }
    }
    if (more) {
#pragma unroll
        for (int pz = 0; pz < MT; ++pz) *reinterpret_cast<u32x4*>(lds_nxt + wr_off + pz * 16 * kLdsRow) = xr[pz];
    }
    __syncthreads();
}

template <bool kGateUp, int MT>
__device__ __forceinline__ void ffn_tile(const FfnArgs& a, const Tile t, const int nt, char* lds) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r16 = lane & 15, q = lane >> 4;
    const int H = a.H, I = a.I;
    const int K = kGateUp ? H : I;
    const int n_steps = K / kBK;
    const int mt_count = (t.rows + 15) >> 4;

    // weight rows of this wave: two blocks of 16 rows; lane (r16, q) streams 64 contiguous bytes
    // of row r16 per step (k = step*128 + q*32 .. +32), i.e. four MFMA operands.
    int row_a0, row_a1;
    size_t slot_elems;
    if (kGateUp) {
        row_a0 = nt * 64 + wv * 16 + r16;
        row_a1 = row_a0 + I;
        slot_elems = (size_t)2 * I * H;
    } else {
        row_a0 = nt * 128 + wv * 32 + r16;
        row_a1 = row_a0 + 16;
        slot_elems = (size_t)H * I;
    }
    const __bf16* wbase = a.w + (size_t)t.slot * slot_elems;
    const u32x4* pa0 = reinterpret_cast<const u32x4*>(wbase + (size_t)row_a0 * K + q * 32);
    const u32x4* pa1 = reinterpret_cast<const u32x4*>(wbase + (size_t)row_a1 * K + q * 32);

    // activation staging: thread (frow, fchunk) copies 16 bytes of row pz*16+frow per step.
    const int frow = tid >> 4, fchunk = tid & 15;
    const u32x4* px[MT];
#pragma unroll
    for (int pz = 0; pz < MT; ++pz) {
        int row = pz * 16 + frow;
        row = row < t.rows ? row : t.rows - 1;              // rows past the tile repeat its last row
        const size_t src_row = kGateUp ? (size_t)min(max(a.perm_pair[t.row0 + row] / a.k, 0), a.T - 1)
                                       : (size_t)(t.row0 + row);
        px[pz] = reinterpret_cast<const u32x4*>(a.src + src_row * K) + fchunk;
    }
    const int wr_off = frow * kLdsRow + fchunk * 16;
    const int rd_off = r16 * kLdsRow + q * 64;
    char* lds0 = lds;
    char* lds1 = lds + kTileRows * kLdsRow;

    Accum<MT> acc;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        acc.a[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
        acc.b[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    u32x4 w0[8], w1[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        w0[j] = pa0[j];
        w0[4 + j] = pa1[j];
    }
#pragma unroll
    for (int pz = 0; pz < MT; ++pz) *reinterpret_cast<u32x4*>(lds0 + wr_off + pz * 16 * kLdsRow) = px[pz][0];
    __syncthreads();

    for (int s = 0; s < n_steps; s += 2) {
        k_step<MT>(w0, w1, pa0, pa1, px, s, n_steps, mt_count, lds0, lds1, rd_off, wr_off, acc);
        if (s + 1 < n_steps)
            k_step<MT>(w1, w0, pa0, pa1, px, s + 1, n_steps, mt_count, lds1, lds0, rd_off, wr_off, acc);
    }

    // D[i][j]: i = weight row 4*q + v of the 16-row block, j = tile row r16.
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int row = mt * 16 + r16;
        if (mt < mt_count && row < t.rows) {
            if (kGateUp) {
                const floatx4 g = acc.a[mt], u = acc.b[mt];
                u32x2 o;
                o.x = pack_bf16x2(silu(g[0]) * u[0], silu(g[1]) * u[1]);
                o.y = pack_bf16x2(silu(g[2]) * u[2], silu(g[3]) * u[3]);
                *reinterpret_cast<u32x2*>(a.dst + (size_t)(t.row0 + row) * I + nt * 64 + wv * 16 + q * 4) = o;
            } else {
                __bf16* out = a.dst + (size_t)(t.row0 + row) * H + nt * 128 + wv * 32 + q * 4;
                u32x2 o;
                o.x = pack_bf16x2(acc.a[mt][0], acc.a[mt][1]);
                o.y = pack_bf16x2(acc.a[mt][2], acc.a[mt][3]);
                *reinterpret_cast<u32x2*>(out) = o;
                o.x = pack_bf16x2(acc.b[mt][0], acc.b[mt][1]);
                o.y = pack_bf16x2(acc.b[mt][2], acc.b[mt][3]);
                *reinterpret_cast<u32x2*>(out + 16) = o;
            }
        }
    }
}

template <bool kGateUp>
__global__ __launch_bounds__(kThreads, 2) void ffn_mfma_kernel(FfnArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tile_idx = blockIdx.x / a.n_ntiles;
    const int nt = blockIdx.x - tile_idx * a.n_ntiles;
    if (tile_idx >= a.hdr->n_tiles) return;              // uniform: the whole workgroup leaves
    const Tile t = a.tiles[tile_idx];
    if (t.rows <= 16) ffn_tile<kGateUp, 1>(a, t, nt, lds);
    else if (t.rows <= 32) ffn_tile<kGateUp, 2>(a, t, nt, lds);
    else if (t.rows <= 64) ffn_tile<kGateUp, 4>(a, t, nt, lds);
    else ffn_tile<kGateUp, 8>(a, t, nt, lds);
}

// ------------------------------------------------------------------------------------------ general path
// Any shape, fp32 or bf16 storage, fp32 arithmetic: one wave per output element pair.
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

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) v += __shfl_xor(v, d);
    return v;
}

__device__ __forceinline__ int slot_of_row(const int32_t* group_offsets, int spr, int r) {
    int l = 0;
    for (int s = 0; s < spr; ++s)
        if (group_offsets[s] <= r && r < group_offsets[s + 1]) l = s;
    return l;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void general_gate_up_kernel(const T* __restrict__ x,
                                                                   const int32_t* __restrict__ perm_pair,
                                                                   const int32_t* __restrict__ group_offsets, int Tn,
                                                                   int k, int spr, int H, int I,
                                                                   const T* __restrict__ w13, float* __restrict__ act) {
    const int r = blockIdx.x;                     // < T*k by the launch grid
    if (r >= group_offsets[spr]) return;
    const int i = blockIdx.y * (kThreads / kWave) + wave_id();
    if (i >= I) return;
    const int l = slot_of_row(group_offsets, spr, r);
    const T* xr = x + (size_t)min(max(perm_pair[r] / k, 0), Tn - 1) * H;
    const T* wg = w13 + ((size_t)l * 2 * I + i) * H;
    const T* wu = wg + (size_t)I * H;
    float g = 0.f, u = 0.f;
    for (int h = lane_id(); h < H; h += kWave) {
        const float xv = to_f32<T>(xr[h]);
        g = fmaf(xv, to_f32<T>(wg[h]), g);
        u = fmaf(xv, to_f32<T>(wu[h]), u);
    }
    g = wave_sum(g);
    u = wave_sum(u);
    if (lane_id() == 0) act[(size_t)r * I + i] = g / (1.0f + expf(-g)) * u;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void general_down_kernel(const float* __restrict__ act,
                                                                const int32_t* __restrict__ group_offsets, int spr,
                                                                int H, int I, const T* __restrict__ w2,
                                                                T* __restrict__ y) {
    const int r = blockIdx.x;
    if (r >= group_offsets[spr]) return;
    const int c = blockIdx.y * (kThreads / kWave) + wave_id();
    if (c >= H) return;
    const int l = slot_of_row(group_offsets, spr, r);
    const float* ar = act + (size_t)r * I;
    const T* wd = w2 + ((size_t)l * H + c) * I;
    float acc = 0.f;
    for (int i = lane_id(); i < I; i += kWave) acc = fmaf(ar[i], to_f32<T>(wd[i]), acc);
    acc = wave_sum(acc);
    if (lane_id() == 0) y[(size_t)r * H + c] = from_f32<T>(acc);
}

inline bool mfma_shape(int H, int I, int dtype) {
    return dtype == METRO_DTYPE_BF16 && H % 128 == 0 && I % 128 == 0;
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

template <typename Elem>
int launch_general(const void* x, const int32_t* perm_pair, const int32_t* group_offsets, int T, int k, int spr,
                   int H, int I, const void* w13, const void* w2, void* y, float* act, hipStream_t st) {
    const int per = kThreads / kWave, cap = T * k;
    hipLaunchKernelGGL(general_gate_up_kernel<Elem>, dim3(cap, (I + per - 1) / per), dim3(kThreads), 0, st,
                       (const Elem*)x, perm_pair, group_offsets, T, k, spr, H, I, (const Elem*)w13, act);
    hipLaunchKernelGGL(general_down_kernel<Elem>, dim3(cap, (H + per - 1) / per), dim3(kThreads), 0, st, act,
                       group_offsets, spr, H, I, (const Elem*)w2, (Elem*)y);
    return hipGetLastError() == hipSuccess ? METRO_OK : METRO_ERR_HIP;
}

}  // namespace
}  // namespace metro

extern "C" size_t moe_grouped_ffn_workspace_bytes(int T, int k, int spr, int H, int I, int dtype) {
    using namespace metro;
    if (T < 0 || k < 1 || spr < 1 || H < 1 || I < 1) return 0;
    const size_t cap = (size_t)T * k;
    const size_t plan = kPlanBytes + align256(sizeof(Tile) * (size_t)max_tiles((int)cap, spr));
    const size_t act = align256(cap * I * (mfma_shape(H, I, dtype) ? 2 : 4));
    return plan + act + 256;
}

extern "C" int moe_grouped_ffn(const void* x, const int32_t* perm_pair, const int32_t* group_offsets, int T, int k,
                               int spr, int H, int I, int dtype, const void* w13, const void* w2, void* y_perm,
                               void* ws, size_t ws_bytes, void* stream) {
    using namespace metro;
    if (!x || !perm_pair || !group_offsets || !w13 || !w2 || !y_perm || !ws) return METRO_ERR_INVALID_ARG;
    if (T < 0 || k < 1 || spr < 1 || H < 1 || I < 1) return METRO_ERR_INVALID_ARG;
    if (dtype != METRO_DTYPE_BF16 && dtype != METRO_DTYPE_F32) return METRO_ERR_UNSUPPORTED;
    if (spr > kMaxSpr || (int64_t)T * k >= (1 << 24)) return METRO_ERR_UNSUPPORTED;
    if ((((uintptr_t)x | (uintptr_t)w13 | (uintptr_t)w2 | (uintptr_t)y_perm) & 15) != 0 || ((uintptr_t)ws & 255) != 0)
        return METRO_ERR_INVALID_ARG;
    if (ws_bytes < moe_grouped_ffn_workspace_bytes(T, k, spr, H, I, dtype)) return METRO_ERR_WORKSPACE;
    const int cap = T * k;
    if (cap == 0) return METRO_OK;
    hipStream_t st = (hipStream_t)stream;
    char* base = (char*)ws;
    PlanHeader* hdr = (PlanHeader*)base;
    Tile* tiles = (Tile*)(base + kPlanBytes);
    const int mt = max_tiles(cap, spr);
    char* act = base + kPlanBytes + align256(sizeof(Tile) * (size_t)mt);

    if (!mfma_shape(H, I, dtype)) {
        if (dtype == METRO_DTYPE_F32)
            return launch_general<float>(x, perm_pair, group_offsets, T, k, spr, H, I, w13, w2, y_perm,
                                         (float*)act, st);
        return launch_general<__bf16>(x, perm_pair, group_offsets, T, k, spr, H, I, w13, w2, y_perm, (float*)act,
                                      st);
    }

    static bool lds_ok = false;                    // opt in to > 64 KB of dynamic LDS, once
    if (!lds_ok) {
        if (hipFuncSetAttribute((const void*)ffn_mfma_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsBytes) != hipSuccess ||
            hipFuncSetAttribute((const void*)ffn_mfma_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsBytes) != hipSuccess)
            return METRO_ERR_HIP;
        lds_ok = true;
    }
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kWave), 0, st, group_offsets, spr, cap, mt, hdr, tiles);
    FfnArgs a;
    a.perm_pair = perm_pair;
    a.hdr = hdr;
    a.tiles = tiles;
    a.T = T; a.k = k; a.H = H; a.I = I;
    a.src = (const __bf16*)x;
    a.w = (const __bf16*)w13;
    a.dst = (__bf16*)act;
    a.n_ntiles = I / 64;
    hipLaunchKernelGGL(ffn_mfma_kernel<true>, dim3(mt * a.n_ntiles), dim3(kThreads), kLdsBytes, st, a);
    a.src = (const __bf16*)act;
    a.w = (const __bf16*)w2;
    a.dst = (__bf16*)y_perm;
    a.n_ntiles = H / 128;
    hipLaunchKernelGGL(ffn_mfma_kernel<false>, dim3(mt * a.n_ntiles), dim3(kThreads), kLdsBytes, st, a);
    return hipGetLastError() == hipSuccess ? METRO_OK : METRO_ERR_HIP;
}
