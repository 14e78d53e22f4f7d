// moe_unpermute: one rank's share of the combine step -- a gather of the rows a token owns in
// y_perm, weighted by the gating weights and summed in fp32 in ascending j.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "metro.h"

namespace metro {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float v) {
    uint32_t u = __float_as_uint(v);
    if (v != v) return (u >> 16) | 0x0040u;   // NaN stays a (quiet) NaN: the rounding add could carry it into Inf or -0
    u += 0x7fffu + ((u >> 16) & 1u);          // round to nearest even
    return u >> 16;
}

// bf16, H % 8 == 0: every thread owns 8 consecutive columns (one 128-bit load per row).  KMAX > 0:
// k <= KMAX, the token's rows and weights sit in registers and the row loads of a column go out
// together; KMAX == 0: any k.
template <int KMAX>
__global__ __launch_bounds__(kThreads) void unpermute_bf16x8_kernel(const uint4* __restrict__ y,
                                                                    const int32_t* __restrict__ pair_row,
                                                                    const float* __restrict__ topk_w, int k, int H8,
                                                                    uint4* __restrict__ out) {
    const int t = blockIdx.x;
    const int cap = (int)gridDim.x * k;           // rows of y_perm; an entry of pair_row outside [0, cap) is skipped
    auto add = [](float (&acc)[8], float w, const uint4& v) {
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] = fmaf(w, bf16_bits_to_f32(u[i] & 0xffffu), acc[2 * i]);
            acc[2 * i + 1] = fmaf(w, bf16_bits_to_f32(u[i] >> 16), acc[2 * i + 1]);
        }
    };
    auto pack = [](const float (&acc)[8]) {
        uint4 o;
        o.x = f32_to_bf16_bits(acc[0]) | (f32_to_bf16_bits(acc[1]) << 16);
        o.y = f32_to_bf16_bits(acc[2]) | (f32_to_bf16_bits(acc[3]) << 16);
        o.z = f32_to_bf16_bits(acc[4]) | (f32_to_bf16_bits(acc[5]) << 16);
        o.w = f32_to_bf16_bits(acc[6]) | (f32_to_bf16_bits(acc[7]) << 16);
        return o;
    };
    if (KMAX > 0) {
        int rows[KMAX > 0 ? KMAX : 1];
        float ws[KMAX > 0 ? KMAX : 1];
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            rows[j] = j < k ? pair_row[(size_t)t * k + j] : -1;
            if (rows[j] >= cap) rows[j] = -1;
            ws[j] = j < k ? topk_w[(size_t)t * k + j] : 0.f;
        }
        for (int c = threadIdx.x; c < H8; c += kThreads) {
            uint4 v[KMAX > 0 ? KMAX : 1];
#pragma unroll
            for (int j = 0; j < KMAX; ++j)
                if (rows[j] >= 0) v[j] = y[(size_t)rows[j] * H8 + c];     // uniform per workgroup
            float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < KMAX; ++j)
                if (rows[j] >= 0) add(acc, ws[j], v[j]);
            out[(size_t)t * H8 + c] = pack(acc);
        }
    } else {
        for (int c = threadIdx.x; c < H8; c += kThreads) {
            float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            for (int j = 0; j < k; ++j) {
                const int r = pair_row[(size_t)t * k + j];
                if (r < 0 || r >= cap) continue;
                add(acc, topk_w[(size_t)t * k + j], y[(size_t)r * H8 + c]);
            }
            out[(size_t)t * H8 + c] = pack(acc);
        }
    }
}

template <bool kBf16>
__global__ __launch_bounds__(kThreads) void unpermute_scalar_kernel(const void* __restrict__ y,
                                                                    const int32_t* __restrict__ pair_row,
                                                                    const float* __restrict__ topk_w, int k, int H,
                                                                    void* __restrict__ out) {
    const int t = blockIdx.x;
    const int cap = (int)gridDim.x * k;
    for (int c = threadIdx.x; c < H; c += kThreads) {
        float acc = 0.f;
        for (int j = 0; j < k; ++j) {
            const int r = pair_row[(size_t)t * k + j];
            if (r < 0 || r >= cap) continue;
            const float v = kBf16 ? bf16_bits_to_f32(((const uint16_t*)y)[(size_t)r * H + c])
                                  : ((const float*)y)[(size_t)r * H + c];
            acc = fmaf(topk_w[(size_t)t * k + j], v, acc);
        }
        if (kBf16) ((uint16_t*)out)[(size_t)t * H + c] = (uint16_t)f32_to_bf16_bits(acc);
        else ((float*)out)[(size_t)t * H + c] = acc;
    }
}

}  // namespace
}  // namespace metro

extern "C" int moe_unpermute(const void* y_perm, const int32_t* pair_row, const float* topk_w, int T, int k, int H,
                             int dtype, void* out, void* stream) {
    using namespace metro;
    if (!y_perm || !pair_row || !topk_w || !out) return METRO_ERR_INVALID_ARG;
    if (T < 0 || k < 1 || H < 1) return METRO_ERR_INVALID_ARG;
    if (dtype != METRO_DTYPE_BF16 && dtype != METRO_DTYPE_F32) return METRO_ERR_UNSUPPORTED;
    if ((int64_t)T * k >= (1 << 24)) return METRO_ERR_UNSUPPORTED;
    if (T == 0) return METRO_OK;
    hipStream_t st = (hipStream_t)stream;
    const bool aligned = (((uintptr_t)y_perm | (uintptr_t)out) & 15) == 0;
    if (dtype == METRO_DTYPE_BF16 && H % 8 == 0 && aligned && k <= 8)
        hipLaunchKernelGGL(unpermute_bf16x8_kernel<8>, dim3(T), dim3(kThreads), 0, st, (const uint4*)y_perm, pair_row,
                           topk_w, k, H / 8, (uint4*)out);
    else if (dtype == METRO_DTYPE_BF16 && H % 8 == 0 && aligned)
        hipLaunchKernelGGL(unpermute_bf16x8_kernel<0>, dim3(T), dim3(kThreads), 0, st, (const uint4*)y_perm, pair_row,
                           topk_w, k, H / 8, (uint4*)out);
    else if (dtype == METRO_DTYPE_BF16)
        hipLaunchKernelGGL(unpermute_scalar_kernel<true>, dim3(T), dim3(kThreads), 0, st, y_perm, pair_row, topk_w,
                           k, H, out);
    else
        hipLaunchKernelGGL(unpermute_scalar_kernel<false>, dim3(T), dim3(kThreads), 0, st, y_perm, pair_row, topk_w,
                           k, H, out);
    return hipGetLastError() == hipSuccess ? METRO_OK : METRO_ERR_HIP;
}

extern "C" const char* metro_status_string(int status) {
    switch (status) {
        case METRO_OK: return "ok";
        case METRO_ERR_INVALID_ARG: return "invalid argument";
        case METRO_ERR_UNSUPPORTED: return "size or dtype beyond the supported limits";
        case METRO_ERR_WORKSPACE: return "workspace too small";
        case METRO_ERR_HIP: return "HIP launch failed";
        case METRO_ERR_TOO_LARGE: return "problem larger than the library's built-in scratch buffer";
        default: return "unknown status";
    }
}
