// Weighted un-permute (CPM-2 Section 2.1: the selected experts' outputs stand in for the FFN
// output of the token): y[t] = sum_j w[t, j] * Yp[inv[t*k + j]], fp32 sum in slot order, one
// rounding to the storage type.  One block per token, 16-byte vectors, coalesced on both sides.
#include "common.h"

namespace moe {
namespace {

constexpr int kMaxK = 8;

__device__ inline float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ inline uint32_t pack_bf16(float lo, float hi) {
    const uint16_t a = __builtin_bit_cast(uint16_t, static_cast<__bf16>(lo));
    const uint16_t b = __builtin_bit_cast(uint16_t, static_cast<__bf16>(hi));
    return a | (static_cast<uint32_t>(b) << 16);
}

template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint4* __restrict__ Yp, const int32_t* __restrict__ inv,
                                                      const float* __restrict__ w, uint4* __restrict__ y, int k,
                                                      int vec_per_row, int n_rows) {
    const int t = blockIdx.x;
    int rows[kMaxK];
    float wt[kMaxK];
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) {
        rows[j] = j < k ? min(max(inv[static_cast<size_t>(t) * k + j], 0), n_rows - 1) : 0;   // never outside Yp
        wt[j] = j < k ? w[static_cast<size_t>(t) * k + j] : 0.f;
    }
    for (int v = threadIdx.x; v < vec_per_row; v += 256) {
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
#pragma unroll
        for (int j = 0; j < kMaxK; ++j) {
            if (j < k) {
                const uint4 u = Yp[static_cast<size_t>(rows[j]) * vec_per_row + v];
                if (BF16) {
                    acc[0] = fmaf(wt[j], bf16_lo(u.x), acc[0]); acc[1] = fmaf(wt[j], bf16_hi(u.x), acc[1]);
                    acc[2] = fmaf(wt[j], bf16_lo(u.y), acc[2]); acc[3] = fmaf(wt[j], bf16_hi(u.y), acc[3]);
                    acc[4] = fmaf(wt[j], bf16_lo(u.z), acc[4]); acc[5] = fmaf(wt[j], bf16_hi(u.z), acc[5]);
                    acc[6] = fmaf(wt[j], bf16_lo(u.w), acc[6]); acc[7] = fmaf(wt[j], bf16_hi(u.w), acc[7]);
                } else {
                    acc[0] = fmaf(wt[j], __uint_as_float(u.x), acc[0]); acc[1] = fmaf(wt[j], __uint_as_float(u.y), acc[1]);
                    acc[2] = fmaf(wt[j], __uint_as_float(u.z), acc[2]); acc[3] = fmaf(wt[j], __uint_as_float(u.w), acc[3]);
                }
            }
        }
        uint4 o;
        if (BF16) {
            o.x = pack_bf16(acc[0], acc[1]); o.y = pack_bf16(acc[2], acc[3]);
            o.z = pack_bf16(acc[4], acc[5]); o.w = pack_bf16(acc[6], acc[7]);
        } else {
            o.x = __float_as_uint(acc[0]); o.y = __float_as_uint(acc[1]);
            o.z = __float_as_uint(acc[2]); o.w = __float_as_uint(acc[3]);
        }
        y[static_cast<size_t>(t) * vec_per_row + v] = o;
    }
}

}  // namespace

int launch_combine(const moe_cfg& c, const void* Yp, const int32_t* inv, const float* w, void* y, hipStream_t s) {
    if (c.T == 0) return MOE_OK;
    const int vec_per_row = static_cast<int>(c.d * elem_size(c) / 16);
    if (c.dtype == MOE_BF16)
        hipLaunchKernelGGL(combine_kernel<true>, dim3(c.T), dim3(256), 0, s, static_cast<const uint4*>(Yp), inv, w,
                           static_cast<uint4*>(y), c.k, vec_per_row, c.T * c.k);
    else
        hipLaunchKernelGGL(combine_kernel<false>, dim3(c.T), dim3(256), 0, s, static_cast<const uint4*>(Yp), inv, w,
                           static_cast<uint4*>(y), c.k, vec_per_row, c.T * c.k);
    MOE_LAUNCH_CHECK("combine_kernel");
    return MOE_OK;
}

}  // namespace moe
