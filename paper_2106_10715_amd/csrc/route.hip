// Gate of the MoE layer (CPM-2 Section 2.1: each token picks its expert from its hidden state;
// Section 2.3: the gate is a frozen random projection): logits = x W_g (+ bias), top-k with ties to
// the lower expert index, softmax combine weights.
//
// The selection must be the one exact arithmetic would make.  The kernel therefore accumulates
// in fp32 with a summation order whose rounding error has a small rigorous bound, compares the gaps
// between the k+1 best logits with that bound, and re-evaluates in fp64 only the tokens that are
// too close to call (products of two bf16 or two fp32 values are exact in fp64).
#include "common.h"

namespace moe {
namespace {

constexpr int kWaves = 4;      // waves per block
constexpr int kTPW = 4;        // tokens per wave, share every W_g load
constexpr int kBK = 32;        // terms of one blocked partial sum
constexpr int kNE = 4;         // experts per lane at most (E <= 256, 64 lanes)
constexpr int kSel = 9;        // k + 1 <= 9 ranks are looked at

__device__ inline float ldf(const float* p, size_t i) { return p[i]; }
__device__ inline float ldf(const __bf16* p, size_t i) { return static_cast<float>(p[i]); }

// (value, expert) order of the gate: larger logit first, equal logits -> lower expert index first.
__device__ inline bool before(double va, int ea, double vb, int eb) { return va > vb || (va == vb && ea < eb); }

// The kk best of the wave's candidates, in order.  Lane `eg` owns experts eg + 64 i (i < kNE) when
// `owner`; every lane receives the same result.
__device__ inline void wave_topk(const double (&lv)[kNE], int eg, bool owner, int E, int kk,
                                 double (&outv)[kSel], int (&oute)[kSel]) {
    unsigned taken = 0;
#pragma unroll
    for (int r = 0; r < kSel; ++r) {
        if (r < kk) {
            double v = -INFINITY;
            int e = 0x7fffffff;
#pragma unroll
            for (int i = 0; i < kNE; ++i) {
                const int ei = eg + 64 * i;
                if (owner && ei < E && !((taken >> i) & 1u) && before(lv[i], ei, v, e)) { v = lv[i]; e = ei; }
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const double ov = __shfl_xor(v, off);
                const int oe = __shfl_xor(e, off);
                if (before(ov, oe, v, e)) { v = ov; e = oe; }
            }
            outv[r] = v;
            oute[r] = e;
            if (owner && (e & 63) == eg) taken |= 1u << (e >> 6);
        }
    }
}

template <typename XT>
__global__ __launch_bounds__(kWaves * 64) void route_kernel(const XT* __restrict__ x, const XT* __restrict__ Wg,
                                                            const float* __restrict__ bias,
                                                            int32_t* __restrict__ idx, float* __restrict__ w,
                                                            int T, int d, int E, int k, int renorm) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t0 = (blockIdx.x * kWaves + wave) * kTPW;
    if (t0 >= T) return;                       // whole wave leaves; the kernel has no block-wide barrier

    int EP = 1;                                // lanes that hold distinct experts (power of two, <= 64)
    while (EP < E && EP < 64) EP <<= 1;
    const int KS = 64 / EP;                    // lane groups that split the reduction dimension
    const int eg = lane & (EP - 1);
    const int ks = lane / EP;
    const bool owner = ks == 0;

    size_t xrow[kTPW];
#pragma unroll
    for (int tt = 0; tt < kTPW; ++tt) xrow[tt] = static_cast<size_t>(min(t0 + tt, T - 1)) * d;

    float tot[kTPW][kNE], wsq[kNE], xsq[kTPW];
#pragma unroll
    for (int i = 0; i < kNE; ++i) {
        wsq[i] = 0.f;
#pragma unroll
        for (int tt = 0; tt < kTPW; ++tt) tot[tt][i] = 0.f;
    }
#pragma unroll
    for (int tt = 0; tt < kTPW; ++tt) xsq[tt] = 0.f;

    // Blocked summation: partial sums of kBK terms are added into the running total, so a logit goes
    // through at most kBK + ceil(d / (KS kBK)) + log2(KS) + 1 roundings instead of d.
    const int span = KS * kBK;
    for (int kb = 0; kb < d; kb += span) {
        float part[kTPW][kNE];
#pragma unroll
        for (int i = 0; i < kNE; ++i)
#pragma unroll
            for (int tt = 0; tt < kTPW; ++tt) part[tt][i] = 0.f;
        for (int ii = 0; ii < kBK; ++ii) {
            const int kk = kb + ii * KS + ks;
            if (kk < d) {
                float xv[kTPW], wv[kNE];
#pragma unroll
                for (int tt = 0; tt < kTPW; ++tt) xv[tt] = ldf(x, xrow[tt] + kk);
#pragma unroll
                for (int i = 0; i < kNE; ++i) {
                    const int ei = eg + 64 * i;
                    wv[i] = ei < E ? ldf(Wg, static_cast<size_t>(kk) * E + ei) : 0.f;
                }
#pragma unroll
                for (int tt = 0; tt < kTPW; ++tt) {
                    xsq[tt] = fmaf(xv[tt], xv[tt], xsq[tt]);
#pragma unroll
                    for (int i = 0; i < kNE; ++i) part[tt][i] = fmaf(xv[tt], wv[i], part[tt][i]);
                }
#pragma unroll
                for (int i = 0; i < kNE; ++i) wsq[i] = fmaf(wv[i], wv[i], wsq[i]);
            }
        }
#pragma unroll
        for (int i = 0; i < kNE; ++i)
#pragma unroll
            for (int tt = 0; tt < kTPW; ++tt) tot[tt][i] += part[tt][i];
    }
    int log2ks = 0;
    for (int off = EP; off < 64; off <<= 1) {
        ++log2ks;
#pragma unroll
        for (int i = 0; i < kNE; ++i) {
            wsq[i] += __shfl_xor(wsq[i], off);
#pragma unroll
            for (int tt = 0; tt < kTPW; ++tt) tot[tt][i] += __shfl_xor(tot[tt][i], off);
        }
#pragma unroll
        for (int tt = 0; tt < kTPW; ++tt) xsq[tt] += __shfl_xor(xsq[tt], off);
    }
    // largest column norm of W_g among this wave's experts (all lanes end with the wave maximum)
    float wn2 = 0.f;
#pragma unroll
    for (int i = 0; i < kNE; ++i) wn2 = fmaxf(wn2, wsq[i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) wn2 = fmaxf(wn2, __shfl_xor(wn2, off));
    const float n_round = static_cast<float>(kBK + (d + span - 1) / span + log2ks + 2);

    float bl[kNE];
#pragma unroll
    for (int i = 0; i < kNE; ++i) {
        const int ei = eg + 64 * i;
        bl[i] = (bias != nullptr && ei < E) ? bias[ei] : 0.f;
    }

    const int kk_sel = min(k + 1, E);
#pragma unroll
    for (int tt = 0; tt < kTPW; ++tt) {
        const int t = t0 + tt;
        if (t >= T) continue;
        double lv[kNE];
#pragma unroll
        for (int i = 0; i < kNE; ++i) lv[i] = static_cast<double>(tot[tt][i] + bl[i]);
        double sv[kSel];
        int se[kSel];
        wave_topk(lv, eg, owner, E, kk_sel, sv, se);

        // |computed - exact| <= n_round u |x_t| |W_g col| + u |logit| for every logit that matters
        // (Cauchy-Schwarz bounds the sum of |products|); 1/16 of slack covers the fp32 norms themselves.
        double vmax = 0.0, gap = INFINITY;
#pragma unroll
        for (int r = 0; r < kSel; ++r) {
            if (r < kk_sel) vmax = fmax(vmax, fabs(sv[r]));
            if (r + 1 < kk_sel) gap = fmin(gap, sv[r] - sv[r + 1]);
        }
        const double delta = 1.0625 * 5.9604644775390625e-8 *
                             (static_cast<double>(n_round) * sqrt(static_cast<double>(xsq[tt]) * static_cast<double>(wn2)) + vmax);
        if (gap <= 2.0 * delta) {
            // too close to call in fp32: exact products, fp64 sums
            double acc[kNE];
#pragma unroll
            for (int i = 0; i < kNE; ++i) acc[i] = 0.0;
            for (int kk = ks; kk < d; kk += KS) {
                const double xv = static_cast<double>(ldf(x, xrow[tt] + kk));
#pragma unroll
                for (int i = 0; i < kNE; ++i) {
                    const int ei = eg + 64 * i;
                    if (ei < E) acc[i] = fma(xv, static_cast<double>(ldf(Wg, static_cast<size_t>(kk) * E + ei)), acc[i]);
                }
            }
            for (int off = EP; off < 64; off <<= 1)
#pragma unroll
                for (int i = 0; i < kNE; ++i) acc[i] += __shfl_xor(acc[i], off);
#pragma unroll
            for (int i = 0; i < kNE; ++i) lv[i] = acc[i] + static_cast<double>(bl[i]);
            wave_topk(lv, eg, owner, E, kk_sel, sv, se);
        }

        // combine weights, fp32
        float wj[kSel];
        float denom = 0.f;
#pragma unroll
        for (int r = 0; r < kSel; ++r)
            if (r < k) wj[r] = expf(static_cast<float>(sv[r] - sv[0]));
        if (renorm) {
#pragma unroll
            for (int r = 0; r < kSel; ++r)
                if (r < k) denom += wj[r];
        } else {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < kNE; ++i)
                if (owner && eg + 64 * i < E) s += expf(static_cast<float>(lv[i] - sv[0]));
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
            denom = s;
        }
        if (lane == 0) {
#pragma unroll
            for (int r = 0; r < kSel; ++r)
                if (r < k) {
                    idx[static_cast<size_t>(t) * k + r] = se[r];
                    w[static_cast<size_t>(t) * k + r] = wj[r] / denom;
                }
        }
    }
}

}  // namespace

int launch_route(const moe_cfg& c, const void* x, const void* Wg, const float* bias, int32_t* idx, float* w,
                 hipStream_t s) {
    if (c.T == 0) return MOE_OK;
    const int per_block = kWaves * kTPW;
    dim3 grid((c.T + per_block - 1) / per_block), block(kWaves * 64);
    if (c.dtype == MOE_BF16)
        hipLaunchKernelGGL(route_kernel<__bf16>, grid, block, 0, s, static_cast<const __bf16*>(x),
                           static_cast<const __bf16*>(Wg), bias, idx, w, c.T, c.d, c.E, c.k, c.renorm);
    else
        hipLaunchKernelGGL(route_kernel<float>, grid, block, 0, s, static_cast<const float*>(x),
                           static_cast<const float*>(Wg), bias, idx, w, c.T, c.d, c.E, c.k, c.renorm);
    MOE_LAUNCH_CHECK("route_kernel");
    return MOE_OK;
}

}  // namespace moe
