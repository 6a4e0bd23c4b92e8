// Gate of the MoE layer (CPM-2 Section 2.1: each token picks its expert from its hidden state;
// Section 2.3: the gate is a frozen random projection): logits = x W_g (+ bias), top-k with ties to
// the lower expert index, softmax combine weights.
//
// The selection must be the one exact arithmetic would make.  The kernel therefore accumulates
// in fp32 with a summation order whose rounding error has a small rigorous bound, compares the gaps
// between the k+1 best logits with that bound, and re-evaluates only the tokens that are too close to
// call: products of two bf16 or two fp32 values are exact in fp64, and their sum is carried in two doubles
// (value and rounding error), which holds it exactly for any inputs of comparable magnitude, so that
// columns whose exact projections tie do tie.
#include "common.h"

#include <atomic>
#include <type_traits>

namespace moe {
namespace {

constexpr int kWaves = 4;      // waves per block
constexpr int kTPW = 4;        // tokens per wave, share every W_g load
constexpr int kBK = 32;        // terms of one blocked partial sum
constexpr int kNE = 4;         // experts per lane at most (E <= 256, 64 lanes)
constexpr int kSel = 9;        // k + 1 <= 9 ranks are looked at

__device__ inline float ldf(const float* p, size_t i) { return p[i]; }
__device__ inline float ldf(const __bf16* p, size_t i) { return static_cast<float>(p[i]); }

// (value, expert) order of the gate: larger logit first, equal logits -> lower expert index first.  A logit is a
// pair (v, l) whose sum is its value, |l| at most half a unit in the last place of v (l = 0 for logits that were
// not re-evaluated), so pairs compare like their values, part by part.
__device__ inline bool before(double va, double la, int ea, double vb, double lb, int eb) {
    return va > vb || (va == vb && (la > lb || (la == lb && ea < eb)));
}

// Sums in twice the working precision for the re-evaluated logits: the products of two stored values (at most 24
// significant bits each) are exact in fp64, every addition keeps its rounding error (which two floating-point
// numbers always represent exactly) in a second double, and the errors are added up there.  As long as the exact
// sum fits some hundred bits (it does unless the inputs span more than 2^50 in magnitude) the pair holds it without
// any rounding, whatever the order of the terms: columns whose exact projections are equal give identical pairs,
// and a tie is a tie.
__device__ inline void dd_add(double& hi, double& lo, double h2, double l2) {
    const double sum = hi + h2, bb = sum - hi;
    lo += ((hi - (sum - bb)) + (h2 - bb)) + l2;
    hi = sum;
}
__device__ inline void dd_add_product(double& hi, double& lo, double x, double w) { dd_add(hi, lo, x * w, 0.0); }
__device__ inline void dd_normalise(double& hi, double& lo) {
    const double sum = hi + lo, bb = sum - hi;
    lo = (hi - (sum - bb)) + (lo - bb);
    hi = sum;
}

// The kk best of the wave's candidates, in order.  Lane `eg` owns experts eg + 64 i (i < kNE) when
// `owner`; every lane receives the same result.
__device__ __attribute__((always_inline)) inline void wave_topk(const double (&lv)[kNE], const double (&ll)[kNE], int eg, bool owner, int E, int kk,
                                 double (&outv)[kSel], int (&oute)[kSel]) {
    unsigned taken = 0;
#pragma unroll
    for (int r = 0; r < kSel; ++r) {
        if (r < kk) {
            double v = -INFINITY, l = 0.0;
            int e = 0x7fffffff;
#pragma unroll
            for (int i = 0; i < kNE; ++i) {
                const int ei = eg + 64 * i;
                if (owner && ei < E && !((taken >> i) & 1u) && before(lv[i], ll[i], ei, v, l, e)) { v = lv[i]; l = ll[i]; e = ei; }
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const double ov = __shfl_xor(v, off), ol = __shfl_xor(l, off);
                const int oe = __shfl_xor(e, off);
                if (before(ov, ol, oe, v, l, e)) { v = ov; l = ol; e = oe; }
            }
            outv[r] = v;
            oute[r] = e;
            if (owner && (e & 63) == eg) taken |= 1u << (e >> 6);
        }
    }
}

// Combine weights of one token from its ranked logits, written by lane 0.  lv: this lane's logits of
// the experts it owns (only read for the full-softmax denominator).
__device__ __attribute__((always_inline)) inline void emit_token(const double (&lv)[kNE], const double (&sv)[kSel], const int (&se)[kSel], int eg, bool owner,
                                  int E, int k, int renorm, int lane, int32_t* __restrict__ idx_row, float* __restrict__ w_row) {
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
                idx_row[r] = se[r];
                w_row[r] = wj[r] / denom;
            }
    }
}

// Sign-bit gate (the gate of Section 2.3 read as a hashing function): column j of the projection gives
// bit j of the expert id, set when the projection is positive.  Lane j < bits holds projection j in
// lv[0].  gap = the smallest |projection| (how close the token is to a boundary), vmax = the largest.
__device__ __attribute__((always_inline)) inline void sign_bits(const double (&lv)[kNE], const double (&ll)[kNE], int eg, bool owner, int bits, int& code,
                                 double& gap, double& vmax) {
    const bool mine = owner && eg < bits;
    const unsigned long long set = __ballot(mine && (lv[0] > 0.0 || (lv[0] == 0.0 && ll[0] > 0.0)));
    code = static_cast<int>(set & ((1ull << bits) - 1ull));
    double lo = mine ? fabs(lv[0]) : INFINITY, hi = mine ? fabs(lv[0]) : 0.0;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        lo = fmin(lo, __shfl_xor(lo, off));
        hi = fmax(hi, __shfl_xor(hi, off));
    }
    gap = lo;
    vmax = hi;
}

// Smallest gap between consecutive ranks 0..kk-1 and the largest magnitude among them.
__device__ __attribute__((always_inline)) inline void rank_gaps(const double (&sv)[kSel], int kk, double& gap, double& vmax) {
    gap = INFINITY;
    vmax = 0.0;
#pragma unroll
    for (int r = 0; r < kSel; ++r) {
        if (r < kk) vmax = fmax(vmax, fabs(sv[r]));
        if (r + 1 < kk) gap = fmin(gap, sv[r] - sv[r + 1]);
    }
}

template <typename XT>
__global__ __launch_bounds__(kWaves * 64) void route_kernel(const XT* __restrict__ x, const XT* __restrict__ Wg,
                                                            const float* __restrict__ bias,
                                                            int32_t* __restrict__ idx, float* __restrict__ w,
                                                            int T, int d, int E, int k, int renorm, int hash) {
    // hash: E is the number of sign bits (columns of the projection), one expert id per token, weight 1
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
        double lv[kNE], ll[kNE];                // logits as pairs (value, low part); the low part is 0 for fp32 logits
#pragma unroll
        for (int i = 0; i < kNE; ++i) { lv[i] = static_cast<double>(tot[tt][i] + bl[i]); ll[i] = 0.0; }
        double sv[kSel];
        int se[kSel];
        int code = 0;
        double vmax, gap;
        if (hash) {
            sign_bits(lv, ll, eg, owner, E, code, gap, vmax);
        } else {
            wave_topk(lv, ll, eg, owner, E, kk_sel, sv, se);
            rank_gaps(sv, kk_sel, gap, vmax);
        }
        // |computed - exact| <= n_round u |x_t| |W_g col| + u |logit| for every logit that matters
        // (Cauchy-Schwarz bounds the sum of |products|); 1/16 of slack covers the fp32 norms themselves.
        const double delta = 1.0625 * 5.9604644775390625e-8 *
                             (static_cast<double>(n_round) * sqrt(static_cast<double>(xsq[tt]) * static_cast<double>(wn2)) + vmax);
        if (gap <= 2.0 * delta) {
            // too close to call in fp32: exact products, sums in twice the fp64 precision
            double acc[kNE], low[kNE];
#pragma unroll
            for (int i = 0; i < kNE; ++i) { acc[i] = 0.0; low[i] = 0.0; }
            for (int kk = ks; kk < d; kk += KS) {
                const double xv = static_cast<double>(ldf(x, xrow[tt] + kk));
#pragma unroll
                for (int i = 0; i < kNE; ++i) {
                    const int ei = eg + 64 * i;
                    if (ei < E) dd_add_product(acc[i], low[i], xv, static_cast<double>(ldf(Wg, static_cast<size_t>(kk) * E + ei)));
                }
            }
            for (int off = EP; off < 64; off <<= 1)
#pragma unroll
                for (int i = 0; i < kNE; ++i) {
                    const double oh = __shfl_xor(acc[i], off), ol = __shfl_xor(low[i], off);
                    dd_add(acc[i], low[i], oh, ol);
                }
#pragma unroll
            for (int i = 0; i < kNE; ++i) {
                dd_add(acc[i], low[i], static_cast<double>(bl[i]), 0.0);
                dd_normalise(acc[i], low[i]);
                lv[i] = acc[i];
                ll[i] = low[i];
            }
            if (hash) sign_bits(lv, ll, eg, owner, E, code, gap, vmax);
            else wave_topk(lv, ll, eg, owner, E, kk_sel, sv, se);
        }
        if (hash) {
            if (lane == 0) { idx[t] = code; w[t] = 1.f; }
        } else {
            emit_token(lv, sv, se, eg, owner, E, k, renorm, lane, idx + static_cast<size_t>(t) * k,
                       w + static_cast<size_t>(t) * k);
        }
    }
}

// ------------------------------------------------------------------------------------------ bf16: MFMA gate
//
// logits tile = 32 tokens x E on 32x32x16 bf16 MFMAs.  The eight waves of a block split the reduction
// dimension (wave w takes the 64-element groups S = w, w+8, ...), the partial tiles are added in wave
// order through LDS.  W_g is first rewritten (gate_prep_kernel) into MFMA fragment order so that its
// fragments are plain 1 KiB coalesced reads, and so that a lane's four fragments of a group use 64
// contiguous bytes of its token row: fragment (nb, S, q), lane l, element j holds
//     W_g[64 S + 32 (l / 32) + 8 q + j, 32 nb + l % 32]            (0 beyond E).
//
// Error bound of an MFMA logit (measured behaviour of the instruction: the addends of one
// instruction -- accumulator and products -- are aligned to the largest of them and cut to fp32
// precision, so one instruction loses at most 17 units in the last place of its largest addend, which
// is at most the sum of |products|): |error| <= (17 n + 8) 2^-24 |x_t| |W_g column| with n the MFMAs a
// wave chains per logit.  Tokens whose k+1 best logits are not separated by twice that are
// re-evaluated in fp64 by the whole block.

constexpr int kGateTokens = 32;
constexpr int kGateWaves = 8;    // waves of a gate block; they split the reduction dimension

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Block b packs the 64-row group S = b of W_g for every 32-expert block and writes the sums of squares
// of those 64 rows per expert column: part[b][E_pad].
__global__ __launch_bounds__(256) void gate_prep_kernel(const uint16_t* __restrict__ Wg, int d, int E, int NB,
                                                        uint4* __restrict__ pack, float* __restrict__ part) {
    __shared__ float sq[4][32];
    const int S = blockIdx.x, nS = d / 64;
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;      // wave q packs fragment q of the group
    const int col_in = lane & 31, row0 = 64 * S + 32 * (lane >> 5) + 8 * q;
    for (int nb = 0; nb < NB; ++nb) {
        const int col = 32 * nb + col_in;
        uint16_t v[8];
        float ss = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            v[j] = col < E ? Wg[static_cast<size_t>(row0 + j) * E + col] : uint16_t(0);
            const float f = __uint_as_float(static_cast<uint32_t>(v[j]) << 16);
            ss = fmaf(f, f, ss);
        }
        uint4 o;
        o.x = v[0] | (static_cast<uint32_t>(v[1]) << 16);
        o.y = v[2] | (static_cast<uint32_t>(v[3]) << 16);
        o.z = v[4] | (static_cast<uint32_t>(v[5]) << 16);
        o.w = v[6] | (static_cast<uint32_t>(v[7]) << 16);
        pack[((static_cast<size_t>(nb) * nS + S) * 4 + q) * 64 + lane] = o;
        ss += __shfl_xor(ss, 32);
        if (lane < 32) sq[q][lane] = ss;
        __syncthreads();
        if (threadIdx.x < 32)
            part[static_cast<size_t>(S) * NB * 32 + col] = ((sq[0][col_in] + sq[1][col_in]) + sq[2][col_in]) + sq[3][col_in];
        __syncthreads();
    }
}

// ---- wave-wide reductions in the lanes' own registers: an inclusive scan by row shifts, then row
// broadcasts, leaves the total in lane 63 (a dozen vector instructions; a butterfly of lane exchanges goes
// through the LDS permute unit six times, some hundred cycles each, and the selection is a chain of them).
template <int CTRL, int ROW_MASK>
__device__ inline unsigned dpp_from(unsigned identity, unsigned v) {
    return static_cast<unsigned>(__builtin_amdgcn_update_dpp(static_cast<int>(identity), static_cast<int>(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ inline unsigned wave_max_u32(unsigned v) {
    v = max(v, dpp_from<0x111, 0xf>(0u, v));      // row_shr:1
    v = max(v, dpp_from<0x112, 0xf>(0u, v));      // row_shr:2
    v = max(v, dpp_from<0x114, 0xf>(0u, v));      // row_shr:4
    v = max(v, dpp_from<0x118, 0xf>(0u, v));      // row_shr:8: lane 15 of every row of 16 holds the row's maximum
    v = max(v, dpp_from<0x142, 0xa>(0u, v));      // row_bcast:15 into rows 1 and 3
    v = max(v, dpp_from<0x143, 0xc>(0u, v));      // row_bcast:31 into rows 2 and 3: lane 63 holds the wave's
    return static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(v), 63));
}
__device__ inline unsigned wave_min_u32(unsigned v) { return ~wave_max_u32(~v); }
__device__ inline float wave_sum_f32(float x) {
    auto step = [](float v, unsigned got) { return v + __uint_as_float(got); };
    x = step(x, dpp_from<0x111, 0xf>(0u, __float_as_uint(x)));
    x = step(x, dpp_from<0x112, 0xf>(0u, __float_as_uint(x)));
    x = step(x, dpp_from<0x114, 0xf>(0u, __float_as_uint(x)));
    x = step(x, dpp_from<0x118, 0xf>(0u, __float_as_uint(x)));
    x = step(x, dpp_from<0x142, 0xa>(0u, __float_as_uint(x)));
    x = step(x, dpp_from<0x143, 0xc>(0u, __float_as_uint(x)));
    return __uint_as_float(static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(__float_as_uint(x)), 63)));
}
// fp32 values as unsigned keys of the same order (finite values; -0 must have been turned into +0)
__device__ inline unsigned order_key(float v) {
    const unsigned u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float from_order_key(unsigned key) {
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

// Value of column `col` of the projection of token t from exact products, by one wave, from the packed fragments:
// lane j takes the 8-row pieces j, j + 64, ... of the column.  PAIR = false: plain fp64 sums (error at most about
// d 2^-53 |x_t| |column|), lo = 0.  PAIR = true: sums in twice that precision, the pair (hi, lo) not yet normalised;
// only needed when fp64 leaves candidates closer than its own error.  Every lane gets the sum.
template <bool PAIR>
__device__ __attribute__((always_inline)) inline void exact_column_dot(const uint16_t* __restrict__ x, const uint4* __restrict__ pack, size_t t,
                                                           int col, int nS, int d, int lane, double& hi, double& lo) {
    const int nb = col >> 5, cin = col & 31;
    const uint4* xr = reinterpret_cast<const uint4*>(x + t * d);
    double sum = 0.0, low = 0.0;
    for (int j = lane; j < nS * 8; j += 64) {
        const int S = j >> 3, q = (j & 7) >> 1, h = j & 1;          // rows 64 S + 32 h + 8 q .. + 8
        const uint4 wq = pack[((static_cast<size_t>(nb) * nS + S) * 4 + q) * 64 + h * 32 + cin];
        const uint4 xq = xr[S * 8 + h * 4 + q];
        const uint32_t xu[4] = {xq.x, xq.y, xq.z, xq.w}, wu[4] = {wq.x, wq.y, wq.z, wq.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const double x0 = static_cast<double>(__uint_as_float(xu[i] << 16)), w0 = static_cast<double>(__uint_as_float(wu[i] << 16));
            const double x1 = static_cast<double>(__uint_as_float(xu[i] & 0xffff0000u)), w1 = static_cast<double>(__uint_as_float(wu[i] & 0xffff0000u));
            if constexpr (PAIR) {
                dd_add_product(sum, low, x0, w0);
                dd_add_product(sum, low, x1, w1);
            } else {
                sum = fma(x0, w0, sum);
                sum = fma(x1, w1, sum);
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const double oh = __shfl_xor(sum, off);
        if constexpr (PAIR) {
            const double ol = __shfl_xor(low, off);
            dd_add(sum, low, oh, ol);
        } else {
            sum += oh;
        }
    }
    hi = sum;
    lo = low;
}

constexpr int kMaxCand = 12;     // columns of one token that are re-evaluated one by one; more than that: all columns

template <int NB>
constexpr int gate_parts() { return NB <= 4 ? kGateWaves : 1; }      // one partial tile per wave while they fit the LDS
template <int NB>
constexpr size_t gate_tile_bytes() { return static_cast<size_t>(gate_parts<NB>()) * kGateTokens * (NB * 32 + 1) * sizeof(float); }

// TOK: tokens a block really has (32, 16 or 8).  The MFMA tile always has 32 token rows; with fewer tokens
// the rows repeat them (the same addresses, so no more bytes are read) and only the first TOK are ranked.
// A short batch gets more, smaller blocks this way: a block's time is mostly its own loads through one
// compute unit plus a selection that is a latency chain per token, and 128 blocks leave half the chip idle.
template <int NB, int TOK>
__global__ __launch_bounds__(kGateWaves * 64, (TOK == 32 && NB == 1) ? 4 : 2) void route_mfma_kernel(const uint16_t* __restrict__ x,
                                                         const uint4* __restrict__ pack, const float* __restrict__ part,
                                                         const float* __restrict__ bias, int32_t* __restrict__ idx,
                                                         float* __restrict__ w, int T, int d, int E, int k, int renorm,
                                                         int hash) {
    // hash: E is the number of sign bits (columns of the projection), one expert id per token, weight 1
    constexpr int EP = NB * 32;
    constexpr int kParts = gate_parts<NB>();
    extern __shared__ float part_tile[];                   // [kParts][kGateTokens][EP + 1]: partial logit tiles
    __shared__ float xsq_w[kGateWaves][kGateTokens];
    __shared__ float wn2_sh;
    __shared__ int flagged[kGateTokens];
    __shared__ double resc[kGateWaves][EP], resc_lo[kGateWaves][EP];    // re-evaluated logits per wave: value and low part
    auto tile_at = [&](int p, int tok, int e) -> float& { return part_tile[(p * kGateTokens + tok) * (EP + 1) + e]; };

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = blockIdx.x * TOK;
    const int nS = d / 64;

    // A wave's groups S = wave, wave + 8, ... are taken kAhead at a time: the token pieces of all of them are
    // requested first (they come from HBM: one latency instead of one per group; the first batch is
    // requested before the column norms below are worked out), the gate fragments, which every block re-reads
    // from the L2, one or two groups ahead of the MFMAs that use them (as many as the registers of two waves
    // per SIMD hold for this number of expert blocks).
    // Long batches (full 32-token blocks, several per compute unit) prefetch less and stay within the registers
    // of two resident blocks per compute unit, which overlap each other's phases.
    constexpr bool kTwoBlocks = TOK == 32 && NB == 1;
    constexpr int kAhead = kTwoBlocks ? 2 : NB <= 2 ? 4 : NB <= 4 ? 2 : 1;
    constexpr int kRing = (NB <= 1 && !kTwoBlocks) ? 3 : 2;
    const int row = min(t0 + (lane & (TOK - 1)), T - 1);
    const uint4* xrow = reinterpret_cast<const uint4*>(x + static_cast<size_t>(row) * d + 32 * (lane >> 5));
    uint4 xv[kAhead][4];
    auto fetch_x = [&](int S0) {
#pragma unroll
        for (int p = 0; p < kAhead; ++p) {
            const int S = S0 + p * kGateWaves < nS ? S0 + p * kGateWaves : 0;      // past the end: group 0, unused
#pragma unroll
            for (int q = 0; q < 4; ++q) xv[p][q] = xrow[S * 8 + q];                // 64 contiguous bytes of the token row
        }
    };
    fetch_x(wave);

    // ---- largest column norm of W_g: fixed-order sum of the per-group parts, then the block maximum.
    // Thread (g, c) adds the parts S = g, g + G, ... of column c; thread c adds the G partial sums in order.
    {
        float* colpart = part_tile;                        // kGateWaves * 64 floats, free until the tiles are written
        constexpr int G = EP >= kGateWaves * 64 ? 1 : kGateWaves * 64 / EP;
        float best = 0.f;
        for (int c0 = 0; c0 < EP; c0 += kGateWaves * 64) {          // one round unless EP exceeds the block
            const int c = c0 + static_cast<int>(threadIdx.x) % EP, g = static_cast<int>(threadIdx.x) / EP;
            float ssum = 0.f;
            if (c < EP && g < G)
                for (int S = g; S < nS; S += G) ssum += part[static_cast<size_t>(S) * EP + c];
            colpart[threadIdx.x] = ssum;
            __syncthreads();
            if (g == 0 && c < EP) {
                float tot = 0.f;
                for (int gg = 0; gg < G; ++gg) tot += colpart[gg * EP + (c - c0)];
                best = fmaxf(best, tot);
            }
            __syncthreads();
        }
        best = __uint_as_float(wave_max_u32(__float_as_uint(best)));   // sums of squares: not negative, ordered like their bits
        if (lane == 0) xsq_w[wave][0] = best;
        __syncthreads();
        if (threadIdx.x == 0) {
            float m = xsq_w[0][0];
            for (int wv = 1; wv < kGateWaves; ++wv) m = fmaxf(m, xsq_w[wv][0]);
            wn2_sh = m;
        }
        __syncthreads();
    }

    // ---- MFMA partial tiles
    f32x16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] = 0.f;
    float xs = 0.f;
    for (int S0 = wave; S0 < nS; S0 += kGateWaves * kAhead) {
        if (S0 != wave) fetch_x(S0);
        uint4 wv[kRing][NB][4];
        auto fetch_w = [&](int p, uint4 (&dst)[NB][4]) {
            const int S = S0 + p * kGateWaves < nS ? S0 + p * kGateWaves : S0;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const uint4* bp = pack + ((static_cast<size_t>(nb) * nS + S) * 4) * 64 + lane;
#pragma unroll
                for (int q = 0; q < 4; ++q) dst[nb][q] = bp[q * 64];
            }
        };
#pragma unroll
        for (int p = 0; p + 1 < kRing; ++p) fetch_w(p, wv[p]);
#pragma unroll
        for (int p = 0; p < kAhead; ++p) {
            if (p + kRing - 1 < kAhead) fetch_w(p + kRing - 1, wv[(p + kRing - 1) % kRing]);
            if (S0 + p * kGateWaves < nS) {                                        // uniform for the wave
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t u[4] = {xv[p][q].x, xv[p][q].y, xv[p][q].z, xv[p][q].w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float lo = __uint_as_float(u[i] << 16), hi = __uint_as_float(u[i] & 0xffff0000u);
                        xs = fmaf(lo, lo, xs);
                        xs = fmaf(hi, hi, xs);
                    }
                }
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xv[p][q]),
                                                                           __builtin_bit_cast(bf16x8, wv[p % kRing][nb][q]), acc[nb], 0, 0, 0);
            }
        }
    }
    xs += __shfl_xor(xs, 32);
    if (lane < 32) xsq_w[wave][lane] = xs;
    // The partial tiles are added in wave order, ((w0 + w1) + w2) + ...: by the lane that reads a logit when
    // every wave has a tile of its own, else wave after wave into one tile.
    if (kParts == kGateWaves) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                tile_at(wave, 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3), 32 * nb + (lane & 31)) = acc[nb][v];
        __syncthreads();
    } else {
        for (int turn = 0; turn < kGateWaves; ++turn) {
            if (wave == turn) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float& at = tile_at(0, 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3), 32 * nb + (lane & 31));
                        at = turn == 0 ? acc[nb][v] : at + acc[nb][v];
                    }
            }
            __syncthreads();
        }
    }

    // ---- selection: wave w ranks tokens w, w + 8, ...
    const int n_chain = ((nS + kGateWaves - 1) / kGateWaves) * 4;                               // MFMAs a wave chains per logit
    const double gamma = 1.0625 * 5.9604644775390625e-8 * static_cast<double>(17 * n_chain + 8);
    constexpr int NE = (NB + 1) / 2;         // experts a lane holds: eg, eg + 64, ... (kNE at most)
    const int eg = lane;
    const int kk_sel = min(k + 1, E);
    float bl[kNE];
#pragma unroll
    for (int i = 0; i < kNE; ++i) bl[i] = i >= NE ? 0.f : (bias != nullptr && eg + 64 * i < E) ? bias[eg + 64 * i] : 0.f;
    const double wn2 = static_cast<double>(wn2_sh);
    for (int tt = wave; tt < TOK; tt += kGateWaves) {
        const int t = t0 + tt;
        if (t >= T) { if (lane == 0) flagged[tt] = 0; continue; }
        // this lane's logits, fp32 (a -0 becomes +0: equal logits must compare equal) and as ordered keys
        float fv[NE];
        unsigned key[NE];
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            const int ei = eg + 64 * i;
            const int ec = ei < E ? ei : 0;                 // lanes without an expert read column 0 and drop it
            float sum = tile_at(0, tt, ec);
            if (kParts > 1) {
#pragma unroll
                for (int pw = 1; pw < kParts; ++pw) sum += tile_at(pw, tt, ec);
            }
            fv[i] = ei < E ? (sum + bl[i]) + 0.0f : 0.f;
            key[i] = ei < E ? order_key(fv[i]) : 0u;
        }
        double lv[kNE], ll[kNE];                 // (value, low part); entries from NE on belong to no expert and are never looked at
#pragma unroll
        for (int i = 0; i < kNE; ++i) { lv[i] = i < NE ? static_cast<double>(fv[i < NE ? i : 0]) : 0.0; ll[i] = 0.0; }
        double sv[kSel];
        int se[kSel];
        int code = 0;
        double gap, vmax;
        if (hash) {
            sign_bits(lv, ll, eg, true, E, code, gap, vmax);
        } else {
            // rank by rank: the largest key of the wave, then the lowest expert that has it
            unsigned taken = 0;
#pragma unroll
            for (int r = 0; r < kSel; ++r) {
                if (r < kk_sel) {
                    unsigned bk = 0u, be = 0xffffffffu;
#pragma unroll
                    for (int i = 0; i < NE; ++i)
                        if (eg + 64 * i < E && !((taken >> i) & 1u) && key[i] > bk) { bk = key[i]; be = static_cast<unsigned>(eg + 64 * i); }
                    const unsigned top = wave_max_u32(bk);
                    const unsigned who = wave_min_u32(bk == top ? be : 0xffffffffu);
                    sv[r] = static_cast<double>(from_order_key(top));
                    se[r] = static_cast<int>(who);
                    if ((who & 63u) == static_cast<unsigned>(eg)) taken |= 1u << (who >> 6);
                }
            }
            rank_gaps(sv, kk_sel, gap, vmax);
        }
        float xn2f = xsq_w[0][tt];
        for (int wv = 1; wv < kGateWaves; ++wv) xn2f += xsq_w[wv][tt];
        const double xn2 = static_cast<double>(xn2f);
        const double delta = gamma * sqrt(xn2 * wn2) + 1.0625 * 5.9604644775390625e-8 * vmax;
        const bool close = gap <= 2.0 * delta;
        if (!close) {
            if (lane == 0) flagged[tt] = 0;
            if (hash) {
                if (lane == 0) { idx[t] = code; w[t] = 1.f; }
            } else {
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
                    float part_sum = 0.f;
#pragma unroll
                    for (int i = 0; i < NE; ++i)
                        if (eg + 64 * i < E) part_sum += expf(static_cast<float>(lv[i] - sv[0]));
                    denom = wave_sum_f32(part_sum);
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
            continue;
        }
        // Too close to call in fp32.  Which columns can exact arithmetic still change the answer for?
        // Top-k: every logit within 2 delta of the (k+1)-th best, or above it (anything lower stays below
        // all of those even with both errors against it).  Sign bits: every projection within 2 delta of
        // zero.  Usually two or three columns: each is one exact dot product by this wave; the other
        // columns keep their fp32 values, which cannot reach the selected ones.
        const double reach = hash ? 2.0 * delta : sv[kk_sel - 1] - 2.0 * delta;
        unsigned long long in_reach[NE];
        int count = 0;
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            in_reach[i] = __ballot(eg + 64 * i < E && (hash ? fabs(lv[i]) <= reach : lv[i] >= reach));
            count += __popcll(in_reach[i]);
        }
        if (lane == 0) flagged[tt] = count > kMaxCand ? 1 : 0;
        if (count > kMaxCand) continue;                                  // all columns, by the whole block, below
        // the columns in reach from exact products: in fp64 first, and once more in twice that precision if that
        // still leaves the decision inside the rounding error (in practice: exact ties)
        auto evaluate = [&](auto pair) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < NE; ++i) {
                unsigned long long m = in_reach[i];
                while (m != 0ull) {                                      // uniform for the wave
                    const int l = __ffsll(static_cast<long long>(m)) - 1;
                    m &= m - 1ull;
                    double hi, lo;
                    exact_column_dot<decltype(pair)::value>(x, pack, static_cast<size_t>(t), l + 64 * i, nS, d, lane, hi, lo);
                    if (eg == l) {
                        dd_add(hi, lo, static_cast<double>(bl[i]), 0.0);
                        dd_normalise(hi, lo);
                        lv[i] = hi;
                        ll[i] = decltype(pair)::value ? lo : 0.0;
                    }
                }
            }
            if (hash) {
                sign_bits(lv, ll, eg, true, E, code, gap, vmax);
            } else {
                wave_topk(lv, ll, eg, true, E, kk_sel, sv, se);
                rank_gaps(sv, kk_sel, gap, vmax);
            }
        };
        evaluate(std::false_type{});
        const double delta64 = 1.0625 * 1.1102230246251565e-16 * (static_cast<double>(d + 8) * sqrt(xn2 * wn2) + 2.0 * vmax);
        if (gap <= 2.0 * delta64) evaluate(std::true_type{});
        if (hash) {
            if (lane == 0) { idx[t] = code; w[t] = 1.f; }
        } else {
            emit_token(lv, sv, se, eg, true, E, k, renorm, lane, idx + static_cast<size_t>(t) * k, w + static_cast<size_t>(t) * k);
        }
    }
    __syncthreads();

    // ---- tokens with more columns in reach than that: all columns in fp64, by the whole block, from the
    // same packed fragments and with the same split as the MFMA pass: wave w takes the groups
    // S = w, w+8, ..., lane (c, h) the 32 rows 64 S + 32 h .. of column c of every expert block; the two
    // halves are added by a lane exchange, the waves in wave order.
    unsigned long long todo = __ballot(lane < TOK && flagged[lane & (TOK - 1)] != 0);   // the same in every wave
    while (todo != 0ull) {
        const int tt = __ffsll(static_cast<long long>(todo)) - 1;
        todo &= todo - 1ull;
        const int t = t0 + tt;
        const uint4* xr = reinterpret_cast<const uint4*>(x + static_cast<size_t>(t) * d + 32 * (lane >> 5));
        double a64[NB], l64[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) { a64[nb] = 0.0; l64[nb] = 0.0; }
        for (int S = wave; S < nS; S += kGateWaves) {
            uint4 xa[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) xa[q] = xr[S * 8 + q];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const uint4* bp = pack + ((static_cast<size_t>(nb) * nS + S) * 4) * 64 + lane;
                uint4 wb[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) wb[q] = bp[q * 64];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t xu[4] = {xa[q].x, xa[q].y, xa[q].z, xa[q].w};
                    const uint32_t wu[4] = {wb[q].x, wb[q].y, wb[q].z, wb[q].w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        dd_add_product(a64[nb], l64[nb], static_cast<double>(__uint_as_float(xu[i] << 16)),
                                       static_cast<double>(__uint_as_float(wu[i] << 16)));
                        dd_add_product(a64[nb], l64[nb], static_cast<double>(__uint_as_float(xu[i] & 0xffff0000u)),
                                       static_cast<double>(__uint_as_float(wu[i] & 0xffff0000u)));
                    }
                }
            }
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const double oh = __shfl_xor(a64[nb], 32), ol = __shfl_xor(l64[nb], 32);
            dd_add(a64[nb], l64[nb], oh, ol);
            if (lane < 32) { resc[wave][32 * nb + lane] = a64[nb]; resc_lo[wave][32 * nb + lane] = l64[nb]; }
        }
        __syncthreads();
        if (wave == 0) {
            double lv[kNE], ll[kNE];
#pragma unroll
            for (int i = 0; i < kNE; ++i) {
                const int ei = eg + 64 * i;
                double sum = 0.0, low = 0.0;
                if (ei < E) {
                    for (int wv = 0; wv < kGateWaves; ++wv) dd_add(sum, low, resc[wv][ei], resc_lo[wv][ei]);
                    dd_add(sum, low, static_cast<double>(bl[i]), 0.0);
                    dd_normalise(sum, low);
                }
                lv[i] = sum;
                ll[i] = low;
            }
            if (hash) {
                int code;
                double gap, vmax;
                sign_bits(lv, ll, eg, true, E, code, gap, vmax);
                if (lane == 0) { idx[t] = code; w[t] = 1.f; }
            } else {
                double sv[kSel];
                int se[kSel];
                wave_topk(lv, ll, eg, true, E, kk_sel, sv, se);
                emit_token(lv, sv, se, eg, true, E, k, renorm, lane, idx + static_cast<size_t>(t) * k, w + static_cast<size_t>(t) * k);
            }
        }
        __syncthreads();
    }
}

}  // namespace

int gate_columns(const moe_cfg& c) {
    if (c.gate != MOE_GATE_HASH) return c.E;
    int bits = 0;
    while ((1 << bits) < c.E) ++bits;
    return bits;
}

size_t route_scratch_bytes(const moe_cfg& c) {
    if (c.dtype != MOE_BF16) return 0;
    const size_t EP = static_cast<size_t>((gate_columns(c) + 31) / 32) * 32;
    return align256(EP * c.d * 2) + align256(static_cast<size_t>(c.d / 64) * EP * 4);
}

size_t gate_packed_bytes(const moe_cfg& c) {
    if (c.dtype == MOE_BF16) return route_scratch_bytes(c);
    return align256(static_cast<size_t>(c.d) * gate_columns(c) * 4);
}

// The gate in the form the gate kernel reads: bf16, fragments in MFMA operand order followed by the sums of
// squares of every 64-row group of every column; fp32, the matrix itself.
int launch_pack_gate(const moe_cfg& c, const void* Wg, void* packed, hipStream_t s) {
    const int cols = gate_columns(c);
    if (c.dtype == MOE_BF16) {
        const int NB = (cols + 31) / 32;
        const size_t EP = static_cast<size_t>(NB) * 32;
        float* part = reinterpret_cast<float*>(static_cast<char*>(packed) + align256(EP * c.d * 2));
        hipLaunchKernelGGL(gate_prep_kernel, dim3(c.d / 64), dim3(256), 0, s, static_cast<const uint16_t*>(Wg), c.d, cols, NB,
                           static_cast<uint4*>(packed), part);
        MOE_LAUNCH_CHECK("gate_prep_kernel");
        return MOE_OK;
    }
    MOE_HIP_CHECK(hipMemcpyAsync(packed, Wg, static_cast<size_t>(c.d) * cols * 4, hipMemcpyDeviceToDevice, s));
    return MOE_OK;
}

int launch_route(const moe_cfg& c, const void* x, const void* Wg, const float* bias, int32_t* idx, float* w,
                 void* scratch, hipStream_t s) {
    if (c.T == 0) return MOE_OK;
    const int hash = c.gate == MOE_GATE_HASH ? 1 : 0;
    const int cols = gate_columns(c);          // columns of the gate matrix: experts, or sign bits
    if (c.dtype == MOE_BF16) {
        const int NB = (cols + 31) / 32;
        const size_t EP = static_cast<size_t>(NB) * 32;
        // a gate packed once by the caller (it is frozen: Section 2.3) is read where it lies; else it is packed
        // into the workspace first, by every call
        if (!c.gate_packed)
            if (int rc = launch_pack_gate(c, Wg, scratch, s)) return rc;
        const char* gate = static_cast<const char*>(c.gate_packed ? Wg : scratch);
        const uint4* pack = reinterpret_cast<const uint4*>(gate);
        const float* part = reinterpret_cast<const float*>(gate + align256(EP * c.d * 2));
        int dev = 0;
        const DeviceInfo* info = nullptr;
        if (int rc = device_info(&dev, &info)) return rc;
        const int n_cu = info->compute_units;
        // as many tokens per block as still give every compute unit a block
        const int tok = (c.T + 31) / 32 >= n_cu ? 32 : (c.T + 15) / 16 >= n_cu ? 16 : 8;
        dim3 grid((c.T + tok - 1) / tok), block(kGateWaves * 64);
#define MOE_ROUTE_LAUNCH(N, TK)                                                                                       \
    {                                                                                                                 \
        /* the tiles of more than 32 experts exceed the default LDS limit of a launch: raised once per device and   \
           kernel (a bit per device; two threads that both find it clear both raise it, which is harmless) */       \
        static std::atomic<uint64_t> raised{0};                                                                       \
        const uint64_t bit = uint64_t(1) << (dev & 63);                                                               \
        if (gate_tile_bytes<N>() > 48 * 1024 && (dev >= 64 || !(raised.load(std::memory_order_acquire) & bit))) {     \
            MOE_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&route_mfma_kernel<N, TK>),               \
                                              hipFuncAttributeMaxDynamicSharedMemorySize,                             \
                                              static_cast<int>(gate_tile_bytes<N>())));                               \
            if (dev < 64) raised.fetch_or(bit, std::memory_order_release);                                            \
        }                                                                                                             \
        hipLaunchKernelGGL((route_mfma_kernel<N, TK>), grid, block, gate_tile_bytes<N>(), s,                          \
                           static_cast<const uint16_t*>(x), pack, part, bias, idx, w, c.T, c.d, cols, c.k, c.renorm,  \
                           hash);                                                                                     \
    }
#define MOE_ROUTE_CASE(N)                                                                                             \
    case N:                                                                                                           \
        if (tok == 32) MOE_ROUTE_LAUNCH(N, 32) else if (tok == 16) MOE_ROUTE_LAUNCH(N, 16) else MOE_ROUTE_LAUNCH(N, 8) \
        break;
        switch (NB) {
            MOE_ROUTE_CASE(1) MOE_ROUTE_CASE(2) MOE_ROUTE_CASE(3) MOE_ROUTE_CASE(4)
            MOE_ROUTE_CASE(5) MOE_ROUTE_CASE(6) MOE_ROUTE_CASE(7) MOE_ROUTE_CASE(8)
            default: return fail(MOE_ERR_UNSUPPORTED, "E = %d is out of range", c.E);
        }
#undef MOE_ROUTE_LAUNCH
#undef MOE_ROUTE_CASE
        MOE_LAUNCH_CHECK("route_mfma_kernel");
        return MOE_OK;
    }
    const int per_block = kWaves * kTPW;
    dim3 grid((c.T + per_block - 1) / per_block), block(kWaves * 64);
    hipLaunchKernelGGL(route_kernel<float>, grid, block, 0, s, static_cast<const float*>(x),
                       static_cast<const float*>(Wg), bias, idx, w, c.T, c.d, cols, c.k, c.renorm, hash);
    MOE_LAUNCH_CHECK("route_kernel");
    return MOE_OK;
}

}  // namespace moe
