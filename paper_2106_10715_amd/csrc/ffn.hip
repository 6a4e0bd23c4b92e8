// Expert feed-forward networks on the rows batched by expert (CPM-2 Section 2.1 / Table 1: each
// expert is a d_model -> d_ff -> d_model gated-GELU FFN; Section 6.2: an expert's work is
// proportional to its token count and its parameters form one equal-sized block):
//
//     H  = act(Xp W_gate[e]) * (Xp W_in[e])        "up"   grouped GEMM, epilogue fused
//     Yp = H W_out[e]                               "down" grouped GEMM
//
// bf16 path: 32x32x16 bf16 MFMA, fp32 accumulate.  One block = up to 256 rows of one expert x 4 waves;
// every wave owns its own output columns for all rows, so a weight fragment is needed by exactly
// one wave: weights go HBM -> registers directly in pre-packed fragment order (no LDS, fully
// coalesced 1 KiB reads), only the activation tile is shared through LDS (padded rows,
// conflict-free 16-byte reads and writes).  With few rows per expert the layer is bound by streaming the
// weights once from HBM, which is what this layout is built for.
// fp32 path: plain LDS-tiled FMA kernel (small-shape correctness vehicle).
#include "common.h"
#include "ffn_plan.h"

#include <type_traits>

namespace moe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kKC = 64;                 // reduction elements staged per pipeline step (4 MFMA k-steps)
// Rows of a tile when the up-projection gathers its rows itself: a thread then holds one source offset per
// 32-row block, which the registers allow up to seven blocks (eight accumulator blocks leave no room).
constexpr int kGatherTileM = 224;

__device__ inline float act_fn(float z, int act) {
    if (act == 0) return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
    const float u = 0.79788456080286536f * (z + 0.044715f * z * z * z);
    return 0.5f * z * (1.0f + tanhf(u));
}

// Exact GELU for results that are rounded to bf16 right away, written on the lower tail of the normal
// distribution: with q(a) = 0.5 erfc(a / sqrt 2), GELU(z) = z Phi(z) = max(z, 0) - |z| q(|z|), which has no
// cancellation for negative z.  log2 q is smooth, so q = exp2(P(a)) with P a polynomial of degree 6,
// fitted on [0, 8] with the error weighted by a q(a) (so that the absolute error of GELU is level):
// |error| <= 1e-7 on GELU in fp32 arithmetic, four orders below the bf16 rounding of the result, in six
// fused multiply-adds and one hardware exponential instead of the several times longer library erff.
// Beyond 8, q < 1e-15 and the argument is clamped (by a comparison that lets a NaN through).
constexpr float kGeluTail[7] = {-0.999993085861206f,   -1.1512017250061035f,   -0.4587709605693817f, -0.05341210961341858f,
                                0.008080719038844109f, -0.0007692205253988504f, 3.309290696051903e-05f};
__device__ inline float act_fn_bf16(float z, int act) {
    if (act != 0) return act_fn(z, act);
    const float a = fabsf(z);
    const float ac = a > 8.0f ? 8.0f : a;
    float p = kGeluTail[6];
#pragma unroll
    for (int i = 5; i >= 0; --i) p = fmaf(p, ac, kGeluTail[i]);
    float relu;                                  // one instruction: fmaxf would first quiet a signalling NaN, and a NaN comes through ac anyway
    asm("v_max_f32 %0, 0, %1" : "=v"(relu) : "v"(z));
    return fmaf(-ac, __builtin_amdgcn_exp2f(p), relu);
}

// Which (expert, row tile) a block works on: tile slot `slot` counted over the experts
// [e_first, e_first + e_count) in order, at most tile_m rows per tile.  Returns false when the slot is past
// the last tile (uniform for the block).  Must be called by all threads of the block.
__device__ inline bool find_tile(const int32_t* __restrict__ offsets, int e_first, int e_count, int tile_m, int slot,
                                 int total_rows, int& e_out, int& row_begin, int& rows) {
    // segment of expert e, clamped so that whatever the offsets hold no tile reaches outside the rows there are
    auto seg_lo = [&](int e) { return min(max(offsets[e], 0), total_rows); };
    auto seg_hi = [&](int e) { return min(max(offsets[e + 1], seg_lo(e)), total_rows); };
    __shared__ int sh_e, sh_mt;
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        int tl[4], sum = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = lane * 4 + q;
            const int cnt = e < e_count ? seg_hi(e_first + e) - seg_lo(e_first + e) : 0;
            tl[q] = (cnt + tile_m - 1) / tile_m;
            sum += tl[q];
        }
        int incl = sum;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int v = __shfl_up(incl, off);
            if (lane >= off) incl += v;
        }
        const int target = slot;
        int run = incl - sum;
        if (target >= run && target < incl) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (target >= run && target < run + tl[q]) { sh_e = lane * 4 + q; sh_mt = target - run; }
                run += tl[q];
            }
        }
        const int total = __shfl(incl, 63);
        if (lane == 0 && target >= total) sh_e = -1;
    }
    __syncthreads();
    if (sh_e < 0) return false;
    e_out = e_first + sh_e;
    // the expert's rows are split evenly over its tiles (in multiples of 32 rows), not into full tiles
    // and a small remainder: equal tiles finish together and none is nearly empty
    const int lo = seg_lo(e_out), hi = seg_hi(e_out), n = hi - lo;
    const int tiles = (n + tile_m - 1) / tile_m;
    const int per_tile = min(tile_m, ((n + tiles - 1) / tiles + 31) & ~31);
    row_begin = lo + sh_mt * per_tile;
    rows = min(per_tile, hi - row_begin);
    return true;
}

// ------------------------------------------------------------------------------------------ packing

// One thread per 16-byte lane slot of a fragment: element 8 l + j of fragment (n, s) is
// W[16 s + 8 (l / 32) + j, col(n) + l % 32].
__global__ __launch_bounds__(256) void pack_bf16_kernel(const uint16_t* __restrict__ Win, const uint16_t* __restrict__ Wgate,
                                                        const uint16_t* __restrict__ Wout, uint4* __restrict__ packed,
                                                        int d, int f) {
    const long up_frags = static_cast<long>(f / 32) * (d / 16) * 2;
    const long down_frags = static_cast<long>(d / 64) * (f / 16) * 2;
    const long gid = static_cast<long>(blockIdx.x) * 256 + threadIdx.x;
    const long F = gid >> 6;
    const int l = static_cast<int>(gid & 63);
    if (F >= up_frags + down_frags) return;
    const uint16_t* src;
    int ld, row0, col;
    if (F < up_frags) {
        const long per_n = 2L * (d / 16);
        const int n = static_cast<int>(F / per_n);
        const int rem = static_cast<int>(F % per_n);
        src = (rem & 1) ? Win : Wgate;
        ld = f;
        row0 = 16 * (rem >> 1) + 8 * (l >> 5);
        col = 32 * n + (l & 31);
    } else {
        const long G = F - up_frags;
        const long per_p = 2L * (f / 16);
        const int p = static_cast<int>(G / per_p);
        const int rem = static_cast<int>(G % per_p);
        src = Wout;
        ld = d;
        row0 = 16 * (rem >> 1) + 8 * (l >> 5);
        col = 64 * p + 32 * (rem & 1) + (l & 31);
    }
    uint16_t v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = src[static_cast<size_t>(row0 + j) * ld + col];
    uint4 o;
    o.x = v[0] | (static_cast<uint32_t>(v[1]) << 16);
    o.y = v[2] | (static_cast<uint32_t>(v[3]) << 16);
    o.z = v[4] | (static_cast<uint32_t>(v[5]) << 16);
    o.w = v[6] | (static_cast<uint32_t>(v[7]) << 16);
    packed[F * 64 + l] = o;
}

// ------------------------------------------------------------------------------------------ bf16 MFMA
//
// Software pipeline of one block (4 waves, up to 256 rows of one expert, 64 reduction elements per
// step).  In step c every thread
//     issues its share of the activation tile of step c+1            (global -> registers)
//     issues its wave's weight fragments of step c+2                 (global -> registers, ring of 3)
//     runs the MFMAs of step c (weights from the ring, activations from LDS buffer c%2, the LDS
//         reads of k-step s+1 overlapping the MFMAs of k-step s)
//     waits for the activation registers, stores them to LDS buffer (c+1)%2, barrier.
// The compiler would sink all those loads down to their first use and wait there, which serialises
// the pipeline, and it removes prefetches whose result is never read, which changes how many loads
// are in flight.  So every global load of the loop is issued from inline assembly (pinned in program
// order, never removed) and the one wait per step is written by hand: vector memory loads return in
// order, hence "at most 4*NF loads outstanding" at the end of step c means everything but the weight
// fragments issued in this very step has arrived -- the activations of step c+1 and, being older, the
// weights of step c+1.  The wait names those registers as read-write operands so that no use of them
// can be moved above it.

constexpr int kKS = kKC / 16;           // MFMA k-steps per pipeline step
constexpr int kLdsRow = 9;              // uint4 per activation row in LDS: 128 B of data + 16 B pad (conflict-free)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int NF>
struct BFrags { u32x4 v[kKS][NF]; };    // one pipeline step of one wave: 4 k-steps x NF fragments
template <int MBS>
struct ARegs { u32x4 v[MBS]; };         // this thread's share of one activation tile step

__device__ inline bf16x8 as_bf16x8(const u32x4& u) { return __builtin_bit_cast(bf16x8, u); }
__device__ inline bf16x8 as_bf16x8(const uint4& u) { return __builtin_bit_cast(bf16x8, u); }

// 16-byte load from (uniform base + per-lane byte offset + immediate), pinned in program order.
template <int IMM>
__device__ inline void ld_pinned(u32x4& dst, uint32_t voff, const void* sbase) {
    asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=v"(dst) : "v"(voff), "s"(sbase), "n"(IMM) : "memory");
}
// The weight loads.  An expert with one row tile reads its weights once: marked non-temporal they do
// not push the activation tiles (which every column group of the expert re-reads) out of the L2, and the
// stream itself runs faster (a plain read stream of this shape reaches 6.2 TB/s, a non-temporal one 7.1).
// An expert with several row tiles re-reads its weights once per tile: there the plain load, which leaves them
// in the L2 for the tiles that follow, is the faster one (KEEP).
template <int IMM, bool KEEP>
__device__ inline void ld_pinned_stream(u32x4& dst, uint32_t voff, const void* sbase) {
    if constexpr (KEEP)
        asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=v"(dst) : "v"(voff), "s"(sbase), "n"(IMM) : "memory");
    else
        asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3 nt" : "=v"(dst) : "v"(voff), "s"(sbase), "n"(IMM) : "memory");
}

// The two fragments of one (column unit, k-step) are adjacent in the packed block:
// [k-step][2][64 lanes] x 16 bytes (2 KiB per k-step); a wave with NF = 1 reads one of the two.
// voff = byte offset of this lane inside its wave's stream at the first k-step of the pipeline step.
template <bool KEEP, int NF>
__device__ inline void load_b(BFrags<NF>& b, uint32_t voff, const void* wave_base) {
    ld_pinned_stream<0, KEEP>(b.v[0][0], voff, wave_base);
    if (NF == 2) ld_pinned_stream<1024, KEEP>(b.v[0][NF - 1], voff, wave_base);
    ld_pinned_stream<2048, KEEP>(b.v[1][0], voff, wave_base);
    if (NF == 2) ld_pinned_stream<3072, KEEP>(b.v[1][NF - 1], voff, wave_base);
    const uint32_t voff2 = voff + 4096;
    ld_pinned_stream<0, KEEP>(b.v[2][0], voff2, wave_base);
    if (NF == 2) ld_pinned_stream<1024, KEEP>(b.v[2][NF - 1], voff2, wave_base);
    ld_pinned_stream<2048, KEEP>(b.v[3][0], voff2, wave_base);
    if (NF == 2) ld_pinned_stream<3072, KEEP>(b.v[3][NF - 1], voff2, wave_base);
}

// Wait until at most N_YOUNGER loads are outstanding; the registers named become usable afterwards.
template <int N_YOUNGER, int NF, int MBS>
__device__ inline void wait_loads(ARegs<MBS>& a, BFrags<NF>& b) {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N_YOUNGER) : "memory");
#pragma unroll
    for (int mb = 0; mb < MBS; ++mb) asm volatile("" : "+v"(a.v[mb]));
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks)
#pragma unroll
        for (int j = 0; j < NF; ++j) asm volatile("" : "+v"(b.v[ks][j]));
}
// The activation tile lives in LDS row-major, one padded row of kLdsRow uint4 per tile row.
// Staging: thread t moves, for i < MBS, the 16-byte piece (row i*32 + t/8, piece t%8): eight
// neighbouring lanes fetch one whole 128-byte line of a row, and write 128 contiguous bytes of LDS.
template <int MBS>
__device__ inline void store_a(const ARegs<MBS>& a, uint4* lds_buf, unsigned tid) {
    u32x4* p = reinterpret_cast<u32x4*>(lds_buf) + (tid >> 3) * kLdsRow + (tid & 7);
#pragma unroll
    for (int mb = 0; mb < MBS; ++mb) p[mb * 32 * kLdsRow] = a.v[mb];
}

// The MFMAs of a pipeline step are issued in units: unit u = (k-step u / H, row-block group u % H),
// H = 1 or 2 groups of at most 4 row blocks.  The A fragments of unit u+1 are read from LDS while the
// MFMAs of unit u run; two register buffers of G fragments alternate.
// Fragment (mb, ks) of lane l = row mb*32 + l%32, 8 elements at k = 16 ks + 8 (l / 32).
template <int MBS>
struct Units {
    static constexpr int H = MBS > 4 ? 2 : 1;
    static constexpr int G = (MBS + H - 1) / H;
    static constexpr int U = kKS * H;
};

template <int MBS, int UNIT>
__device__ inline void read_unit(uint4 (&af)[Units<MBS>::G], const uint4* lds_buf, int lane) {
    constexpr int ks = UNIT / Units<MBS>::H, mb0 = (UNIT % Units<MBS>::H) * Units<MBS>::G;
    const uint4* rp = lds_buf + (lane & 31) * kLdsRow + (lane >> 5) + 2 * ks;
#pragma unroll
    for (int i = 0; i < Units<MBS>::G; ++i)
        if (mb0 + i < MBS) af[i] = rp[(mb0 + i) * 32 * kLdsRow];
}

template <int NF, int MBS, int UNIT>
__device__ inline void mma_unit(f32x16 (&acc)[MBS][NF], const uint4 (&af)[Units<MBS>::G], const BFrags<NF>& b) {
    constexpr int ks = UNIT / Units<MBS>::H, mb0 = (UNIT % Units<MBS>::H) * Units<MBS>::G;
#pragma unroll
    for (int i = 0; i < Units<MBS>::G; ++i) {
        if (mb0 + i < MBS) {
#pragma unroll
            for (int j = 0; j < NF; ++j)
                acc[mb0 + i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(b.v[ks][j]), as_bf16x8(af[i]),
                                                                          acc[mb0 + i][j], 0, 0, 0);
        }
    }
}

template <int LO, int HI, class F>
__device__ inline void static_for(F&& f) {
    if constexpr (LO < HI) {
        f(std::integral_constant<int, LO>{});
        static_for<LO + 1, HI>(f);
    }
}

// Everything a pipeline step does besides its MFMAs is spread over them, one instruction after each
// MFMA: a load or an LDS access holds the wave's issue slot for some 16 cycles and the matrix pipe
// has only one instruction queued, so a run of them lets it run dry, and a wait that directly follows
// the LDS writes of the whole tile stalls the wave for their full latency.
// Loads (or LDS writes) done after the units 0..u of a step that spreads n of them evenly over U units:
constexpr int loads_upto(int u, int n, int U) { return u < 0 ? 0 : ((u + 1) * n + U - 1) / U < n ? ((u + 1) * n + U - 1) / U : n; }
// The staging writes (one per row block) go into the units before the last one, which holds the barrier:
// spread evenly, except that one or two row blocks are staged as late as that allows.  Their steps are so
// short (one or two MFMAs per unit) that the step time is the time their activation loads take to arrive,
// and every unit the write waits is lead for the load.
constexpr int writes_upto(int u, int n, int U) {
    if (n <= 2) {
        const int done = u - (U - 1 - n) + 1;
        return done < 0 ? 0 : (done > n ? n : done);
    }
    return loads_upto(u, n, U - 1);
}
constexpr int unit_of_write(int w, int n, int U) {
    int u = 0;
    while (writes_upto(u, n, U) <= w) ++u;
    return u;
}
// Global loads a step has issued before those of unit u: one activation load per unit while there are
// row blocks left, then the unit's share of the nb weight loads.
constexpr int issued_before(int u, int MBS, int nb, int U) { return (u < MBS ? u : MBS) + loads_upto(u - 1, nb, U); }
// Loads younger than the activation load of row block w at the moment the next step stages that block:
// what the issuing step issued after it, and what the staging step has issued before the unit that
// stages it.  Loads return in order, so waiting until at most this many are outstanding means the block
// (and every weight load older than it) has landed.
constexpr int younger_at_write(int w, int MBS, int nb, int U) {
    return (MBS + nb - issued_before(w, MBS, nb, U) - 1) + issued_before(unit_of_write(w, MBS, U), MBS, nb, U);
}

template <int MBS>
constexpr int unit_rows(int u) {
    const int left = MBS - (u % Units<MBS>::H) * Units<MBS>::G;
    return left > Units<MBS>::G ? Units<MBS>::G : (left < 0 ? 0 : left);
}
// fragment I of unit UNIT, from the activation tile in lds_buf
template <int MBS, int UNIT, int I>
__device__ inline void read_frag(uint4 (&af)[Units<MBS>::G], const uint4* lds_buf, int lane) {
    constexpr int ks = UNIT / Units<MBS>::H, mb = (UNIT % Units<MBS>::H) * Units<MBS>::G + I;
    af[I] = lds_buf[(lane & 31) * kLdsRow + (lane >> 5) + 2 * ks + mb * 32 * kLdsRow];
}
// MFMA M of unit UNIT: row block M / NF of the unit, weight fragment M % NF
template <int NF, int MBS, int UNIT, int M>
__device__ inline void mma_one(f32x16 (&acc)[MBS][NF], const uint4 (&af)[Units<MBS>::G], const BFrags<NF>& b) {
    constexpr int ks = UNIT / Units<MBS>::H, i = M / NF, j = M % NF, mb = (UNIT % Units<MBS>::H) * Units<MBS>::G + i;
    acc[mb][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(b.v[ks][j]), as_bf16x8(af[i]), acc[mb][j], 0, 0, 0);
}
// Row block mb of the staged activations has landed once at most N_YOUNGER loads are outstanding; it goes
// into the LDS tile (thread t holds the 16-byte piece t%8 of row mb*32 + t/8).
template <int N_YOUNGER>
__device__ inline void stage_block(u32x4& v, uint4* lds_buf, unsigned tid, int mb) {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N_YOUNGER) : "memory");
    asm volatile("" : "+v"(v));
    reinterpret_cast<u32x4*>(lds_buf)[(tid >> 3) * kLdsRow + (tid & 7) + mb * 32 * kLdsRow] = v;
}

// One pipeline step.  Entering, af[0] holds the fragments of unit 0 of this step; leaving, those of
// unit 0 of the next step.
//   cur, nxt : LDS buffers of this and of the next step
//   b        : weight fragments of this step
//   a_next, b_next : registers of the next step's activations and weights (loads in flight)
//   issue_a  : issue_a(integral_constant mb) issues the activation load of row block mb this step prefetches
//   issue_b  : issue_b(integral_constant i) issues load i of the kKS * NF weight loads this step prefetches
// After MFMA s of a unit comes its s-th other instruction, in this order: the LDS reads of the next
// unit's fragments, the staging of the row blocks that fall to this unit (each behind its own wait), the
// unit's activation load, its weight loads.  The last unit holds the barrier after its second MFMA: all
// fragments of this step were requested a unit earlier and nxt was completed a unit earlier, so the wait
// in front of the barrier finds nothing outstanding, and the first fragments of the next step are read
// from nxt under the remaining MFMAs.  nxt may be written from the start of the step: its last readers
// passed the barrier of the step before.
template <int NF, int MBS, class IssueA, class IssueB>
__device__ inline void run_step(f32x16 (&acc)[MBS][NF], uint4 (&af)[2][Units<MBS>::G], const uint4* cur, uint4* nxt,
                                const BFrags<NF>& b, ARegs<MBS>& a_next, BFrags<NF>& b_next, int lane, unsigned tid,
                                IssueA issue_a, IssueB issue_b) {
    constexpr int U = Units<MBS>::U, kB = kKS * NF;
    static_for<0, U>([&](auto uc) {
        constexpr int UU = decltype(uc)::value;
        constexpr bool kLast = UU + 1 == U;
        constexpr int M = unit_rows<MBS>(UU) * NF;                 // MFMAs of this unit
        constexpr int NU = kLast ? 0 : UU + 1;                     // the unit whose fragments are fetched meanwhile
        constexpr int nR = unit_rows<MBS>(NU);
        constexpr int w0 = kLast ? MBS : writes_upto(UU - 1, MBS, U), nW = (kLast ? MBS : writes_upto(UU, MBS, U)) - w0;
        constexpr int nA = UU < MBS ? 1 : 0;
        constexpr int b0 = loads_upto(UU - 1, kB, U), nB = loads_upto(UU, kB, U) - b0;
        constexpr int nOther = nR + nW + nA + nB;
        constexpr int kFirst = kLast && M > 1 ? 1 : 0;             // other instruction s follows MFMA kFirst + s
        auto other = [&](auto sc) {
            constexpr int s = decltype(sc)::value;
            if constexpr (s < nR) {
                read_frag<MBS, NU, s>(af[NU & 1], kLast ? nxt : cur, lane);
            } else if constexpr (s < nR + nW) {
                constexpr int w = w0 + s - nR;
                stage_block<younger_at_write(w, MBS, kB, U)>(a_next.v[w], nxt, tid, w);
                if constexpr (w == 0) {                            // the weights of the next step are older than its activations
#pragma unroll
                    for (int ks = 0; ks < kKS; ++ks)
#pragma unroll
                        for (int j = 0; j < NF; ++j) asm volatile("" : "+v"(b_next.v[ks][j]));
                }
            } else if constexpr (s < nR + nW + nA) {
                issue_a(std::integral_constant<int, UU + 0 * s>{});     // (made dependent on s: only instantiated when taken)
            } else {
                issue_b(std::integral_constant<int, b0 + s - nR - nW - nA>{});
            }
        };
        static_for<0, M>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            mma_one<NF, MBS, UU, m>(acc, af[UU & 1], b);
            if constexpr (kLast && m == kFirst) __syncthreads();
            if constexpr (m >= kFirst) {
                constexpr int lo = m - kFirst;
                constexpr int hi = m == M - 1 ? nOther : (lo + 1 < nOther ? lo + 1 : nOther);
                static_for<lo, hi>(other);
            }
        });
    });
}

// A step without any overlap, for the few steps that do not fill a group of the unrolled pipeline:
// fetch, wait, stage, compute.  Uses LDS buffer 0 and the registers passed in; nothing stays in flight.
template <int NF, int MBS>
__device__ inline void slow_step(f32x16 (&acc)[MBS][NF], uint4 (&af)[2][Units<MBS>::G], uint4* buf, ARegs<MBS>& a,
                                 BFrags<NF>& b, int lane, unsigned tid) {
    wait_loads<0>(a, b);
    __syncthreads();                            // nobody reads buf any more
    store_a(a, buf, tid);
    __syncthreads();
#define FFN_UNIT(UU)                                                          \
    if constexpr ((UU) < Units<MBS>::U) {                                     \
        read_unit<MBS, (UU)>(af[0], buf, lane);                               \
        mma_unit<NF, MBS, (UU)>(acc, af[0], b);                               \
    }
    FFN_UNIT(0) FFN_UNIT(1) FFN_UNIT(2) FFN_UNIT(3) FFN_UNIT(4) FFN_UNIT(5) FFN_UNIT(6) FFN_UNIT(7)
#undef FFN_UNIT
}

// The id of this thread inside its block, rebuilt from the wave number (which sits in a scalar
// register) and the lane number, by instructions the compiler can neither hoist nor keep alive: a
// vector register that holds the id across the main loop is one the loop does not have.
__device__ inline unsigned thread_id(int wave) {
    unsigned lane;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane));
    return static_cast<unsigned>(wave) * 64u + lane;
}

// ---- work items.  A launch's items are positions of 8 queues (one per XCD; see ffn_mfma_kernel); everything a
// block needs to take one and to find out what it means, all of it uniform (scalar registers):
struct ItemQueue {
    unsigned* counters;            // next position of each queue
    unsigned total_q, home;        // positions per queue; this block's own queue
    const int4* tile_list;         // (expert, first row, rows, row tiles of the expert) per row tile
    int tiles, y_chunks, mt_shift;
    const char* W;                 // packed weights of expert e_first (+ block_offset_bytes: the up or the down block)
    size_t expert_stride_bytes, block_offset_bytes;
    int e_first;
};
struct Item {
    bool real;                     // false: padding of the queue (past the last tile or column group)
    int e, row_begin, rows, tiles_of_expert, block_y;
};

__device__ inline Item decode_item(const ItemQueue& Q, unsigned q, unsigned xcd, int units) {
    const unsigned ny = 32u >> Q.mt_shift;     // column groups per run of 32; 1 << mt_shift row tiles
    const unsigned yg = q & (ny - 1u), mt = (q / ny) & ((1u << Q.mt_shift) - 1u), rest = q >> 5;
    const unsigned y_chunk = rest % static_cast<unsigned>(Q.y_chunks), tile_group = rest / static_cast<unsigned>(Q.y_chunks);
    const int slot = static_cast<int>((((tile_group << 3) + xcd) << Q.mt_shift) + mt);
    Item it;
    it.block_y = static_cast<int>(y_chunk * ny + yg);
    it.real = slot < Q.tiles && it.block_y * 4 < units;
    it.e = it.row_begin = it.rows = it.tiles_of_expert = 0;
    if (it.real) {
        // the same for all lanes, and written by an earlier kernel: read through the scalar cache
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        typedef const __attribute__((address_space(4))) i32x4 constant_i32x4;
        const i32x4 tile = ((constant_i32x4*)Q.tile_list)[slot];
        it.e = __builtin_amdgcn_readfirstlane(tile.x);
        it.row_begin = __builtin_amdgcn_readfirstlane(tile.y);
        it.rows = __builtin_amdgcn_readfirstlane(tile.z);
        it.tiles_of_expert = __builtin_amdgcn_readfirstlane(tile.w);
    }
    return it;
}

// Start of a wave's fragment stream in an item and the key that fixes where its sweep over the reduction dimension
// starts: the sweep starts at a step that depends on the expert and on the chunk of 8 column groups only, so blocks that
// share a weight stream or an activation tile walk it together; neighbouring chunks are one step apart (measured:
// far-apart chunks fetch the activation tile again, chunks in step collide on their weight streams), other experts
// anywhere.  The same for all lanes, so the address is handed over in scalar registers.
template <bool GATED, int NF>
__device__ inline const void* wave_stream(const ItemQueue& Q, int e, int block_y, int wave, int units, int K, unsigned& key) {
    const int unit = block_y * 4 + wave;
    const int u = unit < units ? unit : units - 1;     // a wave past the last unit recomputes the last one, stores nothing
    const int steps16 = K / 16;
    // fragment pair index and which half of the pair this wave reads
    const int pair = (GATED || NF == 2) ? u : (u >> 1);
    const int half = (GATED || NF == 2) ? 0 : (u & 1);
    const char* wb = Q.W + static_cast<size_t>(e - Q.e_first) * Q.expert_stride_bytes + Q.block_offset_bytes +
                     (static_cast<size_t>(pair) * steps16 * 128 + half * 64) * 16;
    const uintptr_t wbi = reinterpret_cast<uintptr_t>(wb);
    const uint32_t wb_lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(wbi))));
    const uint32_t wb_hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(wbi >> 32))));
    const unsigned col_chunk = static_cast<unsigned>(block_y) >> ((GATED || NF == 2) ? 3 : 4);   // same for both unit widths
    key = static_cast<unsigned>(e) * 37u + col_chunk;
    return reinterpret_cast<const void*>((static_cast<uintptr_t>(wb_hi) << 32) | static_cast<uintptr_t>(wb_lo));
}

// Thread 0 takes the next position: first from the block's own queue, and when that is empty from the others.
// The first attempt is split from the rest so that its answer can arrive under other work.
__device__ inline unsigned take_first(const ItemQueue& Q) { return atomicAdd(&Q.counters[Q.home], 1u); }
__device__ inline void take_finish(const ItemQueue& Q, unsigned v, int* sh_q, int* sh_x) {
    int got = -1;
    unsigned x = Q.home;
    if (v < Q.total_q) {
        got = static_cast<int>(v);
    } else {
        for (unsigned i = 1; i < 8u; ++i) {
            x = (Q.home + i) & 7u;
            const unsigned w = atomicAdd(&Q.counters[x], 1u);
            if (w < Q.total_q) { got = static_cast<int>(w); break; }
        }
    }
    *sh_q = got;
    *sh_x = static_cast<int>(x);
}

// One tile of MBS 32-row blocks: the whole reduction loop and the epilogue.
// Loads past the end are clamped to valid addresses (rows to the last row of the tile, pipeline steps
// to the last step) instead of being skipped, so every step issues the same loads.  Rows that are
// clamped duplicates only produce output rows that are never stored (an output row depends on its own
// input row only).
// GATHER: A is not the batched row array but the token array it was gathered from, and row r of the batched
// order is token gather[r] / gather_k of A (the batching of Section 6.2 done on the fly: the batched copy of the
// activations is never written); every thread then keeps one byte offset per row block instead of two in all.
template <bool GATED, int NF, int MBS, bool KEEP, bool GATHER = false>
__device__ inline void ffn_tile(uint4 (&lds)[2][kTileM * kLdsRow], const uint16_t* __restrict__ A, int row_begin, int rows,
                                const void* wave_base, uint16_t* __restrict__ C, int K, int N, int unit,
                                bool active, int act, unsigned phase_key, int wave_s, const int32_t* __restrict__ row_map,
                                const int32_t* __restrict__ gather, int gather_k, const ItemQueue& Q, int units, int* sh_q,
                                int* sh_x, int h_rows) {
    unsigned tid = thread_id(wave_s);
    const int lane = tid & 63;
    // every tile height gets its own copy of the loop bounds: shared ones would be computed once for all
    // heights and stay in registers across this one
    asm volatile("" : "+s"(K), "+s"(N), "+s"(phase_key));
    const int chunks = K / kKC, last = chunks - 1;

    // this thread's activation sources (byte offsets from A): row mb*32 + t/8 of every block, piece t%8.
    // All blocks but the last hold 32 rows, so their rows lie a fixed stride apart; rows past the end
    // of the last block re-read the tile's last row.
    const int r0 = tid >> 3;
    const uint32_t piece = 16u * (tid & 7);
    // Layout of A.  The up-projection reads row-major rows (K elements each).  The down-projection reads the
    // intermediate H, which only these two kernels see and which is therefore kept in the order they touch it:
    // [chunk of 64 columns][row][64 columns], all h_rows rows of a chunk back to back, so that a tile's rows of one
    // chunk are one contiguous run, for the up-projection's stores (scattered 256-byte pieces cost the memory far
    // more than their bytes) as for these loads.
    const uint32_t a_row_bytes = GATED ? static_cast<uint32_t>(K) * 2u : static_cast<uint32_t>(kKC * 2);
    const size_t a_chunk_bytes = GATED ? static_cast<size_t>(kKC * 2) : static_cast<size_t>(h_rows) * (kKC * 2);
    const uint32_t a_first = static_cast<uint32_t>(row_begin + r0) * a_row_bytes + piece;
    const uint32_t a_last = static_cast<uint32_t>(row_begin + min((MBS - 1) * 32 + r0, rows - 1)) * a_row_bytes + piece;
    const uint32_t a_stride = 32u * a_row_bytes;        // 32 rows, in bytes
    uint32_t a_off[GATHER ? MBS : 1];           // GATHER: this thread's source row of every block, as a byte offset from A
    if constexpr (GATHER) {
#pragma unroll
        for (int mb = 0; mb < MBS; ++mb) {
            const int row = row_begin + min(mb * 32 + r0, rows - 1);
            a_off[mb] = static_cast<uint32_t>(gather[row] / gather_k) * K * 2u + piece;
        }
    }

    f32x16 acc[MBS][NF];
    // cleared in place, in the accumulation registers: a zero constant would be parked in 16 registers for all
    // tile heights and copied from there
#pragma unroll
    for (int mb = 0; mb < MBS; ++mb)
#pragma unroll
        for (int j = 0; j < NF; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) asm volatile("v_accvgpr_write_b32 %0, 0" : "=a"(acc[mb][j][v]));

    // Pipeline depth: activations 2 steps ahead (two register sets), weights 3 steps ahead (ring of 4).
    // Step c issues A(c+2) and B(c+3), spread over its MFMA units (after unit u the activation load of row
    // block u, if there is one, and the weight loads of that unit's share), and stages A(c+1), one row
    // block at a time, in the units before its last: row block w was requested by step c-1 in unit w and
    // is waited for about one step later, by the count of loads younger than it (younger_at_write).
    // Everything older, B(c+1) included, has then landed.
    constexpr int AD = 2;
    constexpr int R = AD + 2;                   // weight ring; register indices repeat with period R
    constexpr int kB = kKS * NF;                // loads of one weight step
    constexpr int kU = Units<MBS>::U;
    static_assert(MBS <= kU, "one activation load per unit");
    ARegs<MBS> areg[AD];
    BFrags<NF> ring[R];
    uint4 af[2][Units<MBS>::G];
    // the per-block and per-step parts of the address are uniform: they go into the scalar base, and the
    // per-thread part is the same register for every block but the last
    auto fetch_a = [&](ARegs<MBS>& dst, int chunk) {
        const char* base = reinterpret_cast<const char*>(A) + static_cast<size_t>(chunk) * a_chunk_bytes;
        if constexpr (GATHER) {
#pragma unroll
            for (int mb = 0; mb < MBS; ++mb) ld_pinned<0>(dst.v[mb], a_off[mb], base);
        } else {
#pragma unroll
            for (int mb = 0; mb + 1 < MBS; ++mb) ld_pinned<0>(dst.v[mb], a_first, base + static_cast<size_t>(mb) * a_stride);
            ld_pinned<0>(dst.v[MBS - 1], a_last, base);
        }
    };
    auto fetch_b = [&](BFrags<NF>& dst, int chunk) {
        load_b<KEEP>(dst, static_cast<uint32_t>(chunk) * (kKS * 2048) + lane * 16, wave_base);
    };
    const uint32_t lane_off = lane * 16;
    // Blocks that share a weight stream or an activation tile start their sweep over the reduction
    // dimension at the same step (and wrap around), other blocks at other steps, so that concurrent
    // waves do not all walk their weight streams, which lie a power of two apart, in lockstep.  The
    // phase never depends on the launch shape, so a launch over all experts and a launch over one
    // expert sum in the same order (bitwise equal results).
    const int phase = static_cast<int>(phase_key % static_cast<unsigned>(chunks));
    auto at = [&](int i) { const int c = phase + i; return c >= chunks ? c - chunks : c; };   // i < chunks
    int c = 0;
    if (chunks >= R) {
        asm volatile("; pipeline begin");       // from here to the matching end the build allows no spill code
        // Prologue: A(0) B(0) B(1) A(1) B(2), each as a block; then wait for A(0), B(0).  The first steps find
        // more loads younger than the ones they wait for than the steady state assumes, which only makes
        // their waits stricter.
        fetch_a(areg[0], at(0));
        fetch_b(ring[0], at(0));
        fetch_b(ring[1], at(1));
        if (AD == 2) {
            fetch_a(areg[1], at(1));
            fetch_b(ring[2], at(2));
        }
        wait_loads<(AD == 2 ? 2 * kB + MBS : kB)>(areg[0], ring[0]);
        store_a(areg[0], lds[0], tid);
        __syncthreads();
        read_unit<MBS, 0>(af[0], lds[0], lane);
        // Step c = c0 + I, c0 a multiple of R (even when AD = 2): all register indices are static.
#define FFN_STEP(I)                                                                                        \
    {                                                                                                      \
        const int ci = c + (I);                                                                            \
        const char* a_base = reinterpret_cast<const char*>(A) +                                            \
                             static_cast<size_t>(at(min(ci + AD, last))) * a_chunk_bytes;                  \
        /* past the last step there is nothing left to prefetch: the loads still issue (the waits count   \
           them), but all lanes read the same 16 bytes, one cache line instead of a KiB per load */       \
        const uint32_t a_first_c = ci + AD > last ? 0u : a_first, a_last_c = ci + AD > last ? 0u : a_last; \
        const uint32_t a_keep = ci + AD > last ? 0u : ~0u;                                                 \
        auto issue_a = [&](auto ic) {                                                                      \
            constexpr int mb = decltype(ic)::value;                                                        \
            if constexpr (GATHER)                                                                          \
                ld_pinned<0>(areg[((I) + AD) % AD].v[mb], a_off[mb] & a_keep, a_base);                     \
            else if constexpr (mb + 1 < MBS)                                                               \
                ld_pinned<0>(areg[((I) + AD) % AD].v[mb], a_first_c, a_base + static_cast<size_t>(mb) * a_stride); \
            else                                                                                           \
                ld_pinned<0>(areg[((I) + AD) % AD].v[mb], a_last_c, a_base);                               \
        };                                                                                                 \
        const uint32_t voff = static_cast<uint32_t>(at(min(ci + AD + 1, last))) * (kKS * 2048) +           \
                              (ci + AD + 1 > last ? 0u : lane_off);                                        \
        auto issue_b = [&](auto ic) {                                                                      \
            constexpr int i = decltype(ic)::value, ks = i / NF, j = i % NF;                                \
            ld_pinned_stream<(ks & 1) * 2048 + j * 1024, KEEP>(ring[((I) + AD + 1) % R].v[ks][j],          \
                                                         voff + (ks >> 1) * 4096, wave_base);              \
        };                                                                                                 \
        run_step(acc, af, lds[ci & 1], lds[(ci + 1) & 1], ring[(I) % R], areg[((I) + 1) % AD],             \
                 ring[((I) + 1) % R], lane, tid, issue_a, issue_b);                                        \
    }
        for (; c + R <= chunks; c += R) {
            FFN_STEP(0) FFN_STEP(1) FFN_STEP(2) FFN_STEP(3)
        }
#undef FFN_STEP
        asm volatile("; pipeline end");
    }
    // the steps that do not fill a group of R, one by one and without overlap
    for (; c < chunks; ++c) {
        asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
        fetch_a(areg[0], at(c));
        fetch_b(ring[0], at(c));
        slow_step(acc, af, lds[0], areg[0], ring[0], lane, tid);
    }
    // Drain the prefetches nobody consumes, and only then let go of their destination registers: a
    // destination the compiler considers dead would be handed to something else (an LDS read, say)
    // while the load into it is still in flight.
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks)
#pragma unroll
            for (int j = 0; j < NF; ++j) asm volatile("" : : "v"(ring[r].v[ks][j]));
#pragma unroll
    for (int i = 0; i < AD; ++i)
#pragma unroll
        for (int mb = 0; mb < MBS; ++mb) asm volatile("" : : "v"(areg[i].v[mb]));
    __syncthreads();                            // the last LDS reads are done before the epilogue reuses the LDS
    tid = thread_id(wave_s);                    // rebuilt: the first copy need not survive the main loop
    // The block's next work item is taken now, by thread 0: the queue's answer arrives while the output tile is
    // filled, is published with the barrier that follows the filling, and lets every wave request the first weights
    // of its next item before it stores the tile, so that they are in the L2 (and the memory system has had this
    // compute unit's requests) by the time the next item's own first loads ask for them.  An item is taken only a
    // few microseconds before the block turns to it, so the balance of the queues is what it was.
    unsigned taken = 0u;
    if (tid == 0) taken = take_first(Q);
    constexpr int kWarm = kKS * (GATED ? 2 : NF);       // 16-byte pieces per lane of one pipeline step of this wave's stream
    u32x4 warm[kWarm];
#pragma unroll
    for (int i = 0; i < kWarm; ++i) warm[i] = u32x4{0u, 0u, 0u, 0u};
    // Epilogue through LDS (the activation buffers are free now).  The weight fragment is the first MFMA
    // operand and the activation fragment the second, so the accumulators hold the transposed tile: lane l
    // has token row l%32 of its row block and, in v = 4g..4g+3, the four neighbouring output columns
    // 8g + 4(l/32) + 0..3.  Every wave applies the activation, rounds four neighbours to bf16 and writes them
    // as one 8-byte piece into a row-major tile of the block's columns; then the whole block stores that tile
    // with 16 bytes per lane, whole 64-byte segments per row.  All rows are computed (clamped duplicates
    // give finite values), only real rows are stored.
    constexpr int W = 32 * (GATED ? 1 : NF);            // output columns per wave
    constexpr int kTileRowBytes = 4 * W * 2 + 16;       // padded: 4 dwords mod 32, eight rows x two halves cover the banks once
    constexpr int kRowsPerPass = W == 32 ? 256 : 128;   // tile rows that fit the LDS
    constexpr int kLanesPerRow = W / 2;                 // 16-byte stores per tile row
    constexpr int kRowsPerIter = 256 / kLanesPerRow;
    char* tile = reinterpret_cast<char*>(&lds[0][0]);
    static_assert(kRowsPerPass * kTileRowBytes <= static_cast<int>(sizeof(lds)), "epilogue tile must fit the LDS buffers");
    const int wave = wave_s;
    const int row_in = (tid & 31), col_in = 4 * ((tid & 63) >> 5);
    // the first step of this wave's weight stream in the block's next item (plain loads: they stay in the L2)
    auto warm_next = [&]() {
        const int nq = __builtin_amdgcn_readfirstlane(*sh_q);
        if (nq < 0) return;
        const Item nx = decode_item(Q, static_cast<unsigned>(nq), static_cast<unsigned>(__builtin_amdgcn_readfirstlane(*sh_x)), units);
        if (!nx.real) return;
        unsigned nkey;
        const char* nw = static_cast<const char*>(wave_stream<GATED, NF>(Q, nx.e, nx.block_y, wave_s, units, K, nkey));
        // (addressed as global memory, so that the loads return in order with the other global loads and the stores
        // that follow wait for their own operands only)
        typedef const __attribute__((address_space(1))) u32x4 global_u32x4;
        global_u32x4* src = (global_u32x4*)(nw + static_cast<size_t>(nkey % static_cast<unsigned>(chunks)) * (kKS * 2048)) + (tid & 63);
#pragma unroll
        for (int i = 0; i < kWarm; ++i) warm[i] = src[(GATED || NF == 2) ? i * 64 : i * 128];
    };
#pragma unroll
    for (int p0 = 0; p0 < MBS * 32; p0 += kRowsPerPass) {
        if (p0 > 0) __syncthreads();                    // the previous pass has been stored
        // the choice of activation is taken once per pass, outside the value loops, so that the sixteen
        // independent evaluations of a fragment can overlap
        auto fill = [&](auto exact) {
#pragma unroll
            for (int mb = p0 / 32; mb < MBS && mb < (p0 + kRowsPerPass) / 32; ++mb) {
                char* trow = tile + (mb * 32 + row_in - p0) * kTileRowBytes + (wave * W + col_in) * 2;
#pragma unroll
                for (int j = 0; j < (GATED ? 1 : NF); ++j) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        float h[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            if constexpr (GATED)
                                h[i] = act_fn_bf16(acc[mb][0][4 * g + i], decltype(exact)::value ? 0 : 1) * acc[mb][NF - 1][4 * g + i];
                            else
                                h[i] = acc[mb][j][4 * g + i];
                        }
                        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                        const bf16x4 packed = {static_cast<__bf16>(h[0]), static_cast<__bf16>(h[1]), static_cast<__bf16>(h[2]),
                                               static_cast<__bf16>(h[3])};
                        *reinterpret_cast<uint2*>(trow + (32 * j + 8 * g) * 2) = __builtin_bit_cast(uint2, packed);
                    }
                }
            }
        };
        if (!GATED || act == 0) fill(std::true_type{});
        else fill(std::false_type{});
        if (p0 == 0 && tid == 0) take_finish(Q, taken, sh_q, sh_x);
        __syncthreads();
        const int seg = (tid % kLanesPerRow) * 8;       // first of this lane's 8 columns inside the block
        const int src_wave = seg / W;
        const int out_unit = unit - wave + src_wave;            // unit of the wave that produced them
        if (out_unit < N / W) {
            // first of this lane's 8 columns, and the distance between rows, in elements: row-major output, or
            // (the up-projection's) the chunked order of H described above
            const int col = out_unit * W + (seg % W);
            uint16_t* cbase = GATED ? C + static_cast<size_t>(col >> 6) * h_rows * kKC + (col & (kKC - 1)) : C + col;
            const size_t c_row_elems = GATED ? static_cast<size_t>(kKC) : static_cast<size_t>(N);
            // All pieces of the pass are read from the tile (and their output rows looked up) before the first
            // is stored: one LDS and one look-up latency per pass instead of one per piece.
            //   row_map: where each row of the batched order goes (the layer's output rows, when the rows
            //   need no weighting afterwards); none: the batched order itself
            constexpr int kPieces = kRowsPerPass / kRowsPerIter;
            uint4 val[kPieces];
            int out_row[kPieces];
#pragma unroll
            for (int i = 0; i < kPieces; ++i) {
                if (i * kRowsPerIter < MBS * 32 - p0) {                   // rows this tile height has
                    const int r = static_cast<int>(tid) / kLanesPerRow + i * kRowsPerIter;
                    val[i] = *reinterpret_cast<const uint4*>(tile + r * kTileRowBytes + seg * 2);
                    const int row = row_begin + min(p0 + r, rows - 1);    // past the end: the last row again, not stored
                    out_row[i] = row_map != nullptr ? row_map[row] : row;
                }
            }
            if (p0 == 0) warm_next();
#pragma unroll
            for (int i = 0; i < kPieces; ++i) {
                if (i * kRowsPerIter < MBS * 32 - p0) {
                    const int r = static_cast<int>(tid) / kLanesPerRow + i * kRowsPerIter;
                    // written once and next read by another kernel, after far more traffic than the L2 holds: stored
                    // non-temporal, so that the rows do not take the place of weights and activation tiles there
                    // (5 % of the layer's time at 128 tokens per expert)
                    if (p0 + r < rows)
                        __builtin_nontemporal_store(u32x4{val[i].x, val[i].y, val[i].z, val[i].w},
                                                    reinterpret_cast<u32x4*>(cbase + static_cast<size_t>(out_row[i]) * c_row_elems));
                }
            }
        } else if (p0 == 0) {
            warm_next();
        }
    }
    // the requested pieces are only wanted in the cache; their registers are given up once they have arrived
#pragma unroll
    for (int i = 0; i < kWarm; ++i) asm volatile("" : : "v"(warm[i]));
}

// The work list of a launch is written by ffn_plan_block (ffn_plan.h): here as a kernel of its own.
constexpr int kKeepFromTiles = 2;       // row tiles of an expert from which its weights are worth keeping in the L2

__global__ __launch_bounds__(256) void ffn_plan_kernel(const int32_t* __restrict__ offsets, int e_first, int e_count,
                                                       int tile_m_up, int tile_m_down, int32_t* __restrict__ plan, int total_rows,
                                                       int max_tiles) {
    __shared__ int scratch[4][256];
    ffn_plan_block(offsets, e_first, e_count, tile_m_up, plan, total_rows, max_tiles, scratch, 0);
    if (tile_m_down != tile_m_up) {             // else the down kernel reads the up kernel's list
        __syncthreads();
        ffn_plan_block(offsets, e_first, e_count, tile_m_down, plan, total_rows, max_tiles, scratch, 1);
    }
}

// C[rows of one expert tile, N] = A[rows, K] * B_e, B_e in packed fragment order.
// A work item is one row tile (up to 256 rows of one expert; only the 32-row blocks that hold rows are
// computed) by one column group of 4 units, one unit per wave, for all rows.
// GATED (NF = 2): a unit is 32 output columns whose two fragments per k-step are (W_gate, W_in); the
//   epilogue writes act(gate) * in.
// otherwise a unit is 32 * NF output columns of W_out.
// Weight fragments stream HBM -> registers through a ring of buffers so that several KiB per
// wave are always in flight; the activation tile goes through LDS, double buffered.
//
// One block per compute unit stays resident and takes work items from 8 queues, one per XCD (blocks go
// round-robin to the XCDs, each with its own L2, so blockIdx % 8 names the XCD): position q of a
// queue decodes into 32-item runs of 2^mt_shift neighbouring row tiles x 32 / 2^mt_shift neighbouring
// column groups.  Tiles of one expert then share its weight stream, and the column groups of a tile
// share its activation tile, in that XCD's L2; groups of tiles are dealt to the queues in turn.  A
// block whose own queue is empty helps with the others.
// GATHER (up-projection only): A is the token array x and the rows of a tile are looked up through `gather`
// (the permutation written by the batching step; row r is token gather[r] / gather_k); tiles then have at most
// kGatherTileM rows.
template <bool GATED, int NF, bool GATHER = false>
__global__ __launch_bounds__(256) void ffn_mfma_kernel(const uint16_t* __restrict__ A, int32_t* __restrict__ plan,
                                                       int counter_base, int e_first, const char* __restrict__ W,
                                                       size_t expert_stride_bytes, size_t block_offset_bytes,
                                                       uint16_t* __restrict__ C, int K, int N, int act, int y_chunks,
                                                       int mt_shift, const int32_t* __restrict__ row_map,
                                                       const int32_t* __restrict__ gather, int gather_k, int h_rows,
                                                       int list, int max_tiles) {
    __shared__ uint4 lds[2][kTileM * kLdsRow];     // 2 x 36 KiB activation tiles, padded rows
    __shared__ int sh_q, sh_x;
    ItemQueue Q;
    Q.tiles = plan[16 + list];
    Q.y_chunks = y_chunks;
    Q.mt_shift = mt_shift;
    const unsigned per_group = 8u << mt_shift;
    Q.total_q = (static_cast<unsigned>(Q.tiles) + per_group - 1u) / per_group * static_cast<unsigned>(y_chunks) * 32u;
    Q.tile_list = reinterpret_cast<const int4*>(plan + kPlanHeader + 4 * list * max_tiles);
    Q.counters = reinterpret_cast<unsigned*>(plan) + counter_base;
    Q.home = blockIdx.x & 7u;
    Q.W = W;
    Q.expert_stride_bytes = expert_stride_bytes;
    Q.block_offset_bytes = block_offset_bytes;
    Q.e_first = e_first;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
    // an item taken with nothing to do meanwhile: the first one, and the one after a padding position
    auto take_now = [&]() {
        __syncthreads();                           // everybody has read the previous position
        if (thread_id(wave) == 0) take_finish(Q, take_first(Q), &sh_q, &sh_x);
        __syncthreads();
    };
    take_now();
    for (;;) {
        if (sh_q < 0) return;                      // every queue is empty (uniform for the block)
        // The tile code below is compiled for eight tile heights; values that do not change from item to
        // item would be hoisted out of this loop and held in registers across all of them.  The inputs
        // are made opaque per iteration instead.
        int Kl = K, Nl = N;
        asm volatile("" : "+s"(Kl), "+s"(Nl));
        const int units = Nl / (32 * (GATED ? 1 : NF));
        const Item it = decode_item(Q, static_cast<unsigned>(__builtin_amdgcn_readfirstlane(sh_q)),
                                    static_cast<unsigned>(__builtin_amdgcn_readfirstlane(sh_x)), units);
        if (!it.real) { take_now(); continue; }    // past the last tile or column group (uniform)
        const int e = it.e, row_begin = it.row_begin, rows = it.rows, tiles_of_expert = it.tiles_of_expert;
        const int unit = it.block_y * 4 + wave;
        const bool active = unit < units;          // a wave past the last unit recomputes the last one, stores nothing
        unsigned key;
        const void* wave_w = wave_stream<GATED, NF>(Q, e, it.block_y, wave, units, Kl, key);
        // weights of an expert with two row tiles or more are left in the L2 for its other tiles
        const bool keep = tiles_of_expert >= kKeepFromTiles;
        const int blocks = min((rows + 31) >> 5, GATHER ? kGatherTileM / 32 : kTileM / 32);
#define FFN_TILE(M, KP)                                                                                              \
    ffn_tile<GATED, NF, M, KP, GATHER>(lds, A, row_begin, rows, wave_w, C, Kl, Nl, unit, active, act, key, wave, row_map, \
                                       gather, gather_k, Q, units, &sh_q, &sh_x, h_rows)
#define FFN_CASE(M)                                                                                                  \
    case M:                                                                                                          \
        if (keep) FFN_TILE(M, true); else FFN_TILE(M, false);                                                        \
        break;
        if constexpr (GATHER) {
            switch (blocks) { FFN_CASE(1) FFN_CASE(2) FFN_CASE(3) FFN_CASE(4) FFN_CASE(5) FFN_CASE(6) default: if (keep) FFN_TILE(kGatherTileM / 32, true); else FFN_TILE(kGatherTileM / 32, false); break; }
        } else {
            switch (blocks) { FFN_CASE(1) FFN_CASE(2) FFN_CASE(3) FFN_CASE(4) FFN_CASE(5) FFN_CASE(6) FFN_CASE(7) default: if (keep) FFN_TILE(8, true); else FFN_TILE(8, false); break; }
        }
#undef FFN_CASE
#undef FFN_TILE
        __syncthreads();                           // the tile has been read out of the LDS; the next position is in sh_q
    }
}

// ------------------------------------------------------------------------------------------ fp32 FMA

constexpr int kF32Tile = 64;

template <bool GATED>
__global__ __launch_bounds__(256) void ffn_f32_kernel(const float* __restrict__ A, const int32_t* __restrict__ offsets,
                                                      int e_first, int e_count, const float* __restrict__ W,
                                                      size_t expert_stride_elems, size_t off_b0, size_t off_b1,
                                                      float* __restrict__ C, int K, int N, int act, int total_rows) {
    __shared__ float As[16][kF32Tile + 4];
    __shared__ float B0s[16][kF32Tile + 4];
    __shared__ float B1s[GATED ? 16 : 1][kF32Tile + 4];
    int e, row_begin, rows;
    if (!find_tile(offsets, e_first, e_count, kF32Tile, blockIdx.y, total_rows, e, row_begin, rows)) return;
    const float* B0 = W + static_cast<size_t>(e - e_first) * expert_stride_elems + off_b0;
    const float* B1 = W + static_cast<size_t>(e - e_first) * expert_stride_elems + off_b1;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int n0 = blockIdx.x * kF32Tile;
    float acc0[4][4], acc1[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) { acc0[i][j] = 0.f; acc1[i][j] = 0.f; }
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = threadIdx.x + i * 256;
            const int r = id >> 4, kk = id & 15;
            As[kk][r] = r < rows ? A[static_cast<size_t>(row_begin + r) * K + k0 + kk] : 0.f;
            const int kb = id >> 6, cc = id & 63;
            B0s[kb][cc] = B0[static_cast<size_t>(k0 + kb) * N + n0 + cc];
            if (GATED) B1s[kb][cc] = B1[static_cast<size_t>(k0 + kb) * N + n0 + cc];
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], p[4], q[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) { p[j] = B0s[kk][tx * 4 + j]; q[j] = GATED ? B1s[kk][tx * 4 + j] : 0.f; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc0[i][j] = fmaf(a[i], p[j], acc0[i][j]);
                    if (GATED) acc1[i][j] = fmaf(a[i], q[j], acc1[i][j]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = ty * 4 + i;
        if (r < rows) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float v = GATED ? act_fn(acc0[i][j], act) * acc1[i][j] : acc0[i][j];
                C[static_cast<size_t>(row_begin + r) * N + n0 + tx * 4 + j] = v;
            }
        }
    }
}

__global__ __launch_bounds__(256) void copy_vec_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
    const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

}  // namespace

constexpr int kMinTileM = 64;           // lowest row tile a launch is ever cut into
size_t ffn_plan_tiles(const moe_cfg& c) { return static_cast<size_t>(c.T) * c.k / kMinTileM + c.E; }   // room for the lowest tiles
int ffn_tile_rows(bool gather) { return gather ? kGatherTileM : kTileM; }
size_t ffn_plan_bytes(const moe_cfg& c) { return (kPlanHeader + 2 * 4 * ffn_plan_tiles(c)) * sizeof(int32_t); }

// Height of the down-projection's row tiles.  Its work items are (row tile x 256 output columns): with few experts of
// a tile or so each there are fewer items than compute units (8 experts of about 256 rows: 8 to 16 tiles x 16 column
// groups for 256 compute units, and a tile takes as long as its 160 reduction steps whether others run or not).  The
// tiles are then cut lower, so that every expert gives as many tiles as fill the chip (with a quarter of headroom for
// experts above the mean); measured on that layer: 0.235 -> 0.184 ms.  Lower tiles for the up-projection, which has
// five times the column groups, only cost (0.327 -> 0.354 ms), so the two kernels have a tile list each.
int ffn_down_tile_rows(const moe_cfg& c, int e_count, long max_rows, int tile_m_up, int n_cu) {
    const long mean_rows = max_rows / (e_count > 0 ? e_count : 1);
    const int col_groups = (c.d / 64 + 3) / 4;
    if (mean_rows <= 224 || static_cast<long>(e_count) * col_groups >= n_cu) return tile_m_up;
    const long per_expert = (n_cu + static_cast<long>(e_count) * col_groups - 1) / (static_cast<long>(e_count) * col_groups);
    long tm = ((mean_rows * 5 / 4 + per_expert - 1) / per_expert + 31) / 32 * 32;
    tm = tm < kMinTileM ? kMinTileM : tm;
    return tm < tile_m_up ? static_cast<int>(tm) : tile_m_up;
}

int launch_pack(const moe_cfg& c, const void* Win, const void* Wgate, const void* Wout, void* packed, hipStream_t s) {
    const size_t df = static_cast<size_t>(c.d) * c.f;
    if (c.dtype == MOE_BF16) {
        const long frags = static_cast<long>(c.f / 32) * (c.d / 16) * 2 + static_cast<long>(c.d / 64) * (c.f / 16) * 2;
        const long threads = frags * 64;
        hipLaunchKernelGGL(pack_bf16_kernel, dim3(static_cast<unsigned>((threads + 255) / 256)), dim3(256), 0, s,
                           static_cast<const uint16_t*>(Win), static_cast<const uint16_t*>(Wgate),
                           static_cast<const uint16_t*>(Wout), static_cast<uint4*>(packed), c.d, c.f);
        MOE_LAUNCH_CHECK("pack_bf16_kernel");
        return MOE_OK;
    }
    // fp32: W_gate | W_in | W_out, row-major, unchanged
    const size_t vecs = df * 4 / 16;
    const void* srcs[3] = {Wgate, Win, Wout};
    for (int i = 0; i < 3; ++i) {
        hipLaunchKernelGGL(copy_vec_kernel, dim3(static_cast<unsigned>((vecs + 255) / 256)), dim3(256), 0, s,
                           static_cast<const uint4*>(srcs[i]), static_cast<uint4*>(packed) + i * vecs, vecs);
        MOE_LAUNCH_CHECK("copy_vec_kernel");
    }
    return MOE_OK;
}

int launch_expert_ffn(const moe_cfg& c, const void* Xp, const int32_t* offsets, int e_first, int e_count,
                      const void* W, size_t expert_stride_bytes, long max_rows, void* H, void* Yp, int32_t* plan,
                      hipStream_t s, hipEvent_t between, hipEvent_t before_up, const int32_t* row_map, bool plan_ready,
                      const int32_t* gather) {
    if (max_rows <= 0 || e_count <= 0) return MOE_OK;
    const size_t df = static_cast<size_t>(c.d) * c.f;
    if (gather != nullptr && c.dtype != MOE_BF16) return fail(MOE_ERR_UNSUPPORTED, "gathered rows are a bf16 path");
    if (c.dtype == MOE_BF16) {
        // Work items: 8 queues x (groups of row tiles per queue) x (chunks of column groups) x 32; the
        // resident blocks take them until the queues are empty.
        int dev = 0;
        const DeviceInfo* info = nullptr;
        if (int rc = device_info(&dev, &info)) return rc;
        const int n_cu = info->compute_units;
        const int tile_m = ffn_tile_rows(gather != nullptr);
        const int tile_m_down = ffn_down_tile_rows(c, e_count, max_rows, tile_m, n_cu);
        const long slots = max_rows / tile_m + e_count;                // upper bound of the number of row tiles
        const long slots_down = max_rows / tile_m_down + e_count;
        if (slots_down > static_cast<long>(ffn_plan_tiles(c)))
            return fail(MOE_ERR_INVALID_ARG, "more row tiles (%ld) than the workspace plans for", slots_down);
        if (slots > static_cast<long>(ffn_plan_tiles(c)))
            return fail(MOE_ERR_INVALID_ARG, "more row tiles (%ld) than the workspace plans for", slots);
        // Row tiles per group (4, 2 or 1): neighbouring tiles in the list belong to one expert when experts have
        // several tiles, and then a group shares the expert's weight stream in one XCD's L2; when experts have
        // a single tile each, a group of several would only put several activation tiles into that L2 at once
        // (measured at 128 tokens per expert: 3 % of the layer's time).  Decided from the mean rows per expert,
        // all the host knows.
        const long mean_rows = max_rows / e_count;
        const int by_rows = mean_rows > 384 ? 2 : mean_rows > 192 ? 1 : 0;
        auto shift_for = [&](long n_slots) {
            const int by_tiles = n_slots >= 32 ? 2 : n_slots >= 16 ? 1 : 0;
            return by_rows < by_tiles ? by_rows : by_tiles;
        };
        const int mt_shift = shift_for(slots), mt_shift_down = shift_for(slots_down);
        auto items_for = [&](long n_slots, int shift, int col_groups, int& y_chunks) {
            const long tile_groups = (n_slots + (8L << shift) - 1) / (8L << shift);   // per queue
            const int ny = 32 >> shift;
            y_chunks = (col_groups + ny - 1) / ny;
            return tile_groups * y_chunks * 32 * 8;
        };
        const int max_tiles = static_cast<int>(ffn_plan_tiles(c));
        const int down_list = tile_m_down != tile_m ? 1 : 0;       // equal heights: one list serves both kernels
        auto grid_for = [&](long items) { return dim3(static_cast<unsigned>(items < n_cu ? items : n_cu)); };
        if (!plan_ready) {          // else the kernel that batched the tokens has written the work list as well
            hipLaunchKernelGGL(ffn_plan_kernel, dim3(1), dim3(256), 0, s, offsets, e_first, e_count, tile_m, tile_m_down, plan,
                               c.T * c.k, max_tiles);
            MOE_LAUNCH_CHECK("ffn_plan_kernel");
        }
        if (before_up != nullptr) MOE_HIP_CHECK(hipEventRecord(before_up, s));
        const size_t down_off = 2 * df * 2;
        dim3 block(256);
        int yc = 0;
        long items = items_for(slots, mt_shift, (c.f / 32 + 3) / 4, yc);
        if (items > 0x7fffffffL) return fail(MOE_ERR_UNSUPPORTED, "too many work items for one launch (%ld)", items);
        // (with `gather`, Xp is the token array and the kernel looks its rows up itself)
        if (gather != nullptr)
            hipLaunchKernelGGL((ffn_mfma_kernel<true, 2, true>), grid_for(items), block, 0, s, static_cast<const uint16_t*>(Xp), plan, 0,
                               e_first, static_cast<const char*>(W), expert_stride_bytes, size_t(0), static_cast<uint16_t*>(H),
                               c.d, c.f, c.act, yc, mt_shift, static_cast<const int32_t*>(nullptr), gather, c.k, c.T * c.k, 0, max_tiles);
        else
            hipLaunchKernelGGL((ffn_mfma_kernel<true, 2>), grid_for(items), block, 0, s, static_cast<const uint16_t*>(Xp), plan, 0,
                               e_first, static_cast<const char*>(W), expert_stride_bytes, size_t(0), static_cast<uint16_t*>(H),
                               c.d, c.f, c.act, yc, mt_shift, static_cast<const int32_t*>(nullptr),
                               static_cast<const int32_t*>(nullptr), 1, c.T * c.k, 0, max_tiles);
        MOE_LAUNCH_CHECK("ffn_mfma_kernel<up>");
        if (between != nullptr) MOE_HIP_CHECK(hipEventRecord(between, s));
        // down-projection: narrow (32-column) units when wide ones would leave compute units idle
        const long tiles_hint = (max_rows + tile_m - 1) / tile_m > e_count ? (max_rows + tile_m - 1) / tile_m : e_count;
        // (only while the experts are likely to have a single tile each, mean rows up to 224, and their items are
        // bound by the weight stream: on 256-row tiles, and once experts spill into second tiles, the narrow unit's
        // second LDS read per MFMA costs more than the idle compute units do; measured on 8 experts: 128 rows per
        // expert 0.148 ms narrow against 0.177 ms wide, 256 rows 0.274 against 0.239)
        const bool narrow = tiles_hint * ((c.d / 64 + 3) / 4) < 2 * 256 && mean_rows <= 224;
        items = items_for(slots_down, mt_shift_down, ((narrow ? c.d / 32 : c.d / 64) + 3) / 4, yc);
        if (items > 0x7fffffffL) return fail(MOE_ERR_UNSUPPORTED, "too many work items for one launch (%ld)", items);
        if (narrow)
            hipLaunchKernelGGL((ffn_mfma_kernel<false, 1>), grid_for(items), block, 0, s, static_cast<const uint16_t*>(H), plan, 8,
                               e_first, static_cast<const char*>(W), expert_stride_bytes, down_off, static_cast<uint16_t*>(Yp),
                               c.f, c.d, c.act, yc, mt_shift_down, row_map, static_cast<const int32_t*>(nullptr), 1, c.T * c.k, down_list, max_tiles);
        else
            hipLaunchKernelGGL((ffn_mfma_kernel<false, 2>), grid_for(items), block, 0, s, static_cast<const uint16_t*>(H), plan, 8,
                               e_first, static_cast<const char*>(W), expert_stride_bytes, down_off, static_cast<uint16_t*>(Yp),
                               c.f, c.d, c.act, yc, mt_shift_down, row_map, static_cast<const int32_t*>(nullptr), 1, c.T * c.k, down_list, max_tiles);
        MOE_LAUNCH_CHECK("ffn_mfma_kernel<down>");
        return MOE_OK;
    }
    const long slots = max_rows / kF32Tile + e_count;
    if (slots > 65535) return fail(MOE_ERR_UNSUPPORTED, "too many row tiles for one launch (%ld)", slots);
    const size_t stride = expert_stride_bytes / 4;
    const float* Wf = static_cast<const float*>(W);
    hipLaunchKernelGGL(ffn_f32_kernel<true>, dim3(c.f / kF32Tile, static_cast<unsigned>(slots)), dim3(256), 0, s,
                       static_cast<const float*>(Xp), offsets, e_first, e_count, Wf, stride, size_t(0), df,
                       static_cast<float*>(H), c.d, c.f, c.act, c.T * c.k);
    MOE_LAUNCH_CHECK("ffn_f32_kernel<up>");
    if (between != nullptr) MOE_HIP_CHECK(hipEventRecord(between, s));
    hipLaunchKernelGGL(ffn_f32_kernel<false>, dim3(c.d / kF32Tile, static_cast<unsigned>(slots)), dim3(256), 0, s,
                       static_cast<const float*>(H), offsets, e_first, e_count, Wf, stride, 2 * df, 2 * df,
                       static_cast<float*>(Yp), c.f, c.d, c.act, c.T * c.k);
    MOE_LAUNCH_CHECK("ffn_f32_kernel<down>");
    return MOE_OK;
}

}  // namespace moe
