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

namespace moe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kKC = 64;                 // reduction elements staged per pipeline step (4 MFMA k-steps)

__device__ inline float act_fn(float z, int act) {
    if (act == 0) return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
    const float u = 0.79788456080286536f * (z + 0.044715f * z * z * z);
    return 0.5f * z * (1.0f + tanhf(u));
}

// Activation for results that are rounded to bf16 right away: erf from the rational-times-Gaussian
// approximation 7.1.26 of Abramowitz & Stegun (|error| <= 1.5e-7 on erf, 5e-7 on GELU, three orders
// below the bf16 rounding of the result) instead of the library erff, which is several times longer.
__device__ inline float act_fn_bf16(float z, int act) {
    if (act != 0) return act_fn(z, act);
    const float x = fabsf(z) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * x);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    const float erf_abs = 1.0f - poly * __expf(-x * x);
    return 0.5f * z * (1.0f + copysignf(erf_abs, z));
}

// Which (expert, row tile) a block works on: tile slot `slot` counted over the experts
// [e_first, e_first + e_count) in order, at most tile_m rows per tile.  Returns false when the slot is past
// the last tile (uniform for the block).  Must be called by all threads of the block.
__device__ inline bool find_tile(const int32_t* __restrict__ offsets, int e_first, int e_count, int tile_m, int slot,
                                 int& e_out, int& row_begin, int& rows) {
    __shared__ int sh_e, sh_mt;
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        int tl[4], sum = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = lane * 4 + q;
            const int cnt = e < e_count ? offsets[e_first + e + 1] - offsets[e_first + e] : 0;
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
    const int n = offsets[e_out + 1] - offsets[e_out];
    const int tiles = (n + tile_m - 1) / tile_m;
    const int per_tile = min(tile_m, ((n + tiles - 1) / tiles + 31) & ~31);
    row_begin = offsets[e_out] + sh_mt * per_tile;
    rows = min(per_tile, offsets[e_out + 1] - row_begin);
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
constexpr int kRing = 3;                // weight-fragment register buffers
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
// Same, marked non-temporal: the weights are read once, they should not push the activation tiles
// (which every column group of an expert re-reads) out of the L2.
template <int IMM>
__device__ inline void ld_pinned_stream(u32x4& dst, uint32_t voff, const void* sbase) {
    asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3 nt" : "=v"(dst) : "v"(voff), "s"(sbase), "n"(IMM) : "memory");
}

// The two fragments of one (column unit, k-step) are adjacent in the packed block:
// [k-step][2][64 lanes] x 16 bytes (2 KiB per k-step); a wave with NF = 1 reads one of the two.
// voff = byte offset of this lane inside its wave's stream at the first k-step of the pipeline step.
template <int NF>
__device__ inline void load_b(BFrags<NF>& b, uint32_t voff, const void* wave_base) {
    ld_pinned_stream<0>(b.v[0][0], voff, wave_base);
    if (NF == 2) ld_pinned_stream<1024>(b.v[0][NF - 1], voff, wave_base);
    ld_pinned_stream<2048>(b.v[1][0], voff, wave_base);
    if (NF == 2) ld_pinned_stream<3072>(b.v[1][NF - 1], voff, wave_base);
    const uint32_t voff2 = voff + 4096;
    ld_pinned_stream<0>(b.v[2][0], voff2, wave_base);
    if (NF == 2) ld_pinned_stream<1024>(b.v[2][NF - 1], voff2, wave_base);
    ld_pinned_stream<2048>(b.v[3][0], voff2, wave_base);
    if (NF == 2) ld_pinned_stream<3072>(b.v[3][NF - 1], voff2, wave_base);
}

// End-of-step wait: at most 4*NF loads (this step's weight prefetch) may still be outstanding.
template <int NF, int MBS>
__device__ inline void wait_step(ARegs<MBS>& a, BFrags<NF>& next) {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(kKS * NF) : "memory");
#pragma unroll
    for (int mb = 0; mb < MBS; ++mb) asm volatile("" : "+v"(a.v[mb]));
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks)
#pragma unroll
        for (int j = 0; j < NF; ++j) asm volatile("" : "+v"(next.v[ks][j]));
}

// The activation tile lives in LDS row-major, one padded row of kLdsRow uint4 per tile row.
// Staging: thread t moves, for i < MBS, the 16-byte piece (row i*32 + t/8, piece t%8): eight
// neighbouring lanes fetch one whole 128-byte line of a row, and write 128 contiguous bytes of LDS.
template <int MBS>
__device__ inline void store_a(const ARegs<MBS>& a, uint4* lds_buf) {
    u32x4* p = reinterpret_cast<u32x4*>(lds_buf) + (threadIdx.x >> 3) * kLdsRow + (threadIdx.x & 7);
#pragma unroll
    for (int mb = 0; mb < MBS; ++mb) p[mb * 32 * kLdsRow] = a.v[mb];
}

// One pipeline step: 4 k-steps of MBS x NF MFMAs.  The A fragments of the next k-step are read from
// LDS while the MFMAs of the current one run.  Fragment (mb, ks) of lane l = row mb*32 + l%32,
// 8 elements at k = 16 ks + 8 (l / 32).
template <int NF, int MBS>
__device__ inline void mma_step(f32x16 (&acc)[MBS][NF], const uint4* lds_buf, const BFrags<NF>& b, int lane) {
    const uint4* rp = lds_buf + (lane & 31) * kLdsRow + (lane >> 5);
    uint4 af[2][MBS];
#pragma unroll
    for (int mb = 0; mb < MBS; ++mb) af[0][mb] = rp[mb * 32 * kLdsRow];
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) {
        if (ks + 1 < kKS) {
#pragma unroll
            for (int mb = 0; mb < MBS; ++mb) af[(ks + 1) & 1][mb] = rp[mb * 32 * kLdsRow + 2 * (ks + 1)];
        }
#pragma unroll
        for (int mb = 0; mb < MBS; ++mb) {
#pragma unroll
            for (int j = 0; j < NF; ++j)
                acc[mb][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(af[ks & 1][mb]), as_bf16x8(b.v[ks][j]),
                                                                     acc[mb][j], 0, 0, 0);
        }
    }
}

// One tile of MBS 32-row blocks: the whole reduction loop and the epilogue.
// Loads past the end are clamped to valid addresses (rows to the last row of the tile, pipeline steps
// to the last step) instead of being skipped, so every step issues the same loads.  Rows that are
// clamped duplicates only produce output rows that are never stored (an output row depends on its own
// input row only).
template <bool GATED, int NF, int MBS>
__device__ inline void ffn_tile(uint4 (&lds)[2][kTileM * kLdsRow], const uint16_t* __restrict__ A, int row_begin, int rows,
                                const void* wave_base, uint16_t* __restrict__ C, int K, int N, int unit,
                                bool active, int act, unsigned phase_key) {
    const int lane = threadIdx.x & 63;
    const int chunks = K / kKC, last = chunks - 1;

    // this thread's activation sources (byte offsets from A): row mb*32 + t/8 of every block, piece t%8;
    // rows past the tile end re-read the last row
    const int r0 = threadIdx.x >> 3;
    uint32_t a_off[MBS];
#pragma unroll
    for (int mb = 0; mb < MBS; ++mb)
        a_off[mb] = (static_cast<uint32_t>(row_begin + min(mb * 32 + r0, rows - 1)) * K + 8 * (threadIdx.x & 7)) * 2u;

    f32x16 acc[MBS][NF];
#pragma unroll
    for (int mb = 0; mb < MBS; ++mb)
#pragma unroll
        for (int j = 0; j < NF; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][j][v] = 0.f;

    ARegs<MBS> areg;
    BFrags<NF> ring[kRing];
    auto fetch_a = [&](int chunk) {
        const uint32_t step_off = static_cast<uint32_t>(chunk) * (kKC * 2);
#pragma unroll
        for (int mb = 0; mb < MBS; ++mb) ld_pinned<0>(areg.v[mb], a_off[mb] + step_off, A);
    };
    auto fetch_b = [&](BFrags<NF>& dst, int chunk) {
        load_b(dst, static_cast<uint32_t>(chunk) * (kKS * 2048) + lane * 16, wave_base);
    };
    // Blocks that run at the same time start their sweep over the reduction dimension at different
    // steps (and wrap around), so that concurrent waves do not walk their weight streams, which lie a
    // power of two apart, in lockstep.  The phase depends only on (expert, row tile, column group),
    // never on the launch shape, so a launch over all experts and a launch over one expert sum in the
    // same order (bitwise equal results).
    const int phase = static_cast<int>(phase_key % static_cast<unsigned>(chunks));
    auto at = [&](int i) { const int c = phase + i; return c >= chunks ? c - chunks : c; };   // i < chunks
    fetch_a(at(0));
    fetch_b(ring[0], at(0));
    fetch_b(ring[1], at(min(1, last)));
    wait_step(areg, ring[0]);                  // everything but the newest weight step has landed
    store_a(areg, lds[0]);
    __syncthreads();

#define FFN_STEP(I)                                                                   \
    {                                                                                 \
        const int ci = c + (I);                                                       \
        fetch_a(at(min(ci + 1, last)));                                               \
        fetch_b(ring[((I) + 2) % kRing], at(min(ci + 2, last)));                      \
        mma_step(acc, lds[(ci) & 1], ring[(I)], lane);                                \
        wait_step(areg, ring[((I) + 1) % kRing]);                                     \
        store_a(areg, lds[(ci + 1) & 1]);                                             \
        __syncthreads();                                                              \
    }
    int c = 0;
    for (; c + kRing <= chunks; c += kRing) {
        FFN_STEP(0) FFN_STEP(1) FFN_STEP(2)
    }
    const int left = chunks - c;               // 0..2 steps that do not fill a group
    if (left > 0) FFN_STEP(0)
    if (left > 1) FFN_STEP(1)
#undef FFN_STEP
    // Drain the prefetches nobody consumes, and only then let go of their destination registers: a
    // destination the compiler considers dead would be handed to something else (an LDS read, say)
    // while the load into it is still in flight.
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
#pragma unroll
    for (int r = 0; r < kRing; ++r)
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks)
#pragma unroll
            for (int j = 0; j < NF; ++j) asm volatile("" : : "v"(ring[r].v[ks][j]));
#pragma unroll
    for (int mb = 0; mb < MBS; ++mb) asm volatile("" : : "v"(areg.v[mb]));
    // Epilogue through LDS (the activation buffers are free now): every wave applies the activation to
    // its accumulators and writes bf16 values into a row-major tile of the block's columns; then the
    // whole block stores that tile with 16 bytes per lane, whole 64-byte segments per row.  All rows
    // are computed (clamped duplicates give finite values), only real rows are stored.
    constexpr int W = 32 * (GATED ? 1 : NF);            // output columns per wave
    constexpr int kTileRowBytes = 4 * W * 2 + 16;       // padded: the two row groups of a wave hit different banks
    constexpr int kRowsPerPass = W == 32 ? 256 : 128;   // tile rows that fit the LDS
    constexpr int kLanesPerRow = W / 2;                 // 16-byte stores per tile row
    constexpr int kRowsPerIter = 256 / kLanesPerRow;
    char* tile = reinterpret_cast<char*>(&lds[0][0]);
    static_assert(kRowsPerPass * kTileRowBytes <= static_cast<int>(sizeof(lds)), "epilogue tile must fit the LDS buffers");
    const int wave = threadIdx.x >> 6;
    const int col_in = lane & 31, row_in = 4 * (lane >> 5);
#pragma unroll
    for (int p0 = 0; p0 < MBS * 32; p0 += kRowsPerPass) {
        if (p0 > 0) __syncthreads();                    // the previous pass has been stored
#pragma unroll
        for (int mb = p0 / 32; mb < MBS && mb < (p0 + kRowsPerPass) / 32; ++mb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                // accumulator layout of the 32x32 MFMA: lane holds column lane%32, rows 8*(v/4) + 4*(lane/32) + v%4
                const int r = mb * 32 + 8 * (v >> 2) + row_in + (v & 3) - p0;
                uint16_t* trow = reinterpret_cast<uint16_t*>(tile + r * kTileRowBytes) + wave * W + col_in;
                if (GATED) {
                    const float h = act_fn_bf16(acc[mb][0][v], act) * acc[mb][1][v];
                    trow[0] = __builtin_bit_cast(uint16_t, static_cast<__bf16>(h));
                } else {
#pragma unroll
                    for (int j = 0; j < NF; ++j) trow[32 * j] = __builtin_bit_cast(uint16_t, static_cast<__bf16>(acc[mb][j][v]));
                }
            }
        }
        __syncthreads();
        const int seg = (threadIdx.x % kLanesPerRow) * 8;       // first of this lane's 8 columns inside the block
        const int src_wave = seg / W;
        const int out_unit = unit - wave + src_wave;            // unit of the wave that produced them
        if (out_unit < N / W) {
            uint16_t* cbase = C + static_cast<size_t>(out_unit) * W + (seg % W);
            for (int r = threadIdx.x / kLanesPerRow; r < kRowsPerPass && p0 + r < rows; r += kRowsPerIter) {
                const uint4 val = *reinterpret_cast<const uint4*>(tile + r * kTileRowBytes + seg * 2);
                *reinterpret_cast<uint4*>(cbase + static_cast<size_t>(row_begin + p0 + r) * N) = val;
            }
        }
    }
}

// C[rows of one expert tile, N] = A[rows, K] * B_e, B_e in packed fragment order.
// A block is up to 256 rows of one expert (only the 32-row blocks that hold rows are computed) by
// 4 waves; wave w owns column unit 4*(column group) + w for all rows.
// GATED (NF = 2): a unit is 32 output columns whose two fragments per k-step are (W_gate, W_in); the
//   epilogue writes act(gate) * in.
// otherwise a unit is 32 * NF output columns of W_out.
// Weight fragments stream HBM -> registers through a ring of kRing buffers so that several KiB per
// wave are always in flight; the activation tile goes through LDS, double buffered.
template <bool GATED, int NF>
__global__ __launch_bounds__(256) void ffn_mfma_kernel(const uint16_t* __restrict__ A, const int32_t* __restrict__ offsets,
                                                       int e_first, int e_count, const char* __restrict__ W,
                                                       size_t expert_stride_bytes, size_t block_offset_bytes,
                                                       uint16_t* __restrict__ C, int K, int N, int act, int y_chunks,
                                                       int mt_shift) {
    __shared__ uint4 lds[2][kTileM * kLdsRow];     // 2 x 36 KiB activation tiles, padded rows
    // Block id -> (row-tile slot, column group).  Workgroups go round-robin to the 8 XCDs, each with its
    // own L2, so the id is split into x = id % 8 (the XCD) and the position q in that XCD's queue; 32
    // consecutive positions (about what an XCD runs at a time) are 2^mt_shift neighbouring row tiles x
    // 32 / 2^mt_shift neighbouring column groups.  Tiles of one expert then share its weight stream, and
    // the column groups of a tile share its activation tile, in that XCD's L2; the groups of tiles are
    // dealt to the XCDs in turn so that the load is even (fewer tiles per group when there are few).
    const unsigned xcd = blockIdx.x & 7u, q = blockIdx.x >> 3;
    const unsigned ny = 32u >> mt_shift;           // column groups per run of 32; 1 << mt_shift row tiles
    const unsigned yg = q & (ny - 1u), mt = (q / ny) & ((1u << mt_shift) - 1u), rest = q >> 5;
    const unsigned y_chunk = rest % static_cast<unsigned>(y_chunks), tile_group = rest / static_cast<unsigned>(y_chunks);
    const int slot = static_cast<int>((((tile_group << 3) + xcd) << mt_shift) + mt);
    const int block_y = static_cast<int>(y_chunk * ny + yg);
    int e, row_begin, rows;
    if (!find_tile(offsets, e_first, e_count, kTileM, slot, e, row_begin, rows)) return;

    const int wave = threadIdx.x >> 6;
    const int units = N / (32 * (GATED ? 1 : NF));
    const int unit = block_y * 4 + wave;
    const bool active = unit < units;              // a wave past the last unit recomputes the last one, stores nothing
    const int u = active ? unit : units - 1;
    const int steps16 = K / 16;
    // fragment pair index and which half of the pair this wave reads
    const int pair = (GATED || NF == 2) ? u : (u >> 1);
    const int half = (GATED || NF == 2) ? 0 : (u & 1);
    // start of this wave's fragment stream; the same for all lanes, so it is handed over in scalar registers
    const char* wb = W + static_cast<size_t>(e - e_first) * expert_stride_bytes + block_offset_bytes +
                     (static_cast<size_t>(pair) * steps16 * 128 + half * 64) * 16;
    const uintptr_t wbi = reinterpret_cast<uintptr_t>(wb);
    const uint32_t wb_lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(wbi))));
    const uint32_t wb_hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(wbi >> 32))));
    const void* wave_w = reinterpret_cast<const void*>((static_cast<uintptr_t>(wb_hi) << 32) | static_cast<uintptr_t>(wb_lo));
    if (block_y * 4 >= units) return;              // past the last column group (uniform for the block)
    // The sweep over the reduction dimension starts at a step that depends on the expert and on the
    // chunk of 8 column groups only: blocks that share a weight stream or an activation tile walk it
    // together, other blocks are out of step with them.
    const unsigned col_chunk = static_cast<unsigned>(block_y) >> ((GATED || NF == 2) ? 3 : 4);   // same for both unit widths
    const unsigned key = static_cast<unsigned>(e) * 37u + col_chunk * 17u;
    switch ((rows + 31) >> 5) {
        case 1: ffn_tile<GATED, NF, 1>(lds, A, row_begin, rows, wave_w, C, K, N, unit, active, act, key); break;
        case 2: ffn_tile<GATED, NF, 2>(lds, A, row_begin, rows, wave_w, C, K, N, unit, active, act, key); break;
        case 3: ffn_tile<GATED, NF, 3>(lds, A, row_begin, rows, wave_w, C, K, N, unit, active, act, key); break;
        case 4: ffn_tile<GATED, NF, 4>(lds, A, row_begin, rows, wave_w, C, K, N, unit, active, act, key); break;
        case 5: ffn_tile<GATED, NF, 5>(lds, A, row_begin, rows, wave_w, C, K, N, unit, active, act, key); break;
        case 6: ffn_tile<GATED, NF, 6>(lds, A, row_begin, rows, wave_w, C, K, N, unit, active, act, key); break;
        case 7: ffn_tile<GATED, NF, 7>(lds, A, row_begin, rows, wave_w, C, K, N, unit, active, act, key); break;
        default: ffn_tile<GATED, NF, 8>(lds, A, row_begin, rows, wave_w, C, K, N, unit, active, act, key); break;
    }
}

// ------------------------------------------------------------------------------------------ fp32 FMA

constexpr int kF32Tile = 64;

template <bool GATED>
__global__ __launch_bounds__(256) void ffn_f32_kernel(const float* __restrict__ A, const int32_t* __restrict__ offsets,
                                                      int e_first, int e_count, const float* __restrict__ W,
                                                      size_t expert_stride_elems, size_t off_b0, size_t off_b1,
                                                      float* __restrict__ C, int K, int N, int act) {
    __shared__ float As[16][kF32Tile + 4];
    __shared__ float B0s[16][kF32Tile + 4];
    __shared__ float B1s[GATED ? 16 : 1][kF32Tile + 4];
    int e, row_begin, rows;
    if (!find_tile(offsets, e_first, e_count, kF32Tile, blockIdx.y, e, row_begin, rows)) return;
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
                      const void* W, size_t expert_stride_bytes, long max_rows, void* H, void* Yp, hipStream_t s,
                      hipEvent_t between) {
    if (max_rows <= 0 || e_count <= 0) return MOE_OK;
    const size_t df = static_cast<size_t>(c.d) * c.f;
    if (c.dtype == MOE_BF16) {
        // grid.x = row-tile slots (fastest varying, padded to the 8 XCDs so that the blocks sharing one
        // activation tile land on one XCD and its L2), grid.y = groups of 4 column units
        // one-dimensional grid: 8 XCDs x (groups of 4 row-tile slots per XCD) x (chunks of 8 column groups) x 32
        long slots = max_rows / kTileM + e_count;
        const int mt_shift = slots >= 32 ? 2 : slots >= 16 ? 1 : 0;   // row tiles per group: 4, 2 or 1
        const long tile_groups = (slots + (8L << mt_shift) - 1) / (8L << mt_shift);   // per XCD
        auto grid_for = [&](int col_groups, int& y_chunks) {
            const int ny = 32 >> mt_shift;
            y_chunks = (col_groups + ny - 1) / ny;
            return tile_groups * y_chunks * 32 * 8;
        };
        const size_t down_off = 2 * df * 2;
        dim3 block(256);
        int yc = 0;
        long blocks = grid_for((c.f / 32 + 3) / 4, yc);
        if (blocks > 0x7fffffffL) return fail(MOE_ERR_UNSUPPORTED, "too many blocks for one launch (%ld)", blocks);
        hipLaunchKernelGGL((ffn_mfma_kernel<true, 2>), dim3(static_cast<unsigned>(blocks)), block, 0, s,
                           static_cast<const uint16_t*>(Xp), offsets, e_first, e_count, static_cast<const char*>(W),
                           expert_stride_bytes, size_t(0), static_cast<uint16_t*>(H), c.d, c.f, c.act, yc, mt_shift);
        MOE_LAUNCH_CHECK("ffn_mfma_kernel<up>");
        if (between != nullptr) MOE_HIP_CHECK(hipEventRecord(between, s));
        // down-projection: narrow (32-column) units when wide ones would leave compute units idle
        const long tiles_hint = (max_rows + kTileM - 1) / kTileM > e_count ? (max_rows + kTileM - 1) / kTileM : e_count;
        const bool narrow = tiles_hint * ((c.d / 64 + 3) / 4) < 2 * 256;
        if (narrow) {
            blocks = grid_for((c.d / 32 + 3) / 4, yc);
            if (blocks > 0x7fffffffL) return fail(MOE_ERR_UNSUPPORTED, "too many blocks for one launch (%ld)", blocks);
            hipLaunchKernelGGL((ffn_mfma_kernel<false, 1>), dim3(static_cast<unsigned>(blocks)), block, 0, s,
                               static_cast<const uint16_t*>(H), offsets, e_first, e_count, static_cast<const char*>(W),
                               expert_stride_bytes, down_off, static_cast<uint16_t*>(Yp), c.f, c.d, c.act, yc, mt_shift);
        } else {
            blocks = grid_for((c.d / 64 + 3) / 4, yc);
            if (blocks > 0x7fffffffL) return fail(MOE_ERR_UNSUPPORTED, "too many blocks for one launch (%ld)", blocks);
            hipLaunchKernelGGL((ffn_mfma_kernel<false, 2>), dim3(static_cast<unsigned>(blocks)), block, 0, s,
                               static_cast<const uint16_t*>(H), offsets, e_first, e_count, static_cast<const char*>(W),
                               expert_stride_bytes, down_off, static_cast<uint16_t*>(Yp), c.f, c.d, c.act, yc, mt_shift);
        }
        MOE_LAUNCH_CHECK("ffn_mfma_kernel<down>");
        return MOE_OK;
    }
    const long slots = max_rows / kF32Tile + e_count;
    if (slots > 65535) return fail(MOE_ERR_UNSUPPORTED, "too many row tiles for one launch (%ld)", slots);
    const size_t stride = expert_stride_bytes / 4;
    const float* Wf = static_cast<const float*>(W);
    hipLaunchKernelGGL(ffn_f32_kernel<true>, dim3(c.f / kF32Tile, static_cast<unsigned>(slots)), dim3(256), 0, s,
                       static_cast<const float*>(Xp), offsets, e_first, e_count, Wf, stride, size_t(0), df,
                       static_cast<float*>(H), c.d, c.f, c.act);
    MOE_LAUNCH_CHECK("ffn_f32_kernel<up>");
    if (between != nullptr) MOE_HIP_CHECK(hipEventRecord(between, s));
    hipLaunchKernelGGL(ffn_f32_kernel<false>, dim3(c.d / kF32Tile, static_cast<unsigned>(slots)), dim3(256), 0, s,
                       static_cast<const float*>(H), offsets, e_first, e_count, Wf, stride, 2 * df, 2 * df,
                       static_cast<float*>(Yp), c.f, c.d, c.act);
    MOE_LAUNCH_CHECK("ffn_f32_kernel<down>");
    return MOE_OK;
}

}  // namespace moe
