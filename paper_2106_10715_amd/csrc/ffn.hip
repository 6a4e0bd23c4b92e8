// Expert feed-forward networks on the rows batched by expert (CPM-2 Section 2.1 / Table 1: each
// expert is a d_model -> d_ff -> d_model gated-GELU FFN; Section 6.2: an expert's work is
// proportional to its token count and its parameters form one equal-sized block):
//
//     H  = act(Xp W_gate[e]) * (Xp W_in[e])        "up"   grouped GEMM, epilogue fused
//     Yp = H W_out[e]                               "down" grouped GEMM
//
// bf16 path: 32x32x16 bf16 MFMA, fp32 accumulate.  One block = 128 rows of one expert x 4 waves;
// every wave owns its own output columns for all 128 rows, so a weight fragment is needed by exactly
// one wave: weights go HBM -> registers directly in pre-packed fragment order (no LDS, fully
// coalesced 1 KiB reads), only the activation tile is shared through LDS (stored in fragment order,
// conflict-free 16-byte reads).  With few rows per expert the layer is bound by streaming the
// weights once from HBM, which is what this layout is built for.
// fp32 path: plain LDS-tiled FMA kernel (small-shape correctness vehicle).
#include "common.h"

namespace moe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kKC = 64;                 // reduction elements staged per pipeline step (4 MFMA k-steps)
constexpr int kMB = kTileM / 32;        // 32-row MFMA blocks per tile

__device__ inline float act_fn(float z, int act) {
    if (act == 0) return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
    const float u = 0.79788456080286536f * (z + 0.044715f * z * z * z);
    return 0.5f * z * (1.0f + tanhf(u));
}

// Which (expert, row tile) a block works on: tile slot blockIdx.y counted over the experts
// [e_first, e_first + e_count) in order, tile_m rows per tile.  Returns false when the slot is past
// the last tile (uniform for the block).  Must be called by all threads of the block.
__device__ inline bool find_tile(const int32_t* __restrict__ offsets, int e_first, int e_count, int tile_m,
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
        const int target = blockIdx.y;
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
    row_begin = offsets[e_out] + sh_mt * tile_m;
    rows = min(tile_m, offsets[e_out + 1] - row_begin);
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

struct BFrags { uint4 v[kKC / 16][2]; };   // one pipeline step of one wave: 4 k-steps x 2 fragments

__device__ inline bf16x8 as_bf16x8(const uint4& u) { return __builtin_bit_cast(bf16x8, u); }

__device__ inline void load_b(BFrags& b, const uint4* __restrict__ wave_w, int chunk, int lane) {
    // fragments of one (column unit, k-step) are adjacent: [k-step][2][64 lanes] x 16 bytes
    const uint4* p = wave_w + static_cast<size_t>(chunk) * (kKC / 16) * 128 + lane;
#pragma unroll
    for (int ks = 0; ks < kKC / 16; ++ks) {
        b.v[ks][0] = p[ks * 128];
        b.v[ks][1] = p[ks * 128 + 64];
    }
}

struct ARegs { uint4 v[kMB]; };             // this thread's share of one activation tile step

__device__ inline void load_a(ARegs& a, const uint16_t* __restrict__ A, int K, int row_begin, int rows, int chunk,
                              int wave, int lane) {
    // thread (wave, lane) fetches, for each 32-row block mb, row mb*32 + lane%32, 8 elements at
    // k = chunk*64 + wave*16 + 8*(lane/32): exactly LDS slot (mb, k-step = wave, lane) of the fragment order
    const int kcol = chunk * kKC + wave * 16 + 8 * (lane >> 5);
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb) {
        const int r = mb * 32 + (lane & 31);
        if (r < rows)
            a.v[mb] = *reinterpret_cast<const uint4*>(A + static_cast<size_t>(row_begin + r) * K + kcol);
        else
            a.v[mb] = make_uint4(0, 0, 0, 0);
    }
}

__device__ inline void store_a(const ARegs& a, uint4* lds_buf, int wave, int lane) {
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb) lds_buf[(mb * (kKC / 16) + wave) * 64 + lane] = a.v[mb];
}

__device__ inline void mma_step(f32x16 (&acc)[kMB][2], const uint4* lds_buf, const BFrags& b, int lane) {
#pragma unroll
    for (int ks = 0; ks < kKC / 16; ++ks) {
        bf16x8 af[kMB];
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb) af[mb] = as_bf16x8(lds_buf[(mb * (kKC / 16) + ks) * 64 + lane]);
        const bf16x8 b0 = as_bf16x8(b.v[ks][0]), b1 = as_bf16x8(b.v[ks][1]);
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb) {
            acc[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mb], b0, acc[mb][0], 0, 0, 0);
            acc[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mb], b1, acc[mb][1], 0, 0, 0);
        }
    }
}

// C[rows of one expert tile, N] = A[rows, K] * B_e, B_e in packed fragment order.
// GATED: every wave unit is 32 output columns whose two fragments per k-step are (W_gate, W_in);
//        the epilogue writes act(gate) * in.   Otherwise a unit is 64 output columns.
template <bool GATED>
__global__ __launch_bounds__(256) void ffn_mfma_kernel(const uint16_t* __restrict__ A, const int32_t* __restrict__ offsets,
                                                       int e_first, int e_count, const char* __restrict__ W,
                                                       size_t expert_stride_bytes, size_t block_offset_bytes,
                                                       uint16_t* __restrict__ C, int K, int N, int act) {
    __shared__ uint4 lds[2][kMB * (kKC / 16) * 64];   // 2 x 16 KiB activation tiles in fragment order
    int e, row_begin, rows;
    if (!find_tile(offsets, e_first, e_count, kTileM, e, row_begin, rows)) return;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int unit_cols = GATED ? 32 : 64;
    const int units = N / unit_cols;
    const int unit = blockIdx.x * 4 + wave;
    const bool active = unit < units;              // idle waves still help staging the activation tile
    const int steps16 = K / 16;
    const uint4* wave_w = reinterpret_cast<const uint4*>(W + static_cast<size_t>(e - e_first) * expert_stride_bytes +
                                                         block_offset_bytes) +
                          static_cast<size_t>(active ? unit : 0) * steps16 * 128;
    const int chunks = K / kKC;

    f32x16 acc[kMB][2];
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][j][v] = 0.f;

    ARegs areg;
    BFrags b0, b1;
    load_a(areg, A, K, row_begin, rows, 0, wave, lane);
    if (active) load_b(b0, wave_w, 0, lane);
    store_a(areg, lds[0], wave, lane);
    __syncthreads();

    // two pipeline steps per iteration so the fragment registers ping-pong without copies
    int c = 0;
    for (; c + 1 < chunks; c += 2) {
        load_a(areg, A, K, row_begin, rows, c + 1, wave, lane);
        if (active) load_b(b1, wave_w, c + 1, lane);
        if (active) mma_step(acc, lds[0], b0, lane);
        store_a(areg, lds[1], wave, lane);
        __syncthreads();
        const bool more = c + 2 < chunks;
        if (more) {
            load_a(areg, A, K, row_begin, rows, c + 2, wave, lane);
            if (active) load_b(b0, wave_w, c + 2, lane);
        }
        if (active) mma_step(acc, lds[1], b1, lane);
        if (more) store_a(areg, lds[0], wave, lane);
        __syncthreads();
    }
    if (c < chunks && active) mma_step(acc, lds[0], b0, lane);   // odd number of steps: last one is staged in lds[0]
    if (!active) return;

    // accumulator layout of the 32x32 MFMA: lane holds column lane%32, rows 8*(v/4) + 4*(lane/32) + v%4
    const int col_in = lane & 31, row_in = 4 * (lane >> 5);
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = mb * 32 + 8 * (v >> 2) + row_in + (v & 3);
            if (r < rows) {
                uint16_t* crow = C + static_cast<size_t>(row_begin + r) * N;
                if (GATED) {
                    const float h = act_fn(acc[mb][0][v], act) * acc[mb][1][v];
                    crow[unit * 32 + col_in] = __builtin_bit_cast(uint16_t, static_cast<__bf16>(h));
                } else {
                    crow[unit * 64 + col_in] = __builtin_bit_cast(uint16_t, static_cast<__bf16>(acc[mb][0][v]));
                    crow[unit * 64 + 32 + col_in] = __builtin_bit_cast(uint16_t, static_cast<__bf16>(acc[mb][1][v]));
                }
            }
        }
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
    if (!find_tile(offsets, e_first, e_count, kF32Tile, e, row_begin, rows)) return;
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
        const long slots = max_rows / kTileM + e_count;
        if (slots > 65535) return fail(MOE_ERR_UNSUPPORTED, "too many row tiles for one launch (%ld)", slots);
        const size_t down_off = 2 * df * 2;
        dim3 block(256);
        dim3 grid_up((c.f / 32 + 3) / 4, static_cast<unsigned>(slots));
        hipLaunchKernelGGL(ffn_mfma_kernel<true>, grid_up, block, 0, s, static_cast<const uint16_t*>(Xp), offsets, e_first,
                           e_count, static_cast<const char*>(W), expert_stride_bytes, size_t(0),
                           static_cast<uint16_t*>(H), c.d, c.f, c.act);
        MOE_LAUNCH_CHECK("ffn_mfma_kernel<up>");
        if (between != nullptr) MOE_HIP_CHECK(hipEventRecord(between, s));
        dim3 grid_dn((c.d / 64 + 3) / 4, static_cast<unsigned>(slots));
        hipLaunchKernelGGL(ffn_mfma_kernel<false>, grid_dn, block, 0, s, static_cast<const uint16_t*>(H), offsets, e_first,
                           e_count, static_cast<const char*>(W), expert_stride_bytes, down_off,
                           static_cast<uint16_t*>(Yp), c.f, c.d, c.act);
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
