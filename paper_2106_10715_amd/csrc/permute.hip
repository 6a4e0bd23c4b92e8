// Batching of assignments by expert (CPM-2 Section 6.2: tokens are routed and batched to their
// experts before computation): a deterministic, stable counting sort of a = t*k + j by expert id,
// followed by the row gather Xp[row] = x[perm[row] / k].
//
//   1. chunk_hist_kernel : LDS histogram of each chunk of kPermChunk assignments
//   2. scan_kernel       : counts, offsets and, per chunk, the first row of every expert
//   3. scatter_kernel    : stable rank inside the chunk from wave ballots (no ordered atomics)
//   4. gather_rows_kernel: 16-byte-vector row copy
#include "common.h"
#include "ffn_plan.h"

#include <mutex>

// Scratch of moe_permute_static, the variant of moe_permute for callers that can neither allocate nor pass a
// workspace: the per-chunk expert histograms / running bases of the chunked kernels, [chunks][E] int32, for
// up to kStaticChunks chunks of kPermChunk assignments and 256 experts.  Every device the library runs on
// holds its own copy of the array (256 KiB) until the process ends.  In host code the name is only a handle
// for hipGetSymbolAddress, never an address.
constexpr int kStaticChunks = 256;
constexpr int kStaticExperts = 256;
static __device__ __align__(256) int32_t scratch[kStaticChunks * kStaticExperts];

namespace moe {
namespace {

__device__ inline int clamp_expert(int e, int E) { return min(max(e, 0), E - 1); }

__global__ __launch_bounds__(256) void chunk_hist_kernel(const int32_t* __restrict__ idx, int A, int E,
                                                         int32_t* __restrict__ chunk_hist) {
    __shared__ int hist[256];
    hist[threadIdx.x] = 0;
    __syncthreads();
    const int a0 = blockIdx.x * kPermChunk;
    for (int i = threadIdx.x; i < kPermChunk; i += 256) {
        const int a = a0 + i;
        if (a < A) atomicAdd(&hist[clamp_expert(idx[a], E)], 1);   // integer counts: order cannot matter
    }
    __syncthreads();
    if (threadIdx.x < E) chunk_hist[static_cast<size_t>(blockIdx.x) * E + threadIdx.x] = hist[threadIdx.x];
}

// One block; thread e walks the chunks of expert e, turning histograms into running bases.  The chunk
// histograms are read kScanBatch at a time (independent loads: one memory latency per batch, not per chunk).
constexpr int kScanBatch = 16;

__global__ __launch_bounds__(256) void scan_kernel(int32_t* __restrict__ chunk_hist, int chunks, int E,
                                                   int32_t* __restrict__ counts, int32_t* __restrict__ offsets) {
    __shared__ int total[256];
    __shared__ int start[257];
    const int e = threadIdx.x;
    int run = 0;
    if (e < E) {
        for (int b0 = 0; b0 < chunks; b0 += kScanBatch) {
            int h[kScanBatch];
#pragma unroll
            for (int i = 0; i < kScanBatch; ++i)
                h[i] = b0 + i < chunks ? chunk_hist[static_cast<size_t>(b0 + i) * E + e] : 0;
#pragma unroll
            for (int i = 0; i < kScanBatch; ++i) run += h[i];
        }
    }
    total[e] = e < E ? run : 0;
    __syncthreads();
    if (e == 0) {
        int acc = 0;
        for (int i = 0; i < E; ++i) { start[i] = acc; acc += total[i]; }
        start[E] = acc;
    }
    __syncthreads();
    if (e < E) {
        counts[e] = total[e];
        offsets[e] = start[e];
        int base = start[e];                   // first row of expert e in the chunk at hand: its rows in earlier chunks come first
        for (int b0 = 0; b0 < chunks; b0 += kScanBatch) {
            int h[kScanBatch];
#pragma unroll
            for (int i = 0; i < kScanBatch; ++i)
                h[i] = b0 + i < chunks ? chunk_hist[static_cast<size_t>(b0 + i) * E + e] : 0;
#pragma unroll
            for (int i = 0; i < kScanBatch; ++i) {
                if (b0 + i < chunks) chunk_hist[static_cast<size_t>(b0 + i) * E + e] = base;
                base += h[i];
            }
        }
    }
    if (e == 0) offsets[E] = start[E];
}

__global__ __launch_bounds__(256) void scatter_kernel(const int32_t* __restrict__ idx, int A, int E,
                                                      const int32_t* __restrict__ chunk_base,
                                                      int32_t* __restrict__ perm, int32_t* __restrict__ inv) {
    __shared__ int run[256];          // next free row of each expert for this chunk
    __shared__ int wcnt[4][256];      // per wave, rows each expert takes in the current round
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    run[threadIdx.x] = threadIdx.x < E ? chunk_base[static_cast<size_t>(blockIdx.x) * E + threadIdx.x] : 0;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) wcnt[wv][threadIdx.x] = 0;
    __syncthreads();
    int bits = 0;
    while ((1 << bits) < E) ++bits;
    const int a0 = blockIdx.x * kPermChunk;
    for (int round = 0; round < kPermChunk / 256; ++round) {
        const int a = a0 + round * 256 + threadIdx.x;
        const bool valid = a < A;
        const int e = valid ? clamp_expert(idx[a], E) : 0;
        // lanes of this wave that hold the same expert
        unsigned long long peers = __ballot(valid);
        for (int b = 0; b < bits; ++b) {
            const bool bit = (e >> b) & 1;
            const unsigned long long bal = __ballot(bit);
            peers &= bit ? bal : ~bal;
        }
        const int rank = __popcll(peers & ((1ull << lane) - 1ull));
        if (valid && rank == 0) wcnt[wave][e] = __popcll(peers);
        __syncthreads();
        if (valid) {
            int row = run[e] + rank;
            for (int wv = 0; wv < wave; ++wv) row += wcnt[wv][e];
            perm[row] = a;
            inv[a] = row;
        }
        __syncthreads();
        {
            const int t = threadIdx.x;
            run[t] += wcnt[0][t] + wcnt[1][t] + wcnt[2][t] + wcnt[3][t];
            wcnt[0][t] = 0; wcnt[1][t] = 0; wcnt[2][t] = 0; wcnt[3][t] = 0;
        }
        __syncthreads();
    }
}

// Short batches: the same three steps by one block of 16 waves, with no trip through memory between them:
// LDS histogram of all assignments, exclusive scan over the experts, then the stable scatter in rounds
// of 1024 assignments (rank inside the wave from ballots, waves in order, rounds in order).
constexpr int kSmallWaves = 16;
constexpr int kSmallMaxA = 16 * kSmallWaves * 64;      // beyond this the chunked kernels spread the work over the chip

__global__ __launch_bounds__(kSmallWaves * 64) void permute_small_kernel(const int32_t* __restrict__ idx, int A, int E,
                                                                         int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                                         int32_t* __restrict__ perm, int32_t* __restrict__ inv,
                                                                         int32_t* __restrict__ plan, int plan_max_tiles,
                                                                         int plan_tile_rows, int plan_tile_rows_down) {
    __shared__ int run[256];                       // histogram, then the next free row of each expert
    __shared__ int wcnt[kSmallWaves][256];         // per wave, rows each expert takes in the current round
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x < 256) {
        run[threadIdx.x] = 0;
#pragma unroll
        for (int wv = 0; wv < kSmallWaves; ++wv) wcnt[wv][threadIdx.x] = 0;
    }
    __syncthreads();
    for (int a = threadIdx.x; a < A; a += kSmallWaves * 64) atomicAdd(&run[clamp_expert(idx[a], E)], 1);   // integer counts: order cannot matter
    __syncthreads();
    if (wave == 0) {
        // exclusive scan of up to 256 counts by one wave: four experts per lane, then across the lanes
        int c[4], sum = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) { c[j] = run[4 * lane + j]; sum += c[j]; }
        int incl = sum;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        int start = incl - sum;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = 4 * lane + j;
            if (e < E) { counts[e] = c[j]; offsets[e] = start; }
            run[e] = start;
            start += c[j];
        }
        if (lane == 63) offsets[E] = incl;         // experts past E hold no assignment, so this is the total
    }
    __syncthreads();
    // the work list of the expert kernels that follow, when the caller wants it from here (saves a launch)
    if (plan != nullptr) {
        int (&scratch)[4][256] = reinterpret_cast<int (&)[4][256]>(wcnt);      // not in use yet; cleared again below
        ffn_plan_block(offsets, 0, E, plan_tile_rows, plan, A, plan_max_tiles, scratch, 0);
        if (plan_tile_rows_down != plan_tile_rows) {        // else the down kernel reads the up kernel's list
            __syncthreads();
            ffn_plan_block(offsets, 0, E, plan_tile_rows_down, plan, A, plan_max_tiles, scratch, 1);
        }
        __syncthreads();
        if (threadIdx.x < 256) {
#pragma unroll
            for (int wv = 0; wv < 4; ++wv) wcnt[wv][threadIdx.x] = 0;
        }
        __syncthreads();
    }
    int bits = 0;
    while ((1 << bits) < E) ++bits;
    for (int a0 = 0; a0 < A; a0 += kSmallWaves * 64) {
        const int a = a0 + threadIdx.x;
        const bool valid = a < A;
        const int e = valid ? clamp_expert(idx[a], E) : 0;
        unsigned long long peers = __ballot(valid);       // lanes of this wave that hold the same expert
        for (int b = 0; b < bits; ++b) {
            const bool bit = (e >> b) & 1;
            const unsigned long long bal = __ballot(bit);
            peers &= bit ? bal : ~bal;
        }
        const int rank = __popcll(peers & ((1ull << lane) - 1ull));
        if (valid && rank == 0) wcnt[wave][e] = __popcll(peers);
        __syncthreads();
        if (valid) {
            int row = run[e] + rank;
            for (int wv = 0; wv < wave; ++wv) row += wcnt[wv][e];
            perm[row] = a;
            inv[a] = row;
        }
        __syncthreads();
        if (threadIdx.x < 256) {
            int taken = 0;
#pragma unroll
            for (int wv = 0; wv < kSmallWaves; ++wv) { taken += wcnt[wv][threadIdx.x]; wcnt[wv][threadIdx.x] = 0; }
            run[threadIdx.x] += taken;
        }
        __syncthreads();
    }
}

// One block per destination row; 16-byte vectors, coalesced on both sides.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ perm,
                                                          int k, int vec_per_row, uint4* __restrict__ Xp) {
    const int row = blockIdx.x;
    const int t = perm[row] / k;
    const uint4* src = x + static_cast<size_t>(t) * vec_per_row;
    uint4* dst = Xp + static_cast<size_t>(row) * vec_per_row;
    // stored non-temporal: the rows are next read by the expert kernels, which want the L2 for themselves
    // (left there as dirty lines, the batch costs the up-projection 2.5 % at 128 tokens per expert)
    typedef unsigned int u4v __attribute__((ext_vector_type(4)));
    for (int v = threadIdx.x; v < vec_per_row; v += 256) {
        const uint4 piece = src[v];
        __builtin_nontemporal_store(u4v{piece.x, piece.y, piece.z, piece.w}, reinterpret_cast<u4v*>(dst + v));
    }
}

}  // namespace

int launch_permute(const moe_cfg& c, const void* x, const int32_t* idx, int32_t* counts, int32_t* offsets,
                   int32_t* perm, int32_t* inv, void* Xp, int32_t* chunk_hist, hipStream_t s, int32_t* plan,
                   int plan_max_tiles, bool* planned, int plan_tile_rows, int plan_tile_rows_down) {
    if (planned != nullptr) *planned = false;
    const int A = c.T * c.k;
    const int chunks = (A + kPermChunk - 1) / kPermChunk;
    if (A <= kSmallMaxA) {
        const bool with_plan = plan != nullptr && planned != nullptr && c.dtype == MOE_BF16 && A > 0;
        hipLaunchKernelGGL(permute_small_kernel, dim3(1), dim3(kSmallWaves * 64), 0, s, idx, A, c.E, counts, offsets, perm, inv,
                           with_plan ? plan : nullptr, plan_max_tiles, plan_tile_rows, plan_tile_rows_down);
        MOE_LAUNCH_CHECK("permute_small_kernel");
        if (with_plan) *planned = true;
    } else {
        if (chunk_hist == nullptr) return fail(MOE_ERR_WORKSPACE, "the batching of %d assignments needs scratch memory", A);
        hipLaunchKernelGGL(chunk_hist_kernel, dim3(chunks), dim3(256), 0, s, idx, A, c.E, chunk_hist);
        MOE_LAUNCH_CHECK("chunk_hist_kernel");
        hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(256), 0, s, chunk_hist, chunks, c.E, counts, offsets);
        MOE_LAUNCH_CHECK("scan_kernel");
        hipLaunchKernelGGL(scatter_kernel, dim3(chunks), dim3(256), 0, s, idx, A, c.E, chunk_hist, perm, inv);
        MOE_LAUNCH_CHECK("scatter_kernel");
    }
    if (chunks > 0) {
        if (Xp != nullptr) {
            const int vec_per_row = static_cast<int>(c.d * elem_size(c) / 16);
            hipLaunchKernelGGL(gather_rows_kernel, dim3(A), dim3(256), 0, s, static_cast<const uint4*>(x), perm, c.k,
                               vec_per_row, static_cast<uint4*>(Xp));
            MOE_LAUNCH_CHECK("gather_rows_kernel");
        }
    }
    return MOE_OK;
}

long permute_static_max_assignments() { return static_cast<long>(kStaticChunks) * kPermChunk; }

int launch_permute_static(const moe_cfg& c, const void* x, const int32_t* idx, int32_t* counts, int32_t* offsets,
                          int32_t* perm, int32_t* inv, void* Xp, hipStream_t s) {
    const long A = static_cast<long>(c.T) * c.k;
    const long chunks = (A + kPermChunk - 1) / kPermChunk;
    if (chunks > kStaticChunks || c.E > kStaticExperts)
        return fail(MOE_ERR_WORKSPACE, "moe_permute_static batches at most %ld assignments over at most %d experts "
                    "(got %ld and %d): its scratch is a fixed array; use moe_permute with a workspace",
                    permute_static_max_assignments(), kStaticExperts, A, c.E);
    // the array's address on the current device, looked up once per device
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static int32_t* on_device[kMaxDevices] = {};
    int dev = 0;
    MOE_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(MOE_ERR_UNSUPPORTED, "device %d: only devices 0..%d are supported", dev, kMaxDevices - 1);
    int32_t* ptr = nullptr;
    {
        std::lock_guard<std::mutex> guard(lock);
        if (on_device[dev] == nullptr) {
            void* p = nullptr;
            MOE_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            if (p == nullptr) return fail(MOE_ERR_HIP, "hipGetSymbolAddress returned no address for the scratch array");
            on_device[dev] = static_cast<int32_t*>(p);
        }
        ptr = on_device[dev];
    }
    // Nothing has to be cleared: the histogram kernel writes all chunks x E entries the two kernels after it
    // read, whatever an earlier call left in the array.
    return launch_permute(c, x, idx, counts, offsets, perm, inv, Xp, ptr, s);
}

}  // namespace moe
