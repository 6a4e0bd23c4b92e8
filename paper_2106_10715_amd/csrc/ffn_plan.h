// Work list of one launch of the expert FFN kernels: which (expert, rows) every row tile covers, in the
// order the tiles are handed out.  Experts with more rows come first, so that the tiles that finish last are
// the short ones; an expert's rows are split evenly over its tiles (in multiples of 32 rows), not into full
// tiles and a small remainder.  Also clears the work counters of the two kernels that follow.
// The two kernels of a launch have a list each when their row tiles differ in height (else both read the first):
//   plan[0..7], plan[8..15] : next work item of each of the 8 queues, up and down kernel
//   plan[16], plan[17]      : number of tiles of the up and of the down kernel's list
//   plan[32 + 4 s ..]       : up kernel's tile s = (expert, first row, rows, row tiles of this expert)
//   plan[32 + 4 max_tiles + 4 s ..] : the same for the down kernel
#pragma once
#include "common.h"

namespace moe {

constexpr int kPlanHeader = 32;

// By one block of at least 256 threads (all of them must call; the first 256 work): offsets[e_first ..
// e_first + e_count] -> list `list` (0: up kernel, 1: down kernel) of the plan, in tiles of at most tile_m rows.
// `scratch` is LDS of the caller.  e_count <= 256.  The call for list 0 also clears the work counters.
__device__ inline void ffn_plan_block(const int32_t* offsets, int e_first, int e_count, int tile_m, int32_t* plan,
                                      int total_rows, int max_tiles, int (&scratch)[4][256], int list) {
    int (&n)[256] = scratch[0], (&first)[256] = scratch[1], (&order)[256] = scratch[2], (&tl)[256] = scratch[3];
    const int t = threadIdx.x;
    const bool worker = t < 256;
    int cnt = 0, lo = 0;
    if (worker && t < e_count) {
        // whatever the offsets hold, no tile may reach outside the total_rows rows or the work list
        lo = min(max(offsets[e_first + t], 0), total_rows);
        cnt = min(max(offsets[e_first + t + 1] - lo, 0), total_rows - lo);
    }
    if (worker) {
        n[t] = cnt;
        first[t] = lo;
        order[t] = t;
        tl[t] = 0;
    }
    __syncthreads();
    if (worker && t < e_count) {
        int rank = 0;                   // more rows first, equal counts by expert index: a permutation of 0..e_count-1
        for (int u = 0; u < e_count; ++u) rank += (n[u] > cnt || (n[u] == cnt && u < t)) ? 1 : 0;
        order[rank] = t;
    }
    __syncthreads();
    const int mine = worker ? order[t] : 0, my_n = worker && t < e_count ? n[mine] : 0;
    const int my_tiles = (my_n + tile_m - 1) / tile_m;
    if (worker) tl[t] = my_tiles;
    __syncthreads();
    if (!worker) return;
    int start = 0;
    const int upto = t < e_count ? t : e_count;
    for (int r = 0; r < upto; ++r) start += tl[r];
    if (my_tiles > 0) {
        const int per_tile = min(tile_m, ((my_n + my_tiles - 1) / my_tiles + 31) & ~31);
        int4* tiles = reinterpret_cast<int4*>(plan + kPlanHeader + 4 * list * max_tiles);
        for (int mt = 0; mt < my_tiles && start + mt < max_tiles; ++mt)
            tiles[start + mt] = make_int4(e_first + mine, first[mine] + mt * per_tile, min(per_tile, my_n - mt * per_tile), my_tiles);
    }
    if (t == 255) plan[16 + list] = min(start + my_tiles, max_tiles);
    if (list == 0 && t < 16) plan[t] = 0;
}

}  // namespace moe
