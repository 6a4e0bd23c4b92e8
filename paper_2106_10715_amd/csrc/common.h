// Shared host-side declarations of the moe355 library: error reporting, argument checks,
// workspace layout and the launchers each stage file defines.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "moe355.h"

namespace moe {

// Records a message for moe_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

#define MOE_HIP_CHECK(expr)                                                                   \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return ::moe::fail(MOE_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));   \
    } while (0)

#define MOE_LAUNCH_CHECK(name)                                                                \
    do {                                                                                      \
        hipError_t e_ = hipGetLastError();                                                    \
        if (e_ != hipSuccess)                                                                 \
            return ::moe::fail(MOE_ERR_HIP, "launch of %s failed: %s", name, hipGetErrorString(e_)); \
    } while (0)

int check_cfg(const moe_cfg* cfg);

// What the launchers need to know about a device, looked up once per device (under a lock) and kept.
struct DeviceInfo {
    int compute_units = 256;
};
// The current device and its entry; MOE_ERR_HIP (message recorded) if the device cannot be queried.
int device_info(int* device, const DeviceInfo** info);

inline size_t elem_size(const moe_cfg& c) { return c.dtype == MOE_BF16 ? 2 : 4; }
inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Assignments handled by one block of the histogram / scatter kernels of the permutation.
constexpr int kPermChunk = 1024;
// Rows of one expert segment covered by one block of the FFN kernels.
constexpr int kTileM = 256;

// Byte offsets of every region inside the caller's workspace.
struct WsLayout {
    size_t H;          // [A, f] dtype: gated intermediate of the expert FFNs
    size_t Xp;         // [A, d] dtype
    size_t Yp;         // [A, d] dtype
    size_t idx;        // [A] int32
    size_t w;          // [A] fp32
    size_t counts;     // [E] int32
    size_t offsets;    // [E+1] int32
    size_t perm;       // [A] int32
    size_t inv;        // [A] int32
    size_t chunk_hist; // [chunks, E] int32: per-chunk expert histograms, then per-chunk bases
    size_t route;      // gate projection in MFMA fragment order + per-group column sums of squares
    size_t ffn_plan;   // work list and work counters of the expert FFN kernels
    size_t total;
};
WsLayout ws_layout(const moe_cfg& c);

// ---- launchers (each enqueues on `s` and returns MOE_OK or an error already recorded) ----
// `scratch`: route_scratch_bytes(c) bytes of workspace (the gate re-packed for the matrix cores).
size_t route_scratch_bytes(const moe_cfg& c);
// Columns of the gate matrix: E for the projection gate, log2(E) sign bits for the hashing gate.
int gate_columns(const moe_cfg& c);
// Wg: the gate matrix, or (c.gate_packed) the block launch_pack_gate wrote, gate_packed_bytes(c) bytes.
int launch_route(const moe_cfg& c, const void* x, const void* Wg, const float* bias, int32_t* idx, float* w,
                 void* scratch, hipStream_t s);
size_t gate_packed_bytes(const moe_cfg& c);
int launch_pack_gate(const moe_cfg& c, const void* Wg, void* packed, hipStream_t s);
int launch_permute(const moe_cfg& c, const void* x, const int32_t* idx, int32_t* counts, int32_t* offsets,
                   int32_t* perm, int32_t* inv, void* Xp, int32_t* chunk_hist, hipStream_t s, int32_t* plan = nullptr,
                   int plan_max_tiles = 0, bool* planned = nullptr, int plan_tile_rows = kTileM,
                   int plan_tile_rows_down = kTileM);
// plan/planned: for short bf16 batches the kernel that batches the tokens also writes the work list of the expert
// FFN launch over all experts that follows (room for plan_max_tiles row tiles) and sets *planned; the caller then
// passes plan_ready to launch_expert_ffn.
// The same with the chunk histograms in a fixed array of the library instead of the caller's workspace (at most
// permute_static_max_assignments() assignments); never writes a work list.
int launch_permute_static(const moe_cfg& c, const void* x, const int32_t* idx, int32_t* counts, int32_t* offsets,
                          int32_t* perm, int32_t* inv, void* Xp, hipStream_t s);
long permute_static_max_assignments();
int launch_pack(const moe_cfg& c, const void* Win, const void* Wgate, const void* Wout, void* packed, hipStream_t s);
// Runs the FFN of experts [e_first, e_first + e_count); W points at the packed block of e_first and
// consecutive experts are expert_stride_bytes apart.  max_rows bounds the rows those experts can hold
// (it sizes the grid; blocks past the real row count exit).
// `between`, if not null, is recorded on `s` after the up kernel and before the down kernel;
// `before_up`, if not null, right before the up kernel.
int launch_expert_ffn(const moe_cfg& c, const void* Xp, const int32_t* offsets, int e_first, int e_count,
                      const void* W, size_t expert_stride_bytes, long max_rows, void* H, void* Yp, int32_t* plan,
                      hipStream_t s, hipEvent_t between = nullptr, hipEvent_t before_up = nullptr,
                      const int32_t* row_map = nullptr, bool plan_ready = false, const int32_t* gather = nullptr);
// gather (bf16 only): Xp is then the token array x[T, d] itself and batched row r is its row gather[r] / k (gather = the
// perm written by the batching step), so the batched copy of the activations need not exist; row tiles are then
// ffn_tile_rows(true) rows high instead of ffn_tile_rows(false), and a work list written elsewhere (plan_ready) must
// have been cut to that height.
int ffn_tile_rows(bool gather);
// Height of the down-projection's row tiles for a launch over e_count experts with at most max_rows rows in all (the two
// kernels have a tile list each); n_cu: compute units of the device.
int ffn_down_tile_rows(const moe_cfg& c, int e_count, long max_rows, int tile_m_up, int n_cu);
// row_map (bf16 only): row r of the batched order is written to row row_map[r] of Yp instead of row r, which
// turns the down-projection's output into the layer's output when no weighting follows (see moe_layer_forward).
// `plan`: ffn_plan_bytes(c) bytes of workspace, rewritten by every launch_expert_ffn (room for ffn_plan_tiles(c) row tiles).
size_t ffn_plan_tiles(const moe_cfg& c);
size_t ffn_plan_bytes(const moe_cfg& c);
// Greedy execution order of the non-empty experts (host arrays); see schedule.hip.
int schedule_order(const int32_t* counts, int E, double tokens_per_load, int K, int32_t* order, int* n_order,
                   int* satisfiable);
// Slot and load decision for every expert of a call when slots keep their experts; see schedule.hip.
int plan_slots(const int32_t* order, int n, int K, int32_t* slot_expert, int64_t* slot_tick, int64_t* tick,
               int32_t* slot_of, int32_t* load);
int launch_combine(const moe_cfg& c, const void* Yp, const int32_t* inv, const float* w, void* y, hipStream_t s);

}  // namespace moe
