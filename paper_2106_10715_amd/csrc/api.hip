// C-ABI entry points of the moe355 library: argument checks, workspace carving, and the host
// side of the two execution modes of the layer (CPM-2 Section 6: experts resident on the device, or
// kept in CPU memory and loaded on a second stream while earlier experts compute).
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>

#include "common.h"

namespace moe {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = '\0'; }

int device_info(int* device, const DeviceInfo** info) {
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static DeviceInfo table[kMaxDevices];
    static bool known[kMaxDevices] = {};
    int dev = 0;
    MOE_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(MOE_ERR_UNSUPPORTED, "device %d: only devices 0..%d are supported", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> guard(lock);
    if (!known[dev]) {
        int n = 0;
        MOE_HIP_CHECK(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
        table[dev].compute_units = n > 0 ? n : 256;
        known[dev] = true;
    }
    *device = dev;
    *info = &table[dev];
    return MOE_OK;
}

int check_cfg(const moe_cfg* c) {
    if (c == nullptr) return fail(MOE_ERR_INVALID_ARG, "cfg is NULL");
    if (c->dtype != MOE_F32 && c->dtype != MOE_BF16) return fail(MOE_ERR_INVALID_ARG, "dtype must be MOE_F32 or MOE_BF16");
    if (c->T < 0) return fail(MOE_ERR_INVALID_ARG, "T must be >= 0 (got %d)", c->T);
    if (c->d <= 0 || c->d % 64 != 0) return fail(MOE_ERR_INVALID_ARG, "d must be a positive multiple of 64 (got %d)", c->d);
    if (c->f <= 0 || c->f % 64 != 0) return fail(MOE_ERR_INVALID_ARG, "f must be a positive multiple of 64 (got %d)", c->f);
    if (c->E < 1 || c->E > 256) return fail(MOE_ERR_INVALID_ARG, "E must be in [1, 256] (got %d)", c->E);
    if (c->k < 1 || c->k > 8 || c->k > c->E) return fail(MOE_ERR_INVALID_ARG, "k must be in [1, min(E, 8)] (got %d)", c->k);
    if (c->renorm != 0 && c->renorm != 1) return fail(MOE_ERR_INVALID_ARG, "renorm must be 0 or 1");
    if (c->act != 0 && c->act != 1) return fail(MOE_ERR_INVALID_ARG, "act must be 0 (erf GELU) or 1 (tanh GELU)");
    if (c->gate != MOE_GATE_TOPK && c->gate != MOE_GATE_HASH) return fail(MOE_ERR_INVALID_ARG, "gate must be MOE_GATE_TOPK or MOE_GATE_HASH");
    if (c->gate == MOE_GATE_HASH && (c->E < 2 || (c->E & (c->E - 1)) != 0 || c->k != 1))
        return fail(MOE_ERR_INVALID_ARG, "the hashing gate needs E a power of two >= 2 and k = 1 (got E = %d, k = %d)", c->E, c->k);
    if (c->gate_packed != 0 && c->gate_packed != 1) return fail(MOE_ERR_INVALID_ARG, "gate_packed must be 0 or 1");
    const long long A = static_cast<long long>(c->T) * c->k;
    const long long widest = c->d > c->f ? c->d : c->f;
    if (A * widest >= (1LL << 31)) return fail(MOE_ERR_INVALID_ARG, "T*k*max(d,f) must stay below 2^31");
    return MOE_OK;
}

WsLayout ws_layout(const moe_cfg& c) {
    const size_t A = static_cast<size_t>(c.T) * c.k, es = elem_size(c);
    const size_t chunks = (A + kPermChunk - 1) / kPermChunk;
    WsLayout L;
    size_t at = 0;
    auto take = [&at](size_t bytes) { const size_t o = at; at += align256(bytes); return o; };
    L.H = take(A * c.f * es);
    L.Xp = take(A * c.d * es);
    L.Yp = take(A * c.d * es);
    L.idx = take(A * 4);
    L.w = take(A * 4);
    L.counts = take(static_cast<size_t>(c.E) * 4);
    L.offsets = take(static_cast<size_t>(c.E + 1) * 4);
    L.perm = take(A * 4);
    L.inv = take(A * 4);
    L.chunk_hist = take((chunks > 0 ? chunks : 1) * c.E * 4);
    L.route = take(route_scratch_bytes(c));
    L.ffn_plan = take(ffn_plan_bytes(c));
    L.total = at > 0 ? at : 256;
    return L;
}

}  // namespace moe

using namespace moe;

constexpr int kMaxSlots = 64;

struct moe_stream_ctx {
    moe_cfg cfg;
    const char* host_experts;
    size_t expert_bytes;
    char* dev_slots;
    int K;
    int device;
    // Loads alternate between two copy streams: after every copy the stream has an event to process (the compute
    // stream waits for it) before its next copy may start, some 30 us during which the link would idle; with two
    // streams the other one's copy is running meanwhile (measured on 32 copies of 240 MiB: 141.97 ms with one
    // stream, 141.13 ms with two, 140.82 ms for the bare copies).
    // The streams are created when the first load needs them: a context that shares another one's loader never
    // creates any (HIP maps all streams of a process onto a few hardware queues, 4 by default, and a copy stream
    // that lands on the hardware queue of the compute stream waits behind its kernels).
    hipStream_t copy_streams[2];
    bool owns_copy_streams;           // false: the streams belong to another context (moe_stream_ctx_share_loader)
    moe_stream_ctx* loader;           // the context whose streams are used, if not this one's own
    int next_copy;                    // which of the two takes the next load
    int slot_writer[kMaxSlots];       // copy stream of the last load into each slot; -1 once a compute has read it
    hipEvent_t loaded[kMaxSlots];     // copy into slot s finished
    hipEvent_t released[kMaxSlots];   // compute that read slot s finished
    bool released_valid[kMaxSlots];
    // Slot reuse: every release is recorded on the compute stream and numbered; a copy stream that has waited for
    // release number n has waited for all releases up to n recorded on that same stream (a stream runs in order),
    // so a copy into a slot needs a wait only if the slot's last release is newer than that.
    int64_t release_seq[kMaxSlots];   // number of the last release recorded for each slot (0: never used)
    int64_t seq;                      // releases recorded so far
    int64_t copy_waited_seq[2];       // each copy stream has waited for the release with this number
    hipStream_t release_stream;       // the compute stream those numbers belong to
    bool keep;                        // slots keep their experts between calls
    int32_t slot_expert[kMaxSlots];   // expert held by each slot, -1 = none (only meaningful with keep)
    int64_t slot_tick[kMaxSlots];     // when each slot was last used
    int64_t tick;
    int n_order;                      // experts run by the last call
    hipEvent_t first_copy, last_copy[2];
    int timed_streams;                // bit q: last_copy[q] was recorded by the last call
    bool timed;
    int32_t* h_counts;         // pinned [256]
    int n_loaded;
    int policy;                // MOE_ORDER_ASCENDING or MOE_ORDER_GREEDY
    double tokens_per_load;    // for the greedy order: tokens whose computation lasts as long as one load
    int order_K;               // K of the order's second constraint
    int satisfiable;           // whether the last greedy order met both constraints
    int32_t order[256];
};

// Event timing of resident layer calls (measurement aid): the caller's object, filled by moe_layer_forward_timed.
constexpr int kStageEvents = 6;   // before route, after route, permute, up, down, combine
struct moe_timer {
    int mode = MOE_TIME_STAGES;
    int cap = 0, n = 0;
    hipEvent_t* ev = nullptr;     // [cap][kStageEvents]
};

#define REQUIRE(ptr, name) \
    if ((ptr) == nullptr) return fail(MOE_ERR_INVALID_ARG, "%s is NULL", name)
#define REQUIRE_ALIGNED(ptr, name) \
    if (!aligned16(ptr)) return fail(MOE_ERR_INVALID_ARG, "%s must be 16-byte aligned", name)

extern "C" {

const char* moe_last_error(void) { return g_err; }

int moe_workspace_bytes(const moe_cfg* cfg, size_t* bytes) {
    if (int rc = check_cfg(cfg)) return rc;
    REQUIRE(bytes, "bytes");
    *bytes = ws_layout(*cfg).total;
    return MOE_OK;
}

int moe_expert_bytes(const moe_cfg* cfg, size_t* bytes) {
    if (int rc = check_cfg(cfg)) return rc;
    REQUIRE(bytes, "bytes");
    *bytes = 3 * static_cast<size_t>(cfg->d) * cfg->f * elem_size(*cfg);
    return MOE_OK;
}

int moe_pack_weights(const moe_cfg* cfg, const void* W_in_e, const void* W_gate_e, const void* W_out_e,
                     void* packed_e, void* stream) {
    if (int rc = check_cfg(cfg)) return rc;
    REQUIRE(W_in_e, "W_in_e"); REQUIRE(W_gate_e, "W_gate_e"); REQUIRE(W_out_e, "W_out_e"); REQUIRE(packed_e, "packed_e");
    REQUIRE_ALIGNED(W_in_e, "W_in_e"); REQUIRE_ALIGNED(W_gate_e, "W_gate_e"); REQUIRE_ALIGNED(W_out_e, "W_out_e");
    REQUIRE_ALIGNED(packed_e, "packed_e");
    return launch_pack(*cfg, W_in_e, W_gate_e, W_out_e, packed_e, static_cast<hipStream_t>(stream));
}

int moe_gate_bytes(const moe_cfg* cfg, size_t* bytes) {
    if (int rc = check_cfg(cfg)) return rc;
    REQUIRE(bytes, "bytes");
    *bytes = gate_packed_bytes(*cfg);
    return MOE_OK;
}

int moe_pack_gate(const moe_cfg* cfg, const void* W_g, void* gate_packed, void* stream) {
    if (int rc = check_cfg(cfg)) return rc;
    REQUIRE(W_g, "W_g"); REQUIRE(gate_packed, "gate_packed");
    REQUIRE_ALIGNED(W_g, "W_g");
    if ((reinterpret_cast<uintptr_t>(gate_packed) & 255) != 0) return fail(MOE_ERR_INVALID_ARG, "gate_packed must be 256-byte aligned");
    return launch_pack_gate(*cfg, W_g, gate_packed, static_cast<hipStream_t>(stream));
}

int moe_route(const moe_cfg* cfg, const void* x, const void* W_g, const float* gate_bias, int32_t* idx, float* w,
              void* ws, void* stream) {
    if (int rc = check_cfg(cfg)) return rc;
    REQUIRE(W_g, "W_g");
    if (cfg->gate_packed) REQUIRE_ALIGNED(W_g, "W_g (packed gate)");
    if (cfg->T == 0) return MOE_OK;
    REQUIRE(x, "x"); REQUIRE(idx, "idx"); REQUIRE(w, "w"); REQUIRE(ws, "ws");
    REQUIRE_ALIGNED(x, "x"); REQUIRE_ALIGNED(ws, "ws");
    if (cfg->gate == MOE_GATE_HASH && gate_bias != nullptr)
        return fail(MOE_ERR_INVALID_ARG, "the hashing gate takes no bias");
    return launch_route(*cfg, x, W_g, gate_bias, idx, w, static_cast<char*>(ws) + ws_layout(*cfg).route,
                        static_cast<hipStream_t>(stream));
}

int moe_permute(const moe_cfg* cfg, const void* x, const int32_t* idx, int32_t* counts, int32_t* offsets,
                int32_t* perm, int32_t* inv, void* Xp, void* ws, void* stream) {
    if (int rc = check_cfg(cfg)) return rc;
    REQUIRE(counts, "counts"); REQUIRE(offsets, "offsets"); REQUIRE(ws, "ws");
    if (cfg->T > 0) {
        REQUIRE(idx, "idx"); REQUIRE(perm, "perm"); REQUIRE(inv, "inv");
        if (Xp != nullptr) { REQUIRE(x, "x"); REQUIRE_ALIGNED(x, "x"); REQUIRE_ALIGNED(Xp, "Xp"); }
    }
    const WsLayout L = ws_layout(*cfg);
    return launch_permute(*cfg, x, idx, counts, offsets, perm, inv, Xp,
                          reinterpret_cast<int32_t*>(static_cast<char*>(ws) + L.chunk_hist),
                          static_cast<hipStream_t>(stream));
}

int moe_permute_static(const moe_cfg* cfg, const void* x, const int32_t* idx, int32_t* counts, int32_t* offsets,
                       int32_t* perm, int32_t* inv, void* Xp, void* stream) {
    if (int rc = check_cfg(cfg)) return rc;
    REQUIRE(counts, "counts"); REQUIRE(offsets, "offsets");
    if (cfg->T > 0) {
        REQUIRE(idx, "idx"); REQUIRE(perm, "perm"); REQUIRE(inv, "inv");
        if (Xp != nullptr) { REQUIRE(x, "x"); REQUIRE_ALIGNED(x, "x"); REQUIRE_ALIGNED(Xp, "Xp"); }
    }
    return launch_permute_static(*cfg, x, idx, counts, offsets, perm, inv, Xp, static_cast<hipStream_t>(stream));
}

int moe_expert_ffn(const moe_cfg* cfg, const void* Xp, const int32_t* offsets, const void* W_packed, void* Yp,
                   void* ws, void* stream) {
    if (int rc = check_cfg(cfg)) return rc;
    REQUIRE(offsets, "offsets");
    if (cfg->T == 0) return MOE_OK;
    REQUIRE(Xp, "Xp"); REQUIRE(W_packed, "W_packed"); REQUIRE(Yp, "Yp"); REQUIRE(ws, "ws");
    REQUIRE_ALIGNED(Xp, "Xp"); REQUIRE_ALIGNED(W_packed, "W_packed"); REQUIRE_ALIGNED(Yp, "Yp"); REQUIRE_ALIGNED(ws, "ws");
    const WsLayout L = ws_layout(*cfg);
    size_t eb = 0;
    moe_expert_bytes(cfg, &eb);
    return launch_expert_ffn(*cfg, Xp, offsets, 0, cfg->E, W_packed, eb, static_cast<long>(cfg->T) * cfg->k,
                             static_cast<char*>(ws) + L.H, Yp,
                             reinterpret_cast<int32_t*>(static_cast<char*>(ws) + L.ffn_plan), static_cast<hipStream_t>(stream));
}

int moe_combine(const moe_cfg* cfg, const void* Yp, const int32_t* inv, const float* w, void* y, void* stream) {
    if (int rc = check_cfg(cfg)) return rc;
    if (cfg->T == 0) return MOE_OK;
    REQUIRE(Yp, "Yp"); REQUIRE(inv, "inv"); REQUIRE(w, "w"); REQUIRE(y, "y");
    REQUIRE_ALIGNED(Yp, "Yp"); REQUIRE_ALIGNED(y, "y");
    return launch_combine(*cfg, Yp, inv, w, y, static_cast<hipStream_t>(stream));
}

}  // extern "C"

namespace {

// Forgets what the slots of a streamed context hold unless the call that planned them got all its copies
// enqueued: a slot marked as holding an expert whose copy was never issued would be computed from as it is.
struct SlotGuard {
    moe_stream_ctx* ctx;
    bool ok = false;
    ~SlotGuard() {
        if (ctx != nullptr && !ok)
            for (int i = 0; i < kMaxSlots; ++i) ctx->slot_expert[i] = -1;
    }
};

// Records that the compute on `s` which read `slot` is done (everything enqueued on `s` so far).
int record_release(moe_stream_ctx* ctx, int slot, hipStream_t s) {
    MOE_HIP_CHECK(hipEventRecord(ctx->released[slot], s));
    ctx->released_valid[slot] = true;
    ctx->release_seq[slot] = ++ctx->seq;
    ctx->slot_writer[slot] = -1;
    return MOE_OK;
}

// Enqueues the copy of expert e into `slot` on the copy stream whose turn it is.  The copy must follow the slot's
// last reader (a wait for its release, unless that stream has already waited for this or a later release of the
// compute stream) and, if the slot was loaded on the other copy stream and never read since (a load requested
// ahead that turned out not to be needed), that load.
int enqueue_load(moe_stream_ctx* ctx, int e, int slot) {
    const int q = ctx->next_copy;
    ctx->next_copy ^= 1;
    if (ctx->copy_streams[q] == nullptr) {
        moe_stream_ctx* owner = ctx->loader != nullptr ? ctx->loader : ctx;
        if (owner->copy_streams[q] == nullptr)
            MOE_HIP_CHECK(hipStreamCreateWithFlags(&owner->copy_streams[q], hipStreamNonBlocking));
        ctx->copy_streams[q] = owner->copy_streams[q];
    }
    hipStream_t cs = ctx->copy_streams[q];
    if (ctx->released_valid[slot] && ctx->release_seq[slot] > ctx->copy_waited_seq[q]) {
        MOE_HIP_CHECK(hipStreamWaitEvent(cs, ctx->released[slot], 0));
        ctx->copy_waited_seq[q] = ctx->release_seq[slot];
    }
    if (ctx->slot_writer[slot] >= 0 && ctx->slot_writer[slot] != q) MOE_HIP_CHECK(hipStreamWaitEvent(cs, ctx->loaded[slot], 0));
    if (ctx->n_loaded == 0) MOE_HIP_CHECK(hipEventRecord(ctx->first_copy, cs));
    MOE_HIP_CHECK(hipMemcpyAsync(ctx->dev_slots + static_cast<size_t>(slot) * ctx->expert_bytes,
                                 ctx->host_experts + static_cast<size_t>(e) * ctx->expert_bytes, ctx->expert_bytes,
                                 hipMemcpyHostToDevice, cs));
    MOE_HIP_CHECK(hipEventRecord(ctx->loaded[slot], cs));
    ctx->slot_writer[slot] = q;
    ++ctx->n_loaded;
    return MOE_OK;
}

// The layer; `timer` (resident mode only) receives this call's events if it has room.
int layer_forward(const moe_cfg* cfg, const void* x, const void* W_g, const float* gate_bias, const void* W_packed,
                  moe_stream_ctx* sctx, void* y, void* ws, void* stream, moe_timer* timer) {
    if (int rc = check_cfg(cfg)) return rc;
    REQUIRE(W_g, "W_g");
    if (cfg->gate_packed) REQUIRE_ALIGNED(W_g, "W_g (packed gate)");
    if (sctx == nullptr) { REQUIRE(W_packed, "W_packed (resident mode)"); REQUIRE_ALIGNED(W_packed, "W_packed"); }
    if (sctx != nullptr &&
        (sctx->cfg.d != cfg->d || sctx->cfg.f != cfg->f || sctx->cfg.E != cfg->E || sctx->cfg.dtype != cfg->dtype))
        return fail(MOE_ERR_INVALID_ARG, "stream context was created for another d/f/E/dtype");
    if (cfg->gate == MOE_GATE_HASH && gate_bias != nullptr)
        return fail(MOE_ERR_INVALID_ARG, "the hashing gate takes no bias");
    if (cfg->T == 0) return MOE_OK;
    REQUIRE(x, "x"); REQUIRE(y, "y"); REQUIRE(ws, "ws");
    REQUIRE_ALIGNED(x, "x"); REQUIRE_ALIGNED(y, "y");
    if ((reinterpret_cast<uintptr_t>(ws) & 255) != 0) return fail(MOE_ERR_WORKSPACE, "ws must be 256-byte aligned");

    const moe_cfg& c = *cfg;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const WsLayout L = ws_layout(c);
    char* base = static_cast<char*>(ws);
    int32_t* idx = reinterpret_cast<int32_t*>(base + L.idx);
    float* w = reinterpret_cast<float*>(base + L.w);
    int32_t* counts = reinterpret_cast<int32_t*>(base + L.counts);
    int32_t* offsets = reinterpret_cast<int32_t*>(base + L.offsets);
    int32_t* perm = reinterpret_cast<int32_t*>(base + L.perm);
    int32_t* inv = reinterpret_cast<int32_t*>(base + L.inv);
    const long A = static_cast<long>(c.T) * c.k;
    size_t eb = 0;
    moe_expert_bytes(cfg, &eb);

    // One expert per token with weight exactly 1 (top-1 with weights renormalised over the selection, or the
    // hashing gate): the combine step would only move row inv[t] of the batched results to row t.  The
    // down-projection then stores its rows at their tokens' places itself (perm[r] is the token of batched
    // row r) and the combine kernel is not run; the bytes written are the same ones.
    const bool direct = c.dtype == MOE_BF16 && c.k == 1 && (c.renorm == 1 || c.gate == MOE_GATE_HASH);
    void* ffn_out = direct ? y : static_cast<void*>(base + L.Yp);
    const int32_t* row_map = direct ? perm : nullptr;
    // With few rows per expert (the layer is then bound by streaming the weights, and every microsecond beside the
    // expert kernels counts) the up-projection reads its rows from x through the permutation itself: the batched
    // copy Xp is neither written nor read.  Row tiles are then slightly lower, which costs experts with many rows
    // an extra pass over their weights, hence the bound on the mean.
    const bool gather_rows = c.dtype == MOE_BF16 && A / c.E <= 160;
    const int32_t* gather = gather_rows ? perm : nullptr;
    const void* ffn_in = gather_rows ? x : static_cast<const void*>(base + L.Xp);

    int early = -1;                // streamed mode: the expert requested before routing, if any
    if (sctx != nullptr) {
        // the release numbers are only ordered among releases of one compute stream: on another stream, wait for
        // every slot's last reader once and start over
        if (sctx->release_stream != s) {
            for (int q = 0; q < 2; ++q) {
                for (int i = 0; i < sctx->K && sctx->copy_streams[q] != nullptr; ++i)
                    if (sctx->released_valid[i]) MOE_HIP_CHECK(hipStreamWaitEvent(sctx->copy_streams[q], sctx->released[i], 0));
                // (a stream that does not exist yet has no copies on it; what it has "waited for" only matters
                // for releases recorded from now on, which carry higher numbers)
                sctx->copy_waited_seq[q] = sctx->copy_streams[q] != nullptr ? sctx->seq : 0;
            }
            sctx->release_stream = s;
        }
        sctx->n_loaded = 0;
        // Every expert but the first is loaded while earlier ones compute (Section 6.2); the first load has
        // nothing of its own call to hide behind except the routing.  When every call reloads every expert in
        // ascending order, the first expert of the previous call is very likely the first of this one: its load is
        // requested now, before the gate runs.  (A wrong guess costs one wasted copy; the slot is loaded again.)
        if (!sctx->keep && sctx->policy == MOE_ORDER_ASCENDING && sctx->n_order > 0) {
            early = sctx->order[0];
            if (int rc = enqueue_load(sctx, early, 0)) return rc;
        }
    }

    hipEvent_t* tev = nullptr;     // this call's events, if it is timed and the timer has room
    if (timer != nullptr && timer->n < timer->cap) tev = timer->ev + kStageEvents * timer->n++;
    const bool up_only = timer != nullptr && timer->mode == MOE_TIME_UP_KERNEL;
    const bool all_stages = tev != nullptr && !up_only;
    if (all_stages) MOE_HIP_CHECK(hipEventRecord(tev[0], s));
    if (int rc = launch_route(c, x, W_g, gate_bias, idx, w, base + L.route, s)) return rc;
    if (all_stages) MOE_HIP_CHECK(hipEventRecord(tev[1], s));
    bool planned = false;          // resident mode: the work list of the one FFN launch may come from the batching kernel
    int plan_rows_down = ffn_tile_rows(gather_rows);      // (resident mode) the tile heights of the launch over all experts
    if (sctx == nullptr && c.dtype == MOE_BF16) {
        int dev = 0;
        const DeviceInfo* info = nullptr;
        if (int rc = device_info(&dev, &info)) return rc;
        plan_rows_down = ffn_down_tile_rows(c, c.E, A, ffn_tile_rows(gather_rows), info->compute_units);
    }
    if (int rc = launch_permute(c, x, idx, counts, offsets, perm, inv, gather_rows ? nullptr : base + L.Xp,
                                reinterpret_cast<int32_t*>(base + L.chunk_hist), s,
                                sctx == nullptr ? reinterpret_cast<int32_t*>(base + L.ffn_plan) : nullptr,
                                static_cast<int>(ffn_plan_tiles(c)), sctx == nullptr ? &planned : nullptr,
                                ffn_tile_rows(gather_rows), plan_rows_down))
        return rc;
    if (all_stages) MOE_HIP_CHECK(hipEventRecord(tev[2], s));

    if (sctx == nullptr) {
        if (int rc = launch_expert_ffn(c, ffn_in, offsets, 0, c.E, W_packed, eb, A, base + L.H, ffn_out,
                                       reinterpret_cast<int32_t*>(base + L.ffn_plan), s, tev ? tev[3] : nullptr,
                                       tev && up_only ? tev[2] : nullptr, row_map, planned, gather))
            return rc;
        if (all_stages) MOE_HIP_CHECK(hipEventRecord(tev[4], s));
    } else {
        SlotGuard guard{sctx};
        // The host has to know which experts hold tokens (and how many) before it can queue loads.
        MOE_HIP_CHECK(hipMemcpyAsync(sctx->h_counts, counts, sizeof(int32_t) * c.E, hipMemcpyDeviceToHost, s));
        MOE_HIP_CHECK(hipStreamSynchronize(s));
        // execution order of the experts that hold tokens (experts without tokens are never loaded)
        int n_order = 0;
        if (sctx->policy == MOE_ORDER_GREEDY) {
            if (int rc = schedule_order(sctx->h_counts, c.E, sctx->tokens_per_load, sctx->order_K, sctx->order, &n_order,
                                        &sctx->satisfiable))
                return rc;
        } else {
            for (int e = 0; e < c.E; ++e)
                if (sctx->h_counts[e] > 0) sctx->order[n_order++] = e;
        }
        // which slot each expert runs from, and whether it must be loaded: round-robin and always, unless the
        // slots keep their experts between calls
        int32_t slot_of[256], load[256];
        const bool all_fit = sctx->keep && sctx->K >= c.E;     // every expert has its own slot: slot e holds expert e
        if (all_fit) {
            for (int pos = 0; pos < n_order; ++pos) {
                const int e = sctx->order[pos];
                slot_of[pos] = e;
                load[pos] = sctx->slot_expert[e] == e ? 0 : 1;
                sctx->slot_expert[e] = e;
                sctx->slot_tick[e] = ++sctx->tick;
            }
        } else if (sctx->keep) {
            if (int rc = plan_slots(sctx->order, n_order, sctx->K, sctx->slot_expert, sctx->slot_tick, &sctx->tick, slot_of, load))
                return rc;
        } else {
            for (int pos = 0; pos < n_order; ++pos) { slot_of[pos] = pos % sctx->K; load[pos] = 1; }
        }
        int to_load = 0;
        for (int pos = 0; pos < n_order; ++pos) to_load += load[pos];
        if (all_fit && to_load == 0 && n_order > 0) {
            // Everything this call needs is resident and the slots are laid out like a resident expert array:
            // one launch over all experts instead of one per expert.
            for (int pos = 0; pos < n_order; ++pos) MOE_HIP_CHECK(hipStreamWaitEvent(s, sctx->loaded[slot_of[pos]], 0));
            if (int rc = launch_expert_ffn(c, ffn_in, offsets, 0, c.E, sctx->dev_slots, eb, A, base + L.H, ffn_out,
                                           reinterpret_cast<int32_t*>(base + L.ffn_plan), s, nullptr, nullptr, row_map, false, gather))
                return rc;
            for (int pos = 0; pos < n_order; ++pos)
                if (int rc = record_release(sctx, slot_of[pos], s)) return rc;
            sctx->n_order = n_order;
            sctx->n_loaded = 0;
            sctx->timed = false;
            n_order = 0;                                        // nothing left for the per-expert loop
        } else {
            sctx->n_order = n_order;
        }
        const bool grouped = n_order == 0 && sctx->n_order > 0 && all_fit;
        for (int pos = 0; pos < n_order; ++pos) {
            const int e = sctx->order[pos];
            const int n_e = sctx->h_counts[e];
            const int slot = slot_of[pos];
            char* dst = sctx->dev_slots + static_cast<size_t>(slot) * eb;
            if (load[pos] && !(pos == 0 && early == e)) {       // (the first expert may have been requested before routing)
                if (int rc = enqueue_load(sctx, e, slot)) return rc;
            }
            MOE_HIP_CHECK(hipStreamWaitEvent(s, sctx->loaded[slot], 0));   // also when kept: its load may still be running
            if (int rc = launch_expert_ffn(c, ffn_in, offsets, e, 1, dst, eb, n_e, base + L.H, ffn_out,
                                           reinterpret_cast<int32_t*>(base + L.ffn_plan), s, nullptr, nullptr, row_map, false, gather))
                return rc;
            if (int rc = record_release(sctx, slot, s)) return rc;
        }
        if (!grouped) {
            if (sctx->n_loaded > 0)
                for (int q = 0; q < 2; ++q)
                    if (sctx->copy_streams[q] != nullptr) MOE_HIP_CHECK(hipEventRecord(sctx->last_copy[q], sctx->copy_streams[q]));
            sctx->timed_streams = (sctx->copy_streams[0] != nullptr ? 1 : 0) | (sctx->copy_streams[1] != nullptr ? 2 : 0);
            sctx->timed = sctx->n_loaded > 0;
        }
        guard.ok = true;
    }
    if (!direct)
        if (int rc = launch_combine(c, base + L.Yp, inv, w, y, s)) return rc;
    if (all_stages) MOE_HIP_CHECK(hipEventRecord(tev[5], s));
    return MOE_OK;
}

}  // namespace

extern "C" {

int moe_layer_forward(const moe_cfg* cfg, const void* x, const void* W_g, const float* gate_bias,
                      const void* W_packed, moe_stream_ctx* sctx, void* y, void* ws, void* stream) {
    return layer_forward(cfg, x, W_g, gate_bias, W_packed, sctx, y, ws, stream, nullptr);
}

int moe_layer_forward_timed(const moe_cfg* cfg, const void* x, const void* W_g, const float* gate_bias,
                            const void* W_packed, void* y, void* ws, void* stream, moe_timer* timer) {
    REQUIRE(timer, "timer");
    return layer_forward(cfg, x, W_g, gate_bias, W_packed, nullptr, y, ws, stream, timer);
}

int moe_timer_create(int32_t max_calls, int32_t mode, moe_timer** out) {
    REQUIRE(out, "out");
    *out = nullptr;
    if (max_calls < 1 || max_calls > 4096) return fail(MOE_ERR_INVALID_ARG, "max_calls must be in [1, 4096]");
    if (mode != MOE_TIME_STAGES && mode != MOE_TIME_UP_KERNEL) return fail(MOE_ERR_INVALID_ARG, "unknown timer mode %d", mode);
    moe_timer* t = new (std::nothrow) moe_timer();
    if (t == nullptr) return fail(MOE_ERR_HIP, "out of host memory");
    t->mode = mode;
    t->ev = new (std::nothrow) hipEvent_t[static_cast<size_t>(max_calls) * kStageEvents]();
    if (t->ev == nullptr) { delete t; return fail(MOE_ERR_HIP, "out of host memory"); }
    t->cap = max_calls;
    for (int i = 0; i < max_calls * kStageEvents; ++i) {
        const hipError_t e = hipEventCreate(&t->ev[i]);
        if (e != hipSuccess) {
            moe_timer_destroy(t);
            return fail(MOE_ERR_HIP, "hipEventCreate failed: %s", hipGetErrorString(e));
        }
    }
    *out = t;
    return MOE_OK;
}

int moe_timer_destroy(moe_timer* t) {
    if (t == nullptr) return MOE_OK;
    if (t->ev != nullptr) {
        for (int i = 0; i < t->cap * kStageEvents; ++i)
            if (t->ev[i]) (void)hipEventDestroy(t->ev[i]);
        delete[] t->ev;
    }
    delete t;
    return MOE_OK;
}

int moe_timer_reset(moe_timer* t) {
    REQUIRE(t, "timer");
    t->n = 0;
    return MOE_OK;
}

int moe_timer_read(moe_timer* t, float* ms, int32_t capacity_calls, int32_t* n_calls) {
    REQUIRE(t, "timer"); REQUIRE(n_calls, "n_calls");
    *n_calls = t->n;
    if (ms == nullptr) return MOE_OK;
    const int n = t->n < capacity_calls ? t->n : capacity_calls;
    for (int c = 0; c < n; ++c) {
        hipEvent_t* ev = t->ev + kStageEvents * c;
        if (t->mode == MOE_TIME_UP_KERNEL) {
            MOE_HIP_CHECK(hipEventSynchronize(ev[3]));
            MOE_HIP_CHECK(hipEventElapsedTime(&ms[c], ev[2], ev[3]));
        } else {
            MOE_HIP_CHECK(hipEventSynchronize(ev[kStageEvents - 1]));
            for (int st = 0; st + 1 < kStageEvents; ++st)
                MOE_HIP_CHECK(hipEventElapsedTime(&ms[c * (kStageEvents - 1) + st], ev[st], ev[st + 1]));
        }
    }
    return MOE_OK;
}

int moe_stream_ctx_create(const moe_cfg* cfg, const void* host_experts, size_t expert_bytes, void* dev_slots,
                          int32_t K, moe_stream_ctx** out) {
    if (int rc = check_cfg(cfg)) return rc;
    REQUIRE(out, "out");
    *out = nullptr;
    REQUIRE(host_experts, "host_experts"); REQUIRE(dev_slots, "dev_slots");
    if (K < 1 || K > kMaxSlots) return fail(MOE_ERR_INVALID_ARG, "K must be in [1, %d] (got %d)", kMaxSlots, K);
    size_t eb = 0;
    moe_expert_bytes(cfg, &eb);
    if (expert_bytes != eb)
        return fail(MOE_ERR_INVALID_ARG, "expert_bytes is %zu but a packed expert of this cfg has %zu", expert_bytes, eb);
    if ((reinterpret_cast<uintptr_t>(dev_slots) & 255) != 0) return fail(MOE_ERR_INVALID_ARG, "dev_slots must be 256-byte aligned");
    moe_stream_ctx* ctx = new (std::nothrow) moe_stream_ctx();
    if (ctx == nullptr) return fail(MOE_ERR_HIP, "out of host memory");
    memset(ctx, 0, sizeof(*ctx));
    ctx->cfg = *cfg;
    ctx->host_experts = static_cast<const char*>(host_experts);
    ctx->expert_bytes = eb;
    ctx->dev_slots = static_cast<char*>(dev_slots);
    ctx->K = K;
    for (int i = 0; i < kMaxSlots; ++i) ctx->slot_expert[i] = -1;
    hipError_t e = hipGetDevice(&ctx->device);
    for (int i = 0; i < kMaxSlots; ++i) ctx->slot_writer[i] = -1;
    ctx->owns_copy_streams = true;
    for (int i = 0; i < K && e == hipSuccess; ++i) {
        e = hipEventCreateWithFlags(&ctx->loaded[i], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->released[i], hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipEventCreate(&ctx->first_copy);
    for (int q = 0; q < 2 && e == hipSuccess; ++q) e = hipEventCreate(&ctx->last_copy[q]);
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&ctx->h_counts), 256 * sizeof(int32_t), hipHostMallocDefault);
    if (e != hipSuccess) {
        const int rc = fail(MOE_ERR_HIP, "creating the stream context failed: %s", hipGetErrorString(e));
        moe_stream_ctx_destroy(ctx);
        return rc;
    }
    *out = ctx;
    return MOE_OK;
}

int moe_schedule_order(const int32_t* counts, int32_t E, double tokens_per_load, int32_t K, int32_t* order,
                       int32_t* n_order, int32_t* satisfiable) {
    REQUIRE(counts, "counts"); REQUIRE(order, "order"); REQUIRE(n_order, "n_order");
    if (E < 1 || E > 256) return fail(MOE_ERR_INVALID_ARG, "E must be in [1, 256] (got %d)", E);
    if (K < 0) return fail(MOE_ERR_INVALID_ARG, "K must not be negative (got %d)", K);
    if (!(tokens_per_load > 0.0)) return fail(MOE_ERR_INVALID_ARG, "tokens_per_load must be positive");
    for (int e = 0; e < E; ++e)
        if (counts[e] < 0) return fail(MOE_ERR_INVALID_ARG, "counts[%d] is negative", e);
    int n = 0, ok = 0;
    if (int rc = schedule_order(counts, E, tokens_per_load, K, order, &n, &ok)) return rc;
    *n_order = n;
    if (satisfiable != nullptr) *satisfiable = ok;
    return MOE_OK;
}

int moe_stream_ctx_set_order(moe_stream_ctx* ctx, int32_t policy, double tokens_per_load, int32_t K) {
    REQUIRE(ctx, "ctx");
    if (policy != MOE_ORDER_ASCENDING && policy != MOE_ORDER_GREEDY)
        return fail(MOE_ERR_INVALID_ARG, "unknown order policy %d", policy);
    if (policy == MOE_ORDER_GREEDY) {
        if (!(tokens_per_load > 0.0)) return fail(MOE_ERR_INVALID_ARG, "tokens_per_load must be positive");
        if (K < 0) return fail(MOE_ERR_INVALID_ARG, "K must not be negative (got %d)", K);
    }
    ctx->policy = policy;
    ctx->tokens_per_load = tokens_per_load;
    ctx->order_K = K;
    ctx->satisfiable = 0;
    return MOE_OK;
}

int moe_plan_slots(const int32_t* order, int32_t n, int32_t K, int32_t* slot_expert, int64_t* slot_tick, int64_t* tick,
                   int32_t* slot_of, int32_t* load) {
    REQUIRE(order, "order"); REQUIRE(slot_expert, "slot_expert"); REQUIRE(slot_tick, "slot_tick"); REQUIRE(tick, "tick");
    REQUIRE(slot_of, "slot_of"); REQUIRE(load, "load");
    if (n < 0 || n > 256) return fail(MOE_ERR_INVALID_ARG, "n must be in [0, 256] (got %d)", n);
    if (K < 1 || K > kMaxSlots) return fail(MOE_ERR_INVALID_ARG, "K must be in [1, %d] (got %d)", kMaxSlots, K);
    return plan_slots(order, n, K, slot_expert, slot_tick, tick, slot_of, load);
}

int moe_stream_ctx_keep_experts(moe_stream_ctx* ctx, int32_t on) {
    REQUIRE(ctx, "sctx");
    ctx->keep = on != 0;
    if (!ctx->keep)
        for (int i = 0; i < kMaxSlots; ++i) ctx->slot_expert[i] = -1;     // nothing is trusted once keeping is off
    return MOE_OK;
}

int moe_stream_ctx_prefetch(moe_stream_ctx* ctx, int32_t expert) {
    REQUIRE(ctx, "sctx");
    if (!ctx->keep) return fail(MOE_ERR_INVALID_ARG, "prefetching needs moe_stream_ctx_keep_experts(sctx, 1)");
    if (expert < 0 || expert >= ctx->cfg.E) return fail(MOE_ERR_INVALID_ARG, "expert %d is out of range", expert);
    int32_t slot = 0, load = 0;
    if (ctx->K >= ctx->cfg.E) {                 // every expert has its own slot
        slot = expert;
        load = ctx->slot_expert[expert] == expert ? 0 : 1;
        ctx->slot_expert[expert] = expert;
        ctx->slot_tick[expert] = ++ctx->tick;
    } else if (int rc = plan_slots(&expert, 1, ctx->K, ctx->slot_expert, ctx->slot_tick, &ctx->tick, &slot, &load)) {
        return rc;
    }
    if (!load) return MOE_OK;
    const int before = ctx->n_loaded;             // a load requested ahead is not one of a call's own loads
    const int rc = enqueue_load(ctx, expert, slot);
    ctx->n_loaded = before;
    if (rc != MOE_OK) ctx->slot_expert[slot] = -1;   // not taken for resident unless its copy is on its way
    return rc;
}

int moe_stream_ctx_share_loader(moe_stream_ctx* ctx, moe_stream_ctx* owner) {
    REQUIRE(ctx, "sctx"); REQUIRE(owner, "owner");
    if (ctx == owner) return MOE_OK;
    if (!owner->owns_copy_streams) return fail(MOE_ERR_INVALID_ARG, "the owner must be a context that loads on its own streams");
    if (ctx->device != owner->device) return fail(MOE_ERR_INVALID_ARG, "both contexts must live on the same device");
    if (ctx->loader == owner) return MOE_OK;
    for (int q = 0; q < 2; ++q) {
        if (ctx->copy_streams[q] != nullptr) {
            MOE_HIP_CHECK(hipStreamSynchronize(ctx->copy_streams[q]));      // nothing of this context is left on its old streams
            if (ctx->owns_copy_streams) MOE_HIP_CHECK(hipStreamDestroy(ctx->copy_streams[q]));
        }
        ctx->copy_streams[q] = nullptr;                                     // taken from the owner at the next load
        ctx->copy_waited_seq[q] = 0;                                        // nothing has been waited for on the new streams
    }
    ctx->owns_copy_streams = false;
    ctx->loader = owner;
    return MOE_OK;
}

int moe_stream_slots_that_fit(const moe_cfg* cfg, size_t reserve_bytes, int32_t* K) {
    if (int rc = check_cfg(cfg)) return rc;
    REQUIRE(K, "K");
    size_t free_b = 0, total_b = 0, eb = 0;
    MOE_HIP_CHECK(hipMemGetInfo(&free_b, &total_b));
    moe_expert_bytes(cfg, &eb);
    const size_t usable = free_b > reserve_bytes ? free_b - reserve_bytes : 0;
    size_t k = usable / align256(eb);
    if (k > static_cast<size_t>(kMaxSlots)) k = kMaxSlots;
    if (k > static_cast<size_t>(cfg->E)) k = cfg->E;          // more slots than experts are never used
    *K = static_cast<int32_t>(k);
    return MOE_OK;
}

int moe_stream_ctx_last_order(const moe_stream_ctx* ctx, int32_t* order, int32_t* n_order, int32_t* satisfiable) {
    REQUIRE(ctx, "ctx"); REQUIRE(order, "order"); REQUIRE(n_order, "n_order");
    for (int i = 0; i < ctx->n_order; ++i) order[i] = ctx->order[i];
    *n_order = ctx->n_order;
    if (satisfiable != nullptr) *satisfiable = ctx->policy == MOE_ORDER_GREEDY ? ctx->satisfiable : 0;
    return MOE_OK;
}

int moe_stream_ctx_destroy(moe_stream_ctx* ctx) {
    if (ctx == nullptr) return MOE_OK;
    for (int q = 0; q < 2; ++q) {
        if (ctx->copy_streams[q] == nullptr) continue;
        (void)hipStreamSynchronize(ctx->copy_streams[q]);
        if (ctx->owns_copy_streams) (void)hipStreamDestroy(ctx->copy_streams[q]);
    }
    for (int i = 0; i < kMaxSlots; ++i) {
        if (ctx->loaded[i]) (void)hipEventDestroy(ctx->loaded[i]);
        if (ctx->released[i]) (void)hipEventDestroy(ctx->released[i]);
    }
    if (ctx->first_copy) (void)hipEventDestroy(ctx->first_copy);
    for (int q = 0; q < 2; ++q)
        if (ctx->last_copy[q]) (void)hipEventDestroy(ctx->last_copy[q]);
    if (ctx->h_counts) (void)hipHostFree(ctx->h_counts);
    delete ctx;
    return MOE_OK;
}

int moe_stream_ctx_stats(moe_stream_ctx* ctx, int32_t* n_loaded, size_t* bytes, float* copy_ms) {
    REQUIRE(ctx, "sctx");
    float ms = 0.f;
    if (ctx->timed) {
        for (int q = 0; q < 2; ++q) {             // the later end of the two copy streams
            if (!((ctx->timed_streams >> q) & 1)) continue;
            float to_end = 0.f;
            MOE_HIP_CHECK(hipEventSynchronize(ctx->last_copy[q]));
            MOE_HIP_CHECK(hipEventElapsedTime(&to_end, ctx->first_copy, ctx->last_copy[q]));
            ms = to_end > ms ? to_end : ms;
        }
    }
    if (n_loaded) *n_loaded = ctx->n_loaded;
    if (bytes) *bytes = static_cast<size_t>(ctx->n_loaded) * ctx->expert_bytes;
    if (copy_ms) *copy_ms = ms;
    return MOE_OK;
}

}  // extern "C"
