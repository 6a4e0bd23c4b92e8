/*
 * moe355 -- the Mixture-of-Experts feed-forward layer of CPM-2-MoE on one AMD MI355X (gfx950).
 *
 * What the layer is (CPM-2, arxiv 2106.10715):
 *   - Section 2.1: the feed-forward layer of each Transformer block is expanded to several
 *     experts; every token is sent to an expert selected from its hidden state by a gate.
 *   - Section 2.3 (MoE stage): the gate is a frozen random projection of the hidden state.
 *   - Table 1: d_model 4096, d_ff 10240; the printed totals (11 B / 198 B parameters) fix a
 *     three-matrix gated expert:  FFN_e(x) = (GELU(x W_gate[e]) * (x W_in[e])) W_out[e].
 *   - Section 6 (InfMoE): tokens are routed and batched by expert before computation; expert
 *     parameters may live in CPU memory and be loaded while other experts compute, on separate
 *     streams, with at most K experts resident on the device.
 *
 * Conventions for every entry point
 *   - C ABI, plain pointers and sizes.  "device" = pointer into this GPU's memory, "host" =
 *     ordinary host pointer, "pinned" = host memory allocated with hipHostMalloc.
 *   - All matrices are row-major and contiguous.  dtype selects the storage type of x, W_g, the
 *     expert weights, Xp, Yp and y (MOE_F32 or MOE_BF16); accumulation is always fp32.
 *     idx/counts/offsets/perm/inv are int32; gate weights w and the gate bias are fp32.
 *   - The caller owns every buffer.  The library never allocates or frees device memory; scratch
 *     is the caller's workspace `ws` of at least moe_workspace_bytes() bytes, 256-byte aligned.
 *     (Only moe_stream_ctx_create allocates: two copy streams, a few events and a small pinned
 *     host buffer, all released by moe_stream_ctx_destroy.)
 *   - Calls are asynchronous: work is enqueued on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and the call returns.  The one exception is moe_layer_forward in
 *     streamed mode, which waits once for the per-expert token counts (see there).
 *   - Return value: MOE_OK or a negative MOE_ERR_* code; moe_last_error() then returns a message
 *     (thread-local, valid until the next failing call on the same thread).  Nothing is printed,
 *     no exception crosses the boundary.  Arguments are validated before anything is launched.
 *   - Limits: d and f multiples of 64; 1 <= k <= min(E, 8); 1 <= E <= 256; T >= 0 (T = 0 is a
 *     legal no-op); T*k*max(d,f) < 2^31.  Inputs must be finite.
 */
#ifndef MOE355_H
#define MOE355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { MOE_OK = 0, MOE_ERR_INVALID_ARG = -1, MOE_ERR_UNSUPPORTED = -2, MOE_ERR_WORKSPACE = -3, MOE_ERR_HIP = -4 };
enum { MOE_F32 = 0, MOE_BF16 = 1 };
enum { MOE_GATE_TOPK = 0, MOE_GATE_HASH = 1 };

typedef struct moe_cfg {
    int32_t T;       /* tokens */
    int32_t d;       /* d_model */
    int32_t f;       /* d_ff */
    int32_t E;       /* experts */
    int32_t k;       /* experts per token; the paper's layer uses 1 */
    int32_t dtype;   /* MOE_F32 | MOE_BF16 */
    int32_t renorm;  /* 1: combine weights = softmax over the k selected logits (k = 1 -> exactly 1.0)
                        0: combine weights = full-softmax probability of each selected expert */
    int32_t act;     /* 0: exact GELU z*Phi(z);  1: tanh approximation of GELU */
    int32_t gate;    /* MOE_GATE_TOPK: the k largest of the E projections x.W_g[:, e] (+ bias);
                        MOE_GATE_HASH: the gate of Section 2.3 read literally as a locality sensitive hash:
                        W_g is [d, log2 E], bit j of the expert id is set when x.W_g[:, j] > 0 (an exactly
                        zero projection gives 0), weight 1; needs E a power of two >= 2, k = 1, no bias */
    int32_t gate_packed; /* 0: W_g arguments are the matrix itself, [d, E] (hashing gate: [d, log2 E]), row-major;
                            every call that routes re-packs it into the workspace first.
                            1: W_g arguments point at the block moe_pack_gate wrote (the gate is frozen, Section 2.3,
                            so it is packed once, like the experts) */
} moe_cfg;

typedef struct moe_stream_ctx moe_stream_ctx;   /* opaque: state of the host-streamed expert mode */

/* Message of the last failing call on this thread ("" if none). */
const char* moe_last_error(void);

/* Bytes of workspace that any entry point needs for this cfg (moe_layer_forward is the largest user). */
int moe_workspace_bytes(const moe_cfg* cfg, size_t* bytes);

/* Bytes of one expert in packed form (3*d*f elements of dtype). */
int moe_expert_bytes(const moe_cfg* cfg, size_t* bytes);

/*
 * Rewrite one expert's three matrices (Table 1 shape; weights are frozen at inference, Section 2.3)
 * into the packed block the FFN kernels read: all experts have the same size (Section 6.2), so a
 * packed expert is one contiguous block of moe_expert_bytes() and "loading an expert" is one copy.
 *   W_in_e, W_gate_e [d, f], W_out_e [f, d]: device, row-major, dtype.
 *   packed_e: device, moe_expert_bytes() bytes, 256-byte aligned, must not overlap the inputs.
 * Packed layout, bf16: up block, then down block.  Up block: for each 32-column group n of d_ff and
 * each 16-row step s of d_model, a 1 KiB W_gate fragment then a 1 KiB W_in fragment; down block: for
 * each 32-column group of d_model and each 16-row step of d_ff one 1 KiB W_out fragment.  A fragment
 * holds W[16 s + 8 (l / 32) + j, 32 n + l % 32] at element 8 l + j (l = 0..63, j = 0..7), i.e. the
 * operand order of the 32x32x16 bf16 matrix instruction.  fp32: W_gate, W_in, W_out concatenated,
 * row-major, unchanged.
 */
int moe_pack_weights(const moe_cfg* cfg, const void* W_in_e, const void* W_gate_e, const void* W_out_e,
                     void* packed_e, void* stream);

/*
 * The gate in the form the gate kernel reads (Section 2.3: the gate is a random projection that is not
 * trained any further, so this is done once per model, not once per call).
 *   W_g: device, dtype, [d, E] row-major (hashing gate: [d, log2 E]), 16-byte aligned.
 *   gate_packed: device, moe_gate_bytes() bytes, 256-byte aligned, must not overlap W_g; written on `stream`.
 * bf16: the matrix in 1 KiB fragments in the operand order of the 32x32x16 bf16 matrix instruction, columns
 * padded with zeros to a multiple of 32, followed by the sum of squares of every 64-row group of every column
 * (fp32; the gate kernel bounds its rounding error with them).  fp32: the matrix unchanged.
 * cfg->gate_packed is ignored here; set it to 1 in the cfg of the calls that are given the block as W_g.
 */
int moe_gate_bytes(const moe_cfg* cfg, size_t* bytes);
int moe_pack_gate(const moe_cfg* cfg, const void* W_g, void* gate_packed, void* stream);

/*
 * Gate (Sections 2.1, 2.3): logits L = x W_g (+ gate_bias); per token the k largest logits, slot j
 * ordered by descending logit, every tie resolved to the lower expert index; combine weights per
 * cfg->renorm.  The selection equals the one exact arithmetic on the stored inputs would make: tokens
 * whose fp32 logits are closer than the fp32 error bound are re-evaluated inside the kernel from exact
 * products, in fp64 and, if that still leaves candidates closer than its rounding error, in twice that
 * precision (value + error term), which represents the sums exactly for inputs of comparable magnitude:
 * columns whose exact projections are equal tie, and the tie goes to the lower expert index.
 *   x [T, d]: device, dtype.  W_g: device, the matrix [d, E] in dtype or, with cfg->gate_packed, the block
 *   written by moe_pack_gate.   gate_bias [E]: device fp32, or NULL.
 *   idx [T, k] int32, w [T, k] fp32: device, written.
 */
int moe_route(const moe_cfg* cfg, const void* x, const void* W_g, const float* gate_bias,
              int32_t* idx, float* w, void* ws, void* stream);

/*
 * Batch assignments by expert (Section 6.2).  Assignment a = t*k + j goes to expert idx[a].
 *   counts[e] = number of assignments of e; offsets = exclusive prefix sum (offsets[E] = T*k);
 *   rows are ordered by expert, then by ascending a (stable, deterministic);
 *   perm[row] = a, inv[a] = row, Xp[row, :] = x[perm[row] / k, :].
 *   x [T, d] device dtype; idx [T, k] device (values must lie in [0, E): out-of-range values are
 *   clamped into range rather than trusted); counts [E], offsets [E+1], perm [T*k], inv [T*k] int32
 *   and Xp [T*k, d] dtype: device, written.  Xp may be NULL (index outputs only).
 */
int moe_permute(const moe_cfg* cfg, const void* x, const int32_t* idx,
                int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv, void* Xp,
                void* ws, void* stream);

/*
 * moe_permute for callers that can neither allocate device memory nor hand over a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation): same arguments without `ws`, same
 * results bit for bit.  The scratch of the batching kernels (per-chunk expert histograms) lies in a fixed
 * 256 KiB array inside the library, one copy per device, looked up on the first call on a device; the call
 * allocates nothing.  Limit: T*k <= 262144 assignments (E <= 256 as everywhere); beyond it MOE_ERR_WORKSPACE
 * and nothing is launched.  All calls on one device share the array: calls that overlap in time on one device
 * (different streams or threads) race and must be ordered by the caller; nothing has to be cleared between
 * calls (every entry that is read is written first by the same call).
 */
int moe_permute_static(const moe_cfg* cfg, const void* x, const int32_t* idx,
                       int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv, void* Xp, void* stream);

/*
 * Expert FFNs on the batched rows: for every expert e with offsets[e] < offsets[e+1] and every row r
 * in that range, Yp[r] = (act(Xp[r] W_gate[e]) * (Xp[r] W_in[e])) W_out[e].  Experts without rows
 * are not read.  The d_ff-wide intermediate is kept in ws in dtype.
 *   Xp [T*k, d] device dtype; offsets [E+1] device int32 (read on the device, no host sync);
 *   W_packed: device, E packed experts back to back (moe_pack_weights); Yp [T*k, d] device, written.
 */
int moe_expert_ffn(const moe_cfg* cfg, const void* Xp, const int32_t* offsets, const void* W_packed,
                   void* Yp, void* ws, void* stream);

/*
 * Weighted un-permute (Section 2.1: the output of the selected expert takes the place of the feed-forward
 * output of the token; with k experts per token, their weighted sum): y[t, :] = sum_{j<k} w[t, j] *
 * Yp[inv[t*k + j], :], summed in slot order in fp32, rounded once to dtype.
 *   Yp [T*k, d], inv [T*k], w [T, k]: device;  y [T, d]: device, written.
 */
int moe_combine(const moe_cfg* cfg, const void* Yp, const int32_t* inv, const float* w, void* y, void* stream);

/*
 * The whole layer, x -> y, as route -> permute -> expert FFNs -> combine on `stream`; every
 * intermediate lives in ws.  When every token has one expert with weight exactly 1 (bf16, k = 1 and
 * renorm = 1 or the hashing gate: the paper's layer) the combine step is only a row permutation, and
 * the down-projection writes its rows to their tokens' rows of y itself instead of a separate pass; the
 * bytes of y are the same as from the four steps called one by one.
 *   Resident mode (sctx == NULL): W_packed holds all E packed experts on the device; nothing waits
 *   on the host.
 *   Streamed mode (sctx != NULL, W_packed ignored): the experts live in pinned host memory (Section 6).
 *   After route + permute the call copies counts[E] to the host and waits for it (the host must know
 *   which experts have tokens; Section 6.2 sizes an expert's compute by its token count), then runs the
 *   non-empty experts in the order of the context (ascending id unless moe_stream_ctx_set_order chose the
 *   greedy order of Section 6.2): each expert's packed block is copied into one of the K device slots on one of the
 *   context's two copy streams (taking turns) while earlier experts compute on `stream`; events order copy-before-compute and
 *   compute-before-slot-reuse.  Experts without tokens are not loaded.  Every call loads every non-empty
 *   expert, unless moe_stream_ctx_keep_experts lets the slots keep theirs between calls (then only experts
 *   no slot holds are loaded).  From the second call on a context in ascending order, the load of the expert the
 *   previous call ran first is requested before the gate runs (it is very likely the first again; a wrong guess
 *   costs one wasted copy).  The call returns with the remaining work enqueued on `stream`.  If the
 *   call fails half-way, the context forgets what its slots hold (nothing is taken for resident that may
 *   not have been copied).
 *   Results are bitwise identical in both modes.
 *   Resident calls consist of kernel launches only and can be recorded into a HIP graph; with more than 32
 *   experts, run one call outside the capture first (the gate kernel raises its LDS limit once per device).
 */
int moe_layer_forward(const moe_cfg* cfg, const void* x, const void* W_g, const float* gate_bias,
                      const void* W_packed, moe_stream_ctx* sctx, void* y, void* ws, void* stream);

/*
 * Streamed-mode state (Section 6.2: K experts resident at once, separate streams for loading and
 * computing).  host_experts: pinned, E packed experts back to back, expert_bytes each (must equal
 * moe_expert_bytes).  dev_slots: device, K * expert_bytes, 256-byte aligned.  1 <= K <= 64.
 * Both buffers stay owned by the caller and must outlive the context.  Must be called with the
 * device that holds dev_slots current.
 */
int moe_stream_ctx_create(const moe_cfg* cfg, const void* host_experts, size_t expert_bytes,
                          void* dev_slots, int32_t K, moe_stream_ctx** out);
int moe_stream_ctx_destroy(moe_stream_ctx* sctx);

/*
 * Execution order of offloaded experts (Section 6.2, the part on scheduling offloaded experts).
 *
 * With alpha_i the computation time of expert i (proportional to its token count), beta the loading
 * time of one expert (the same for all) and K the number of experts loads may run ahead, the paper
 * asks for an order o_1..o_T with, for every t,
 *     sum_{i<t} alpha_{o_i} >= (t - 1) beta     and     sum_{i<t} alpha_{o_i} <= (t + K - 1) beta,
 * found greedily; it does not print the rule.  moe_schedule_order takes, at every position, the
 * remaining non-empty expert with the most tokens that keeps the second constraint, else the one
 * with the fewest (ties: lower expert id).  Times are given in tokens: tokens_per_load =
 * beta / (computation time of one token) > 0.
 *
 *   counts  host [E], tokens per expert (>= 0); experts with 0 tokens are left out of the order
 *   order   host [E] out: expert ids in execution order; *n_order = how many (the non-empty ones)
 *   satisfiable  host out, may be NULL: 1 if the order meets both constraints for all t, else 0
 *                (an order is returned either way)
 * Pure host function; E in [1, 256], K >= 0.  Errors: MOE_ERR_INVALID_ARG.
 */
#define MOE_ORDER_ASCENDING 0   /* experts in ascending id (the naive order of Figure 4a) */
#define MOE_ORDER_GREEDY 1      /* moe_schedule_order on the counts of each call (Figure 4b) */
int moe_schedule_order(const int32_t* counts, int32_t E, double tokens_per_load, int32_t K, int32_t* order,
                       int32_t* n_order, int32_t* satisfiable);

/*
 * Which order streamed moe_layer_forward calls on this context load and run their experts in
 * (default MOE_ORDER_ASCENDING).  tokens_per_load and K are those of moe_schedule_order and are
 * ignored for MOE_ORDER_ASCENDING; K here is the K of the constraint, independent of the number of
 * device slots the context owns (slots are always reused safely through events, in any order).
 * The result of the layer does not depend on the order (bitwise).
 */
int moe_stream_ctx_set_order(moe_stream_ctx* sctx, int32_t policy, double tokens_per_load, int32_t K);

/*
 * The order the last streamed moe_layer_forward on this context used: order host [E] out,
 * *n_order experts; *satisfiable (may be NULL) as in moe_schedule_order, 0 for MOE_ORDER_ASCENDING.
 */
int moe_stream_ctx_last_order(const moe_stream_ctx* sctx, int32_t* order, int32_t* n_order, int32_t* satisfiable);

/*
 * Experts that stay resident (Section 6.2: the device holds K experts at a time, K set by the caller or
 * derived from the memory there is).
 *
 * moe_stream_slots_that_fit: the K a context can be given on the current device: how many packed experts
 * of this cfg fit into the free device memory minus reserve_bytes, at most 64 and at most E.
 *
 * moe_stream_ctx_keep_experts(sctx, 1): from now on the slots keep their experts between calls; a
 * streamed moe_layer_forward loads only the experts of its order that no slot holds.  Since the whole
 * order of a call is known before its first load, the expert that gives way is the one whose next use
 * in this call lies furthest ahead (an empty slot first; never used again before used later; among
 * equals the slot unused for longest, then the lowest slot), which minimises the loads of the call.
 * With K >= E every expert has its own slot, is loaded once, and a call that needs no load runs all its
 * experts in one grouped launch, i.e. at the resident speed.  The host
 * copy of the experts must not change while experts are kept; (sctx, 0) forgets what the slots hold
 * and returns to loading every expert in every call (the default, which is what the measured
 * streamed configurations do).  moe_stream_ctx_stats reports the experts actually copied.
 *
 * moe_stream_ctx_prefetch(sctx, e): start loading expert e into a slot now, on the copy stream, unless a
 * slot holds it (needs keeping switched on).  Meant for a stack of layers: while layer l computes, the
 * caller prefetches the expert it expects layer l+1 to run first, so that the one load nothing hides
 * (Section 6.2: only the first expert waits for its parameters) is paid once per model rather than once
 * per layer.  Returns at once.
 *
 * moe_plan_slots is the replacement rule itself as a pure host function (all arrays host memory):
 *   order [n] experts in execution order;  slot_expert [K] in/out, -1 = empty;  slot_tick [K] in/out, when
 *   each slot was last used;  *tick in/out use counter;  slot_of [n], load [n] (1 = must be loaded) out.
 *
 * moe_stream_ctx_share_loader(sctx, owner): from now on sctx enqueues its loads on owner's copy streams instead of its
 * own, so that the loads of both contexts run one after the other in the order they were requested (one loader for
 * the whole model, as in Section 6.2's timeline) instead of side by side.  With the layers of a model sharing one
 * loader, a prefetch for layer l+1 issued right after the call of layer l has returned is queued behind layer l's last
 * load and runs while layer l finishes computing and layer l+1 routes.  Waits until sctx's own loads have finished.
 * owner must be a context with copy streams of its own, on the same device, and must be destroyed after sctx.
 */
int moe_stream_slots_that_fit(const moe_cfg* cfg, size_t reserve_bytes, int32_t* K);
int moe_stream_ctx_share_loader(moe_stream_ctx* sctx, moe_stream_ctx* owner);
int moe_stream_ctx_keep_experts(moe_stream_ctx* sctx, int32_t on);
int moe_stream_ctx_prefetch(moe_stream_ctx* sctx, int32_t expert);
int moe_plan_slots(const int32_t* order, int32_t n, int32_t K, int32_t* slot_expert, int64_t* slot_tick, int64_t* tick,
                   int32_t* slot_of, int32_t* load);

/*
 * Figures of the last streamed moe_layer_forward on this context; waits for that call's work to
 * finish.  n_loaded = experts copied; bytes = n_loaded * expert_bytes; copy_ms = first copy start to
 * last copy end on the copy streams.  Any pointer may be NULL.
 */
int moe_stream_ctx_stats(moe_stream_ctx* sctx, int32_t* n_loaded, size_t* bytes, float* copy_ms);

/*
 * Measurement aid: a resident moe_layer_forward that also records HIP events on `stream` around its stages
 * (Sections 2.1 and 6.2 name them: route, batch by expert, expert FFNs, combine) into a timer object the
 * caller owns.  The hot entry point itself keeps no timing state.
 *
 * moe_timer_create(max_calls, mode): room for max_calls (1..4096) timed calls.
 *   MOE_TIME_STAGES     events around all five stages (route, permute, expert up-projection kernel, expert
 *                       down-projection kernel, combine); each event between two kernels costs the call a
 *                       few microseconds of idle time
 *   MOE_TIME_UP_KERNEL  two events only, right before and right after the expert up-projection kernel
 * moe_layer_forward_timed: the same work, on the same kernels, as resident moe_layer_forward(cfg, ..., NULL, y, ws,
 *   stream), plus the events; once the timer is full it records nothing more.  A timer must not be used from two
 *   threads at once.
 * moe_timer_read waits for the recorded calls; ms is host memory, row-major [call][5] (MOE_TIME_STAGES) or
 *   [call] (MOE_TIME_UP_KERNEL), at most capacity_calls rows are written; *n_calls = calls recorded.
 * moe_timer_reset forgets the recorded calls (the events are kept); moe_timer_destroy releases everything.
 */
typedef struct moe_timer moe_timer;
enum { MOE_TIME_STAGES = 0, MOE_TIME_UP_KERNEL = 1 };
int moe_timer_create(int32_t max_calls, int32_t mode, moe_timer** out);
int moe_timer_destroy(moe_timer* timer);
int moe_timer_reset(moe_timer* timer);
int moe_timer_read(moe_timer* timer, float* ms, int32_t capacity_calls, int32_t* n_calls);
int moe_layer_forward_timed(const moe_cfg* cfg, const void* x, const void* W_g, const float* gate_bias,
                            const void* W_packed, void* y, void* ws, void* stream, moe_timer* timer);

#ifdef __cplusplus
}
#endif
#endif /* MOE355_H */
