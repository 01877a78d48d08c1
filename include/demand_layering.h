/*
 * demand_layering.h — C ABI of the pipelined Demand Layering library for MI355X (gfx950).
 *
 * The library runs a transformer layer stack whose BF16 parameters live in
 * pinned host memory: each streamed layer is copied host -> device into one of
 * two device slots on a copy stream while the previous layer computes on the
 * compute stream, and a chosen subset of layers stays device-resident.
 *
 * Conventions
 *   - Every call returns an int32_t: DL_OK (0) or a negative DL_ERR_* code;
 *     dl_last_error(ctx) gives a NUL-terminated message owned by the context.
 *   - A failed call leaves the context unchanged (a residency set that does
 *     not fit is rejected whole).  One exception: DL_ERR_DEVICE from a call
 *     that re-places device memory (residency, slot count, workspace size,
 *     registration) can mean that a copy into memory the same call had taken
 *     from a resident layer failed after the new placement was committed; the
 *     context then refuses every further call with DL_ERR_DEVICE (dl_destroy
 *     and dl_last_error still work).  When the new copies touch only free
 *     memory they are made first and a failure changes nothing.
 *   - A context is used from one host thread.  No C++ type crosses the ABI.
 *   - "host" / "device" in a parameter comment says where the pointer lives.
 *   - BF16 data is passed as raw 16-bit patterns; matrices are row-major
 *     [out_features, in_features] (a linear map is y = x * W^T + b).
 *   - The caller owns: its source tensors (copied by the call that takes
 *     them), the arena block, the two streams.  The library owns: the pinned
 *     parameter store, its events, and whatever it carves out of the arena.
 *   - All device memory the library uses comes out of the arena: the arena
 *     size IS the device-memory cap.
 */
#ifndef DEMAND_LAYERING_H
#define DEMAND_LAYERING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dl_ctx dl_ctx;

enum {
    DL_OK = 0,
    DL_ERR_INVALID_ARG = -1,
    DL_ERR_BUDGET_EXCEEDED = -2,
    DL_ERR_HOST_ALLOC = -3,
    DL_ERR_DEVICE = -4,
    DL_ERR_BAD_STATE = -5
};

enum { DL_NORM_RMS = 0, DL_NORM_LN = 1 };
enum { DL_ACT_SWIGLU = 0, DL_ACT_GELU = 1 };
/* Sec. IV-B (sequential: copy, then compute, never overlapped) and Sec. IV-C (pipelined) */
enum { DL_MODE_PIPELINED = 0, DL_MODE_SEQUENTIAL = 1 };

/* per-layer parameter tensors */
enum {
    DL_T_NORM1_G = 0, DL_T_NORM1_B = 1,
    DL_T_WQ = 2, DL_T_WK = 3, DL_T_WV = 4, DL_T_BQ = 5, DL_T_BK = 6, DL_T_BV = 7,
    DL_T_WO = 8, DL_T_BO = 9,
    DL_T_NORM2_G = 10, DL_T_NORM2_B = 11,
    DL_T_W_GATE = 12, DL_T_W_UP = 13, DL_T_B_UP = 14, DL_T_W_DOWN = 15, DL_T_B_DOWN = 16,
    DL_T_NORMC_G = 17, DL_T_NORMC_B = 18,
    DL_T_WQ_C = 19, DL_T_WK_C = 20, DL_T_WV_C = 21, DL_T_BQ_C = 22, DL_T_BK_C = 23, DL_T_BV_C = 24,
    DL_T_WO_C = 25, DL_T_BO_C = 26,
    DL_T_COUNT = 27
};

/* always-resident non-layer parameters (Sec. IV-D: non-layer components stay resident in every configuration) */
enum { DL_R_EMBED = 0, DL_R_HEAD = 1, DL_R_FINAL_NORM_G = 2, DL_R_FINAL_NORM_B = 3, DL_R_COUNT = 4 };

/*
 * One layer stack ("module" in the paper: vision encoder, VLM backbone, expert decoder).
 * Block: h = x + Attn(Norm1 x) [+ CrossAttn(NormC h, ctx) if d_ctx > 0];  y = h + FFN(Norm2 h).
 */
typedef struct {
    int32_t n_layers;
    int32_t d_model;
    int32_t n_q_heads, n_kv_heads, d_head;   /* n_q_heads % n_kv_heads == 0; d_head % 8 == 0, <= 128 */
    int32_t d_ff;                            /* % 32 == 0 for SwiGLU, % 8 == 0 for GELU */
    int32_t norm;                            /* DL_NORM_* */
    int32_t act;                             /* DL_ACT_*: SwiGLU (gate, up, down) or GELU-tanh MLP (up, down) */
    int32_t has_bias;                        /* biases on every linear map */
    int32_t causal;
    int32_t d_ctx;                           /* > 0: cross-attention over a [n_ctx, d_ctx] source */
    int32_t max_seq;                         /* > 0: KV cache with this many positions (forward may then be called with pos0 > 0) */
    int32_t max_tokens;                      /* largest n_tokens of any forward call; sizes the activation workspace */
    int32_t max_ctx;                         /* largest n_ctx (cross-attention), 0 if none */
    int32_t vocab;                           /* > 0: embedding table and output head [vocab, d_model] */
    float rope_theta;                        /* 0 = no rotary embedding; else pair (i, i + d_head/2), angle pos * theta^(-2i/d_head) */
    float norm_eps;
} dl_module_desc;

/* ---- context ---------------------------------------------------------------------------- */

/* device >= 0: HIP device ordinal (made current on every call).  device == -1: host-only
 * context — nothing touches a GPU: parameters go to ordinary host memory, the arena is pure
 * accounting, dl_forward only records its schedule (see dl_trace_read).  Used for planning
 * and for checking the slot protocol without a GPU.  *out is owned by the library. */
int32_t dl_create(dl_ctx** out, int32_t device);
int32_t dl_destroy(dl_ctx* ctx);
/* ctx == NULL: the message of the last failed call that takes no context, on the calling thread. */
const char* dl_last_error(const dl_ctx* ctx);

/* The device-memory budget.  dev_base: device pointer to a block of `bytes` bytes the caller
 * allocated and keeps alive until dl_destroy; 256-byte aligned.  Must be set once, before any
 * module is finalized.  Sec. IV-D: residency costs VRAM; here every device byte is counted. */
int32_t dl_set_arena(dl_ctx* ctx, void* dev_base, uint64_t bytes);
/* Sub-allocate from the arena for the caller's activations (counted against the cap).
 * DL_ERR_BUDGET_EXCEEDED if it does not fit.  Arena discipline: blocks that never move (these, KV caches, resident
 * non-layer tensors, MLPs) are stacked at the top of the arena with the activation workspaces right below them;
 * slots and resident layer copies fill it from the bottom and are placed again (re-copied from the pinned store)
 * when a change does not fit between the holes.  The call synchronises both streams, because the workspaces move
 * down (their contents are scratch within one call of the library and are not kept). */
int32_t dl_arena_alloc(dl_ctx* ctx, uint64_t bytes, void** dev_ptr_out);
int32_t dl_arena_free(dl_ctx* ctx, void* dev_ptr);
int32_t dl_arena_stats(const dl_ctx* ctx, uint64_t* used, uint64_t* peak, uint64_t* capacity);
/* *bytes = what slots and resident layer copies may use together: the arena below its top stack.  Sec. IV-D's
 * budget, as the library accepts it: dl_set_residency / dl_set_slot_count take every choice whose resident copies plus
 * n_slots slots of the largest layer that still streams (dl_module_layer_bytes' packed sizes) sum to at most *bytes,
 * whatever was resident before, so a planner given this figure never proposes a set that is then refused. */
int32_t dl_residency_budget(const dl_ctx* ctx, uint64_t* bytes);

/* compute_stream / copy_stream: hipStream_t handles owned by the caller; distinct; default priority.
 * Sec. IV-C: one queue executes layers, the other prefetches parameters.  Every call of a device context that
 * enqueues work returns DL_ERR_BAD_STATE until the streams are set. */
int32_t dl_set_streams(dl_ctx* ctx, void* compute_stream, void* copy_stream);

/* ---- registering a layer stack (one-time, untimed) ------------------------------------- */

/* Allocates the module's pinned host parameter store (Sec. IV-C(iii)), one contiguous
 * kernel-ready blob per layer so that a layer is ONE host-to-device copy.  DL_ERR_INVALID_ARG for a description outside
 * the limits noted in dl_module_desc, for more than 32 query heads per KV head on a module with a KV cache, and when
 * max(max_seq, max_tokens, max_ctx) times the widest row of the module (2 * d_ff for SwiGLU) times 4 bytes reaches
 * 4 GB (the kernels address one operand with 32-bit byte offsets). */
int32_t dl_module_create(dl_ctx* ctx, const dl_module_desc* desc, int32_t* module_out);
/* host_bf16: host pointer, n_elems BF16 values, shape fixed by the descriptor (see DL_T_*).
 * The data is COPIED into the packed blob (fused / interleaved as the kernels read it). */
int32_t dl_layer_set_tensor(dl_ctx* ctx, int32_t module, int32_t layer, int32_t tensor_id,
                            const void* host_bf16, uint64_t n_elems);
/* host_bf16 -> arena (device-resident for the module's lifetime). Needs the arena. */
int32_t dl_set_resident_tensor(dl_ctx* ctx, int32_t module, int32_t which, const void* host_bf16, uint64_t n_elems);
/* All tensors of all layers must have been set.  Sizes the two shared slots (Sec. IV-C(i): 2 x M_max, M_max
 * taken over the finalized modules that stream at least one layer: a fully resident module never uses a slot)
 * and carves the module's KV cache and activation workspace out of the arena. */
int32_t dl_module_finalize(dl_ctx* ctx, int32_t module);
/* packed_bytes: bytes of one layer's blob (what one copy moves); param_bytes: 2 * parameter count. */
int32_t dl_module_layer_bytes(const dl_ctx* ctx, int32_t module, uint64_t* packed_bytes, uint64_t* param_bytes);

/* ---- residency (Sec. IV-D) ------------------------------------------------------------- */

/* layer_idx: host array of n distinct layer indices that stay device-resident; the rest stream.
 * Uploads newly resident layers, releases dropped ones.  The slot pair is re-sized to the largest layer of the
 * modules that still stream something (making the module with the largest layers fully resident shrinks it);
 * n == n_layers for every module releases it.  Synchronises both streams.  DL_ERR_BUDGET_EXCEEDED: nothing changed. */
int32_t dl_set_residency(dl_ctx* ctx, int32_t module, const int32_t* layer_idx, int32_t n);
/* idx_out: host array of capacity n_layers; *n_out = count */
int32_t dl_get_residency(const dl_ctx* ctx, int32_t module, int32_t* idx_out, int32_t* n_out);

/* mode: DL_MODE_*.  wrap_prefetch != 0: at the end of a forward pass the first streamed layer of the
 * module is prefetched for the next pass (valid while the next pass uses the same module; another
 * module's pass simply re-issues its own first copy). */
int32_t dl_set_mode(dl_ctx* ctx, int32_t mode, int32_t wrap_prefetch);

/* Number of device slots the streamed layers go through, 1 .. 4: 2 (default: the Double Flat Buffer of Sec. IV-C(i), the
 * copy of the next streamed layer overlaps the execution of the current one), 3 or 4 (n - 1 copies run ahead of the
 * executing layer: deeper prefetch, one more layer of memory each), or 1 (the copy of the next streamed layer
 * starts when the current one has executed and overlaps only the resident layers in between).  One slot gives a whole
 * layer of memory back: where a layer's copy takes far longer than its execution (single-token passes: ~60 x) the
 * overlap lost is worth less than one more resident layer.  Synchronises both streams and re-sizes the slots;
 * DL_ERR_BUDGET_EXCEEDED: nothing changed. */
int32_t dl_set_slot_count(dl_ctx* ctx, int32_t n_slots);

/* Re-sizes the activation workspace of a finalized module for passes of at most max_tokens tokens (>= 1).  The
 * workspace is sized by the longest pass (Sec. IV-D counts activations against the same memory as the parameters):
 * after a long prefill, shrinking it to the single-token passes that follow gives that memory to resident layers
 * (8B-class decoder, 3072 -> 1 tokens: 164 MB, which under a 12e9-byte cap is the difference between 26 and 27
 * resident layers).  Synchronises both streams.  Keeps the KV cache, the residency set, the resident tensors and
 * the packed weights; discards the workspace's contents (intermediate activations, the logits and token of the
 * last greedy step).  Afterwards dl_forward / dl_profile accept n_tokens <= max_tokens.
 * DL_ERR_BUDGET_EXCEEDED (growing): nothing changed. */
int32_t dl_module_set_max_tokens(dl_ctx* ctx, int32_t module, int32_t max_tokens);

/* How many streaming passes (passes that copy at least one layer) may be unfinished when the next one is
 * enqueued (1..8; 0 = no limit).  Default 1: each further pass of short streamed layers in flight slowed copies and
 * kernels on MI355X (+4 % with two, +25 % with four).  A pass counts as finished for this purpose when its last
 * layer has started (the head of the next pass is then queued while that layer runs).  Passes of resident layers only
 * are never held back. */
int32_t dl_set_run_ahead(dl_ctx* ctx, int32_t passes);

/* ---- the hot path (Sec. IV-C) ------------------------------------------------------------ */

/* One pass over all layers of `module`; enqueues only, returns before the GPU finishes, except that a pass
 * which streams at least one layer first waits until the streaming pass dl_set_run_ahead (default one) passes
 * back has reached its last layer.
 * x_dev: device fp32 [n_tokens, d_model] input;  y_dev: device fp32 [n_tokens, d_model] output
 * (may equal x_dev).  Token t sits at absolute position pos0 + t; with a KV cache the pass appends
 * its keys/values at those positions and attends over 0 .. pos0+t.  pos0 must be 0 without a cache.
 * ctx_dev: device fp32 [n_ctx, d_ctx] (cross-attention source) or NULL.
 * n_tokens == 1 takes the decode kernels (weight-streaming matrix-vector products, split-key attention over the
 * KV cache), otherwise the MFMA GEMM / tiled attention path. */
int32_t dl_forward(dl_ctx* ctx, int32_t module, const void* x_dev, void* y_dev, int32_t n_tokens,
                   int32_t pos0, const void* ctx_dev, int32_t n_ctx);
/* x_dev[d_model] (fp32) = embedding row `token`, on the compute stream. */
int32_t dl_embed_token(dl_ctx* ctx, int32_t module, int32_t token, void* x_dev);
/* out_dev fp32 [n_tokens, d_model] = FinalNorm(h_dev), on the compute stream. */
int32_t dl_final_norm(dl_ctx* ctx, int32_t module, const void* h_dev, void* out_dev, int32_t n_tokens);
/* Greedy head on one fp32 hidden vector h_dev[d_model]: logits = FinalNorm(h) * W_head^T in fp32,
 * token = lowest index of the maximum.  Synchronises the compute stream.  token_out: host.
 * logits_out_host: host fp32 [vocab] or NULL. */
int32_t dl_logits_argmax(dl_ctx* ctx, int32_t module, const void* h_dev, int32_t* token_out, float* logits_out_host);
/* As above but leaves the token on the device and feeds it back: x_dev[d_model] = E[token].  No host sync.
 * token_dev: device int32[1]. */
int32_t dl_greedy_step(dl_ctx* ctx, int32_t module, const void* h_dev, int32_t* token_dev, void* x_dev);
int32_t dl_sync(dl_ctx* ctx);

/* For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc, or callers that hold the head's tensors in device memory of their own and have no context or arena.
 * The greedy step of dl_greedy_step on plain device pointers: logits = FinalNorm(h) * W_head^T in fp32, token = lowest
 * index of the maximum, x_dev = E[token]; the same two kernels, enqueued on `stream` (a hipStream_t of `device`, which
 * is current while the call runs; the caller's current device is restored on return), no host synchronisation, no context touched.  The logits of the step live in a static device
 * array of the library (one per GPU, 131072 floats + 256 bytes, held until the process ends); the call allocates
 * nothing, creates no event, and records nothing a graph capture could not hold.
 * h_dev: device fp32 [d_model]; head_dev, embed_dev: device BF16 [vocab, d_model] (embed_dev and x_dev may both be
 * NULL: token only); norm_g_dev / norm_b_dev: device BF16 [d_model] (norm_b_dev only for DL_NORM_LN);
 * token_dev: device int32[1]; x_dev: device fp32 [d_model].  d_model % 8 == 0, <= 16384; vocab <= 131072.
 * DL_ERR_INVALID_ARG beyond these limits or with a missing pointer, DL_ERR_DEVICE if the launch fails; the message is
 * read with dl_last_error(NULL) on the same thread.  All calls on one GPU share that GPU's array: calls that overlap
 * in time on one GPU (different streams, or graphs replayed concurrently) race on it. */
int32_t dl_greedy_step_static(int32_t device, void* stream, const void* h_dev, const void* head_dev, const void* embed_dev,
                              const void* norm_g_dev, const void* norm_b_dev, int32_t norm, float norm_eps,
                              int32_t d_model, int32_t vocab, int32_t* token_dev, void* x_dev);

/* ---- always-resident dense parts between the layer stacks (Sec. II-A patch merger, output heads; Sec. IV-D:
 *      non-layer components stay resident in every configuration) ------------------------------------------ */

/* y = W2 * gelu_tanh(W1 * x + b1) + b2 when d_hidden > 0, else y = W2 * x + b2.  w1: host BF16 [d_hidden, d_in],
 * w2: host BF16 [d_out, d_hidden or d_in]; b1, b2: host BF16 or NULL.  Parameters and a [max_tokens, .] BF16
 * workspace are placed in the arena (DL_ERR_BUDGET_EXCEEDED if they do not fit).  d_in, d_hidden % 8 == 0. */
int32_t dl_mlp_create(dl_ctx* ctx, int32_t d_in, int32_t d_hidden, int32_t d_out, const void* w1, const void* b1,
                      const void* w2, const void* b2, int32_t max_tokens, int32_t* mlp_out);
/* x_dev: device fp32 [n_tokens, d_in]; y_dev: device fp32 [n_tokens, d_out]; on the compute stream. */
int32_t dl_mlp_forward(dl_ctx* ctx, int32_t mlp, const void* x_dev, void* y_dev, int32_t n_tokens);
/* y_dev[t, :] = mean of x_dev[t*group .. t*group+group-1, :]  (fp32, d columns, t < n_out) */
int32_t dl_mean_pool(dl_ctx* ctx, const void* x_dev, void* y_dev, int32_t n_out, int32_t group, int32_t d);
/* y_dev[i] += alpha * x_dev[i], i < n  (one Euler step of the flow-matching action head, Sec. II-A) */
int32_t dl_axpy(dl_ctx* ctx, void* y_dev, float alpha, const void* x_dev, uint64_t n);
/* y_dev[t, i] = x_dev[t, i] + e_i(t_value): sinusoidal embedding of the flow time added to every token;
 * e_i = sin(1000 t w_i) for i < d/2, cos(1000 t w_{i-d/2}) otherwise, w_j = 10000^(-j/(d/2)). */
int32_t dl_add_time_embedding(dl_ctx* ctx, const void* x_dev, void* y_dev, float t_value, int32_t n_tokens, int32_t d);

/* ---- the five-stage inference as one call (Sec. II-A: vision encoder, patch merger, prefill, decode, flow-matching
 *      action generator with Euler steps) ---------------------------------------------------------------------- */

typedef struct {
    int32_t m_vit, m_dec, m_act;   /* finalized modules: encoder; causal decoder with KV cache, head and embedding table;
                                      action stack with d_ctx == decoder d_model */
    int32_t mlp_proj;              /* dl_mlp_create id: merger, encoder d_model -> hidden -> decoder d_model */
    int32_t mlp_out;               /* dl_mlp_create id: trajectory head, action d_model -> out_dim (no hidden layer) */
    int32_t n_patches;             /* encoder tokens; n_patches % pool == 0 */
    int32_t pool;                  /* consecutive merged tokens averaged into one visual token (stand-in for the 2x2 merge) */
    int32_t n_text;                /* text embeddings that follow the visual tokens in the prefill */
    int32_t n_actions;             /* action tokens (64 waypoints) */
    int32_t n_decode;              /* greedy decode steps after the prefill (>= 0) */
    int32_t n_euler;               /* Euler steps of the flow-matching loop (10 in the paper) */
    int32_t out_dim;               /* columns of the trajectory (3) */
} dl_vla_desc;

/* Device buffers of one inference, fp32 unless noted, owned by the caller (arena blocks count against the cap).
 * n_vis = n_patches / pool, n_prefill = n_vis + n_text. */
typedef struct {
    const void* patches;   /* in:  [n_patches, vit.d_model] */
    void* vit_out;         /* scratch [n_patches, vit.d_model] */
    void* proj_out;        /* scratch [n_patches, dec.d_model] */
    void* seq;             /* in/out [n_prefill, dec.d_model]: rows n_vis.. hold the text embeddings on entry; rows < n_vis
                              are written (the visual tokens) */
    void* hidden;          /* out: [n_prefill, dec.d_model] decoder output of the prefill */
    void* hidden_ctx;      /* out: [n_prefill, dec.d_model] FinalNorm(hidden): the action stack's cross-attention context */
    void* x1;              /* scratch [dec.d_model] */
    void* y1;              /* scratch [dec.d_model] */
    int32_t* tokens;       /* out: device int32 [n_decode] greedy ids */
    void* actions;         /* in/out [n_actions, act.d_model]: noise on entry, denoised action tokens on return */
    void* act_in;          /* scratch [n_actions, act.d_model] */
    void* velocity;        /* scratch [n_actions, act.d_model] */
    void* trajectory;      /* out: [n_actions, out_dim] */
} dl_vla_buffers;

/* Enqueues one whole inference on the context's streams and returns (dl_sync to wait):
 *   v = Encoder(patches);  p = Merger(v);  seq[t] = mean of p[t*pool .. t*pool+pool-1]  (t < n_vis);
 *   hidden = Decoder(seq) at positions 0 .. n_prefill-1;  hidden_ctx = FinalNorm(hidden);
 *   h = hidden[n_prefill-1];  for s < n_decode: tokens[s] = greedy(head(h)); h = Decoder(E[tokens[s]]) at n_prefill+s;
 *   for s < n_euler: actions += ActionStack(actions + e(s / n_euler); context hidden_ctx) / n_euler;
 *   trajectory = TrajectoryHead(actions).
 * Every step is one of the calls above (dl_forward, dl_mlp_forward, dl_mean_pool, dl_final_norm, dl_greedy_step,
 * dl_add_time_embedding, dl_axpy) issued in this order; residency, mode and slot count apply as set.  Checks shapes
 * against the modules (DL_ERR_INVALID_ARG) before anything is enqueued. */
int32_t dl_vla_infer(dl_ctx* ctx, const dl_vla_desc* desc, const dl_vla_buffers* buf);

/* ---- measurement ------------------------------------------------------------------------ */

typedef struct {
    double c_dma_ms;      /* un-overlapped host-to-device copy time of the layer: an isolated copy, the copy queue
                             idle before and after it */
    double c_dma_cont_ms; /* copy time of the layer inside an uninterrupted train of copies (the next one already
                             queued when this one ends): what a copy costs while the copy queue never runs dry */
    double c_exe_ms;      /* un-overlapped execution time of the layer, run right after its copy (the GPU was idle) */
    double c_exe_hot_ms;  /* execution time of the layer inside an uninterrupted run of all layers (no copies, no
                             idle gaps): what a layer costs when compute is continuous, e.g. between resident layers */
    double c_exe_loaded_ms; /* c_exe_hot_ms as it is while host-to-device copies run the whole time (the copies share HBM
                             and the fabric with the kernels): the uninterrupted run once more next to a train of copies */
    double c_fence_ms;    /* the two cross-stream hand-offs of a streamed layer (copy end -> its first kernel, its last
                             kernel -> next copy start) as the sequential run shows them, less what the timing events
                             themselves cost (a sequential pass without them is timed too, and the hand-offs are
                             reduced so that copies + executions + hand-offs add up to that pass); charged to the
                             compute stream per streamed layer by dl_timeline */
    double c_fence_hot_ms;/* what a streamed layer adds to the compute stream when its copy finished long before (the
                             wait on the already completed DMA-done event and the compute-done record drain the queue
                             between kernels): the uninterrupted run of all layers once more with those two operations
                             around every layer, minus the run without them */
    uint64_t bytes;       /* bytes one copy moves */
} dl_layer_profile;

/* Sec. II-C / Table III: runs the module in sequential mode `iters` times at (n_tokens, pos0),
 * discards the first iteration, writes per-layer means.  Every layer is copied (into a slot)
 * and timed regardless of residency.  Three more sequential passes without per-layer events and three
 * trains of all the layers' copies are each timed in one piece (c_fence_ms, c_dma_cont_ms).  Then all layers are run back to back without copies (on
 * whatever parameters the slot holds: same shapes, same cost) to time them under continuous load, and again with the
 * event protocol of a streamed layer around every layer (c_fence_hot_ms) and next to a train of copies
 * (c_exe_loaded_ms), each in turn with a plain run.  out: host array
 * [n_layers].  A last sequential pass with every layer's own parameters leaves the KV-cache rows pos0 .. pos0+n_tokens-1
 * as a real pass over x_dev writes them.  The call's temporaries (an activation block, weight copies for the continuous
 * run) come out of the arena and are returned before it ends; dl_arena_stats' peak does not include them. */
int32_t dl_profile(dl_ctx* ctx, int32_t module, int32_t n_tokens, int32_t pos0, const void* x_dev,
                   const void* ctx_dev, int32_t n_ctx, int32_t iters, dl_layer_profile* out);

typedef struct {
    double total_ms;          /* first op start to last op end, over the recorded passes */
    double dma_ms;            /* summed copy durations */
    double exe_ms;            /* summed layer execution durations */
    double exposed_ms;        /* summed time the compute stream idled on a DMA-done event */
    double hidden_frac;       /* 1 - exposed/dma (1 when nothing streamed) */
    double h2d_gbps;          /* bytes_streamed / dma_ms */
    uint64_t bytes_streamed;
    uint64_t arena_peak;
    int32_t n_layer_records;  /* layer invocations recorded */
} dl_run_stats;

typedef struct {
    int32_t module, layer, streamed, slot;
    float dma_start_ms, dma_end_ms, exe_start_ms, exe_end_ms;   /* relative to the first recorded op */
} dl_layer_record;

/* on != 0: subsequent forward passes record timing events around every copy and every layer
 * until dl_collect_stats, which synchronises, fills *stats (and up to cap per-layer records,
 * may be NULL), and resets the recording. */
int32_t dl_set_timing(dl_ctx* ctx, int32_t on);
int32_t dl_collect_stats(dl_ctx* ctx, dl_run_stats* stats, dl_layer_record* records, int32_t cap);

/* Per-kernel-class timing inside the layers (HIP events on the compute stream around every launch).
 * flops / bytes are the ALGORITHMIC work of the launches: 2*M*N*K for a linear map, 4*d_head per
 * (query, visible key) pair for attention; operands read once and results written once for bytes. */
enum {
    DL_K_NORM = 0, DL_K_GEMM_QKV = 1, DL_K_QKV_POST = 2, DL_K_ATTN = 3, DL_K_GEMM_O = 4,
    DL_K_GEMM_UP = 5, DL_K_GEMM_DOWN = 6, DL_K_CROSS = 7, DL_K_COUNT = 8
};
typedef struct {
    int32_t kind;        /* DL_K_* */
    int32_t launches;
    double total_ms;
    double flops;
    double bytes;
} dl_kernel_time;
/* mask: bit k set = time launches of class k (DL_K_*); 0 = off; -1 = every class.  Each timed launch costs
 * two event records on the compute stream, which drain the queue between kernels (a few microseconds each). */
int32_t dl_set_kernel_timing(dl_ctx* ctx, int32_t mask);
/* synchronises; out: host array [DL_K_COUNT], entry i describes kind i; resets the accumulation */
int32_t dl_collect_kernel_times(dl_ctx* ctx, dl_kernel_time* out);

/* Diagnostic, not an operation of the paper: the chip's sustained BF16 matrix-core rate with operands held in
 * registers (one workgroup of four wavefronts per compute unit, 16 independent 32x32x16 accumulator tiles each),
 * the denominator for a measured-peak MFMA utilisation.  pattern 0: zero operands, 1: hashed values in +-[1,2)
 * (the rate depends on operand toggling because the chip is power-limited).  Takes blocks*1024 bytes from the arena
 * for the duration of the call, launches on the compute stream, synchronises it, writes TFLOP/s to *tflops_out. */
int32_t dl_probe_mfma_rate(dl_ctx* ctx, int32_t pattern, int32_t iters, double* tflops_out);

/* The schedule one forward pass enqueues, as data (also recorded by host-only contexts). */
enum { DL_OP_WAIT = 0, DL_OP_RECORD = 1, DL_OP_COPY = 2, DL_OP_EXEC = 3 };
enum { DL_EV_DMA_DONE = 0, DL_EV_COMPUTE_DONE = 1, DL_EV_PASS_DONE = 2 };
enum { DL_OPF_NEXT_PASS = 1 };   /* flags of a COPY = how many passes ahead of the current one the copied layer executes
                                    (0: this pass; 1: prefetch for the next pass; up to 3 with four slots) */
typedef struct {
    int32_t queue;       /* 0 = compute stream, 1 = copy stream */
    int32_t op;          /* DL_OP_* */
    int32_t event_kind;  /* DL_EV_* for WAIT / RECORD, else -1 */
    int32_t slot;        /* slot the event / copy / exec refers to, -1 = resident exec */
    int32_t module, layer;
    int32_t flags;       /* DL_OPF_* */
} dl_trace_op;
int32_t dl_trace_enable(dl_ctx* ctx, int32_t on);
/* copies up to cap ops, *n_out = number recorded since the last read; then clears the trace */
int32_t dl_trace_read(dl_ctx* ctx, dl_trace_op* out, int32_t cap, int32_t* n_out);

/* ---- planner and predictor: pure host functions (usable with ctx == NULL semantics: no ctx taken) ---- */

/* Eq. 8 generalised to L layers: idx_out[i] = floor(i * (L-1) / k), i < k, for 1 <= k <= L-1
 * (first layer in, last layer out); k == 0: nothing; k == L: every layer.  idx_out: host, capacity k. */
int32_t dl_place_interleaved(int32_t n_layers, int32_t k, int32_t* idx_out);

/* Residency benefit by position, Eq. 4 with Tables IV-VI.  A module is used in n_phases phases per
 * inference; phase p runs reps[p] passes with per-layer execution time c_exe_ms[p] (e.g. prefill x1,
 * decode xN).  c_dma_ms, m_mib: per-layer copy time and footprint in MiB.
 * out3 = {B_first, B_middle, B_last} in ms per MiB. */
int32_t dl_benefit(double c_dma_ms, double m_mib, int32_t n_phases, const double* c_exe_ms,
                   const int32_t* reps, double* out3);
/* floor(c_dma / c_exe): the consecutive residency limit of Sec. IV-D. */
int32_t dl_consecutive_limit(double c_dma_ms, double c_exe_ms, int32_t* out);
/* Eq. 9: *out = c_total0 - k * slope, slope = B * M in ms per layer. */
int32_t dl_predict_linear(double c_total0_ms, double slope_ms_per_layer, int32_t k, double* out);

/* Predicted time of a sequence of passes: replays the schedule dl_forward enqueues (the two-event
 * protocol of Sec. IV-C(ii)) on two in-order queues.  Eq. 1, 2, 5, 6, 7 are special cases.
 * The n layer invocations of all passes are flattened: c_dma_ms[j], c_exe_ms[j] = times of
 * invocation j; streamed[j] != 0 if its parameters are copied; pass_start[j] != 0 marks the first
 * layer of a pass; module_id[j] (NULL = all the same) tells passes over different stacks apart.
 * c_dma_cont_ms (NULL = same as c_dma_ms): copy time of invocation j when its copy starts at the very
 * instant the previous copy ended, i.e. the copy queue did not wait in between (dl_profile measures both).
 * c_exe_idle_ms (NULL = same as c_exe_ms): time of invocation j when the compute queue sat idle
 * waiting for its copy right before it (a GPU that idled runs the next kernels slower than one
 * kept busy; dl_profile measures both).  c_fence_ms (NULL = zeros): time added on the compute queue to
 * every streamed invocation for its two cross-stream hand-offs (dl_profile's c_fence_ms).  c_fence_hot_ms (NULL =
 * same as c_fence_ms): that time for a streamed invocation whose copy was complete when the compute queue reached
 * it (the queue did not idle: dl_profile's c_fence_hot_ms).  c_exe_loaded_ms (NULL = no slow-down): time of
 * invocation j if a copy ran throughout; an execution then advances at the rate c_exe / c_exe_loaded during the parts
 * of it that overlap a copy already placed on the copy queue (with more than two slots a copy enqueued behind the
 * execution can still start under it: that overlap is not counted).
 * mode, wrap_prefetch: as dl_set_mode; n_slots: as dl_set_slot_count (1 .. 4).  overhead_ms is added to every
 * execution (fixed host/launch cost).  Outputs (any may be NULL): total_ms; exposed_ms = time the compute queue
 * idled on DMA-done while that copy was in flight; hidden_frac = 1 - exposed / summed copy time. */
int32_t dl_timeline(const double* c_dma_ms, const double* c_dma_cont_ms, const double* c_exe_ms,
                    const double* c_exe_idle_ms, const double* c_exe_loaded_ms, const double* c_fence_ms,
                    const double* c_fence_hot_ms, const uint8_t* streamed, const uint8_t* pass_start, const int32_t* module_id, int32_t n,
                    int32_t mode, int32_t wrap_prefetch, int32_t n_slots, double overhead_ms,
                    double* total_ms, double* hidden_frac, double* exposed_ms);

/* Budgeted choice of resident layers over several modules from one profiling run (Sec. IV-D).
 * Per module m: n_layers[m], layer_bytes[m], b3[3*m..] = {B_first, B_mid, B_last} (ms/MiB).
 * Greedy by benefit per MiB: a module's first layer, then its middle layers, then its last layer.
 * k_out[m] = resident count for module m (indices then come from dl_place_interleaved). */
int32_t dl_plan(int32_t n_modules, const int32_t* n_layers, const uint64_t* layer_bytes,
                const double* b3, uint64_t budget_bytes, int32_t* k_out);

/* The same choice when the budget also has to hold the slots (Sec. IV-C(i)) and these are sized by the modules that
 * still stream: budget_bytes is what is left for resident layers AND slots.  A residency (k_m) costs
 * sum_m k_m * layer_bytes[m] + n_slots * max{ layer_bytes[m] : k_m < n_layers[m] } bytes, which is not monotone: the
 * last layer of the module with the largest layers gives slot memory back.  Every set F of fully resident modules is
 * tried: F's layers and the slots of the rest are paid first, the remaining bytes go to the other modules by dl_plan's
 * ranking with their last layer excluded; the candidate with the largest total benefit
 * (sum over resident layers of B * layer MiB, Tables IV-VI) wins, ties to the fewer resident bytes, then to the
 * smaller set F (as a bit mask).  n_modules <= 12.  DL_ERR_BUDGET_EXCEEDED if not even the slots of the all-streamed
 * case fit. */
int32_t dl_plan_shared_slots(int32_t n_modules, const int32_t* n_layers, const uint64_t* layer_bytes,
                             const double* b3, uint64_t budget_bytes, int32_t n_slots, int32_t* k_out);

#ifdef __cplusplus
}
#endif
#endif /* DEMAND_LAYERING_H */
