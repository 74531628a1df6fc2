/*
 * adapmoe.h - C ABI of the decode-time Mixture-of-Experts block of AdapMoE
 * (arXiv 2408.10284) for AMD MI355X (gfx950).
 *
 * Per token and per layer the block runs (Alg.1 of the paper):
 *   gate      router product, softmax, top-2 and the sensitivity-scaled
 *             activation test that decides whether the second expert runs
 *             (Sec. 2.1 Eq.1; Sec. 4.2 Eq.3, Eq.4, Eq.8);
 *   predict   the following layer's gate applied to the same input (Sec. 4.3);
 *   lookup    per-layer expert cache with LRU replacement (Sec. 4.4, Sec. 6.3);
 *   load      on-demand copy of missing experts, host DRAM -> HBM (Alg.1);
 *   compute   SwiGLU expert FFNs and their weighted sum (Sec. 2.1 Eq.2);
 *   prefetch  asynchronous copy of the predicted experts of the following
 *             layer on a side stream (Sec. 4.3, Alg.1 communication stream).
 *
 * Conventions
 *   - Every function returns 0 on success or a negative ADAPMOE_E* code; no
 *     exception or abort crosses this boundary.  adapmoe_strerror() names a
 *     code; adapmoe_last_error() gives the text of the last failure of a context.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host
 *     addresses.  The caller owns every buffer it passes.  The library borrows
 *     it for the duration of the call, except router matrices, registered
 *     expert images and bound device experts, which are borrowed until
 *     adapmoe_destroy().  The library owns its cache slots, events, side
 *     stream and small staging buffers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls enqueue work and return; outputs are valid once the stream has
 *     reached that point, unless stated otherwise.
 *   - A context is not thread-safe, and its compute calls share scratch memory
 *     (intermediate vectors, bucket lists, row counters): the work of two calls
 *     on one context must not overlap on the GPU, i.e. give them the same
 *     stream or order the streams yourself.  Separate contexts are independent.
 *   - Activations and outputs: x is [B,H] in the context's activation type
 *     (float for ADAPMOE_F32, bfloat16 bit patterns otherwise), y is [B,H]
 *     float.  ids [B,2] int32, w [B,2] float, k [B] int32.
 *   - The product path has no CPU fallback: without a usable GPU every compute
 *     call fails with ADAPMOE_EHIP.
 */
#ifndef ADAPMOE_H
#define ADAPMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  ADAPMOE_OK = 0,
  ADAPMOE_EINVAL = -1,  /* null pointer, bad dimension, id out of range, bad slot counts */
  ADAPMOE_ENOMEM = -2,  /* HBM or host allocation failed */
  ADAPMOE_ENOTREG = -3, /* expert has no registered host image */
  ADAPMOE_ENORES = -4,  /* expert FFN asked for an expert that is not resident */
  ADAPMOE_EHIP = -5,    /* HIP runtime failure (text via adapmoe_last_error) */
  ADAPMOE_ESTATE = -6   /* call not valid in the context's current state */
};

enum { ADAPMOE_F32 = 0, ADAPMOE_BF16 = 1, ADAPMOE_INT4G64 = 2, ADAPMOE_INT2G64 = 3 };

typedef struct adapmoe_ctx adapmoe_ctx;

typedef struct {
  int32_t H;       /* hidden size; multiple of 512 (bf16/int4) or 256 (f32) */
  int32_t F;       /* expert FFN size; multiple of 512 (bf16/int4) or 256 (f32) */
  int32_t N;       /* experts per layer, 2..64 */
  int32_t L;       /* layers */
  int32_t dtype;   /* ADAPMOE_F32 | ADAPMOE_BF16 | ADAPMOE_INT4G64 | ADAPMOE_INT2G64 (weights; activations f32 / bf16 / bf16 / bf16) */
  int32_t max_B;   /* largest number of tokens per call, 1..64 */
  int32_t device;  /* HIP device ordinal */
  int32_t trace_capacity; /* cache events kept in the ring (0 = tracing off) */
} adapmoe_config;

/* Cache event kinds (Sec. 4.4 / Alg.1; one record per demanded or predicted expert). */
enum {
  ADAPMOE_EV_HIT = 0,      /* demanded expert resident */
  ADAPMOE_EV_HIT_PF = 1,   /* demanded expert resident (or in a landing buffer) thanks to a prefetch, first use since;
                              a landed expert joins the layer's set if the layer owns slots (victim = evicted expert) */
  ADAPMOE_EV_MISS = 2,     /* demanded expert absent: loaded on demand (victim evicted if the layer was full) */
  ADAPMOE_EV_BYPASS = 3,   /* demanded expert absent and the layer owns no slot: loaded into a spare slot */
  ADAPMOE_EV_PF_TOUCH = 4, /* predicted expert already resident: recency refreshed */
  ADAPMOE_EV_PF_LOAD = 5,  /* predicted expert absent: copy started ahead of time into one of the layer's slots */
  ADAPMOE_EV_PF_LAND = 6   /* predicted expert absent and no slot of the layer free for it: copy started ahead of time
                              into a landing buffer outside the cache budget, kept until the layer's next demand */
};

typedef struct {
  int32_t token;  /* value last given to adapmoe_set_token */
  int32_t layer;
  int32_t kind;   /* ADAPMOE_EV_* */
  int32_t expert;
  int32_t victim; /* evicted expert id or -1 */
  int32_t slot;   /* physical slot used (informative, not part of the policy) */
} adapmoe_event;

typedef struct {
  uint64_t tokens_gated;     /* token-layers passed through moe_layer_step */
  uint64_t single_expert;    /* of which k == 1 */
  uint64_t hits, hits_after_prefetch, misses, bypasses;
  uint64_t prefetch_touches, prefetch_loads;   /* prefetch_loads counts PF_LOAD and PF_LAND */
  uint64_t h2d_bytes;        /* bytes copied host -> HBM (demand + prefetch) */
  uint64_t ffn_launches;
  uint64_t tiled_ffn;       /* experts evaluated tile by tile while their copy was still running */
  uint64_t prefetch_landed; /* of prefetch_loads: copies into landing buffers (PF_LAND) */
} adapmoe_counters_t;

const char* adapmoe_strerror(int code);
const char* adapmoe_last_error(const adapmoe_ctx* ctx);

/* ---- context ------------------------------------------------------------- */

/* Creates a context on cfg->device.  Allocates only small tables; expert
 * storage comes from cache_alloc() or adapmoe_bind_expert_dev(). */
int adapmoe_create(const adapmoe_config* cfg, adapmoe_ctx** out);
int adapmoe_destroy(adapmoe_ctx* ctx);

/* Router matrix W_g of `layer` (Eq.1): device pointer, [N,H] row-major in the
 * activation type, borrowed until destroy. */
int adapmoe_set_router(adapmoe_ctx* ctx, int layer, const void* Wg_dev);

/* Per-layer thresholds tau_l = sqrt(T / S_l) (host, L floats), S_l being the
 * layer's sensitivity sum diag(F): one expert runs iff (1-alpha) <= tau_l,
 * which is Eq.8 with the square root taken on both sides. */
int adapmoe_set_tau(adapmoe_ctx* ctx, const float* tau_host);

/* ---- expert images --------------------------------------------------------- */

/* Size in bytes of one packed expert image for this configuration. */
int adapmoe_expert_bytes(const adapmoe_config* cfg, size_t* bytes_out);

/* Host-side, offline: canonical matrices -> the streaming image the kernels read.
 * W1 (gate proj.) and W3 (up proj.) are [F,H], W2 (down proj.) is [H,F], all
 * row-major, float (ADAPMOE_F32) or bfloat16 bit patterns (ADAPMOE_BF16).
 * Image: rows of W1 and W3 interleaved ([F][2][H]) followed by W2 ([H][F]).
 * `out_host` must hold adapmoe_expert_bytes() bytes. */
int adapmoe_pack_expert(const adapmoe_config* cfg, const void* W1_host, const void* W3_host,
                        const void* W2_host, void* out_host);

/* Same for ADAPMOE_INT4G64: each matrix is given as unpacked 4-bit codes
 * (uint8 0..15, [rows,cols]) plus fp16 scale and zero per 64 consecutive
 * elements of a row ([rows, cols/64] each); decoded weight = code*scale+zero. */
int adapmoe_pack_expert_int4(const adapmoe_config* cfg,
                             const uint8_t* q1, const uint16_t* s1, const uint16_t* z1,
                             const uint8_t* q3, const uint16_t* s3, const uint16_t* z3,
                             const uint8_t* q2, const uint16_t* s2, const uint16_t* z2,
                             void* out_host);

/* Same for ADAPMOE_INT2G64 (the paper's 2-bit MoE blocks, Sec. 6.3): codes are uint8 0..3,
 * scale and zero as above; 5/16 byte per weight in the image. */
int adapmoe_pack_expert_int2(const adapmoe_config* cfg,
                             const uint8_t* q1, const uint16_t* s1, const uint16_t* z1,
                             const uint8_t* q3, const uint16_t* s3, const uint16_t* z3,
                             const uint8_t* q2, const uint16_t* s2, const uint16_t* z2,
                             void* out_host);

/* Registers the packed image of (layer, expert) held in host memory (pinned
 * memory from hipHostMalloc gives full link rate; pageable memory works but is
 * slow).  Borrowed until destroy; this is the source of demand loads and prefetch. */
int adapmoe_register_expert(adapmoe_ctx* ctx, int layer, int expert, const void* image_host, size_t bytes);

/* Declares that the packed image of (layer, expert) lives at `image_dev` in
 * caller-owned HBM for the lifetime of the context: always resident, never
 * evicted, outside the cache budget.  A layer whose N experts are all bound
 * needs no host round trip in moe_layer_step. */
int adapmoe_bind_expert_dev(adapmoe_ctx* ctx, int layer, int expert, const void* image_dev);

/* ---- cache (Sec. 4.4) ------------------------------------------------------ */

/* Pure host function: cache-size allocation by the knapsack dynamic programme
 * of Eq.16-19 over the expected on-demand loads f_{i,t} of Eq.10-15.
 * a[L] = single-expert probability, beta[L] = prefetch accuracy, C = total
 * slots.  Writes t_out[L] (0 <= t <= N, sum <= C; ties go to the smallest t,
 * two costs tie within 1e-12) and the minimum cost. */
int cache_plan(int L, int N, int C, const double* a, const double* beta, int32_t* t_out, double* cost_out);

/* Expected on-demand loads of one layer with t of N experts cached (Eq.15). */
double cache_cost(int N, int t, double a, double beta);

/* Allocates sum(slots_per_layer) + 4*max_B expert-sized slots in HBM and empties every
 * layer's LRU set.  slots_per_layer[l] in 0..N is the layer's cache size t_l of Sec. 4.4.
 * The 4*max_B spare slots are outside that budget: 2*max_B hold what a running step reads
 * beyond its layer's own slots (a layer that owns fewer slots than the step requires
 * experts), 2*max_B are landing buffers for prefetched experts of the next layer that
 * cannot take one of its slots (the on-demand-load model of Eq.11-14 credits a correct
 * prefetch at every cache size, t = 0 included, so a prefetched expert must be able to
 * land).  May be called once. */
int cache_alloc(adapmoe_ctx* ctx, const int32_t* slots_per_layer);

/* Residency query: slot_out[i] = physical slot of ids[i] in `layer` (in the layer's LRU
 * set or in one of its landing buffers), -1 if absent, -2 if bound to caller memory.
 * touch != 0 also makes entries found in the LRU set most recently used (in the order
 * given).  Host-only, no GPU work. */
int cache_lookup(adapmoe_ctx* ctx, int layer, const int32_t* ids_host, int n, int32_t* slot_out, int touch);

/* ---- the block's steps ------------------------------------------------------ */

/* Gate of `layer` on x (Eq.1, Eq.3-4, Eq.8): one workgroup per token computes
 * the N logits, the softmax, the two largest (ties: lower index), alpha and
 * the test (1-alpha) <= tau_layer.  Writes ids[b] = (e1,e2), k[b] in {1,2},
 * w[b] = (1,0) if k==1 else (alpha,1-alpha).  If pred_ids_dev/pred_k_dev are
 * non-NULL and layer+1 < L, the same kernel also applies layer+1's router and
 * threshold to the same x (Sec. 4.3) and writes that decision there
 * (pred_ids [B,2], pred_k [B]); for the last layer it writes pred_k = 0. */
int moe_gate(adapmoe_ctx* ctx, int layer, const void* x_dev, int B,
             int32_t* ids_dev, float* w_dev, int32_t* k_dev,
             int32_t* pred_ids_dev, int32_t* pred_k_dev, void* stream);

/* y[b] = sum_{j<k[b]} w[b][j] * E_{ids[b][j]}(x[b])  (Eq.2 over the activated
 * experts), E(x) = W2 (silu(W1 x) * (W3 x)).  Reads expert images through the
 * context's device-side residency table; every needed expert must be resident
 * (bound, or brought into a cache slot by moe_demand / moe_prefetch before this
 * call; the call makes `stream` wait for those copies).  A non-resident expert
 * contributes nothing and raises a device flag reported as ADAPMOE_ENORES by
 * adapmoe_check().  For a token with k == 2 the two ids must differ. */
int moe_expert_ffn(adapmoe_ctx* ctx, int layer, const void* x_dev, int B,
                   const int32_t* ids_dev, const float* w_dev, const int32_t* k_dev,
                   float* y_dev, void* stream);

/* Demand phase of Alg.1 for `layer` (to_transfer <- E.in_CPU): the experts
 * ids_host[b][0 .. k_host[b]-1] of the B tokens, in token then rank order, are looked up
 * in the layer's LRU set and landing buffers.  Found -> most recently used (HIT, HIT_PF);
 * absent -> least recently used entry evicted if the layer is full and an asynchronous copy
 * started on the library's side stream (MISS), or into a spare slot if the layer owns no
 * slot (BYPASS).  Prefetched experts in landing buffers that are not required are dropped.
 * Host-side only; *loads_out (may be NULL) = number of on-demand loads started.
 * The call must be followed by moe_expert_ffn() on the same layer, which waits for these
 * copies on its stream, evaluates the experts and ends the step; a second moe_demand()
 * before that returns ADAPMOE_ESTATE.  moe_layer_step() is this call, moe_prefetch() for
 * the predicted experts and moe_expert_ffn() in one. */
int moe_demand(adapmoe_ctx* ctx, int layer, const int32_t* ids_host, const int32_t* k_host, int B, int32_t* loads_out);

/* moe_expert_ffn for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  No context: the shape (H, F, N, dtype as in
 * adapmoe_config) and the residency table - table_dev, a device array of N image base pointers,
 * NULL = expert absent - are arguments; x, ids, w, k, y as for moe_expert_ffn, on the current
 * device.  The intermediate vectors live in a fixed device array inside the library (640 KiB per
 * GPU, held until the process ends), so the call is limited to B <= 4 tokens and F <= 16384 and
 * returns ADAPMOE_EINVAL beyond that; it always takes the weight-streaming (GEMV) kernels, also
 * where moe_expert_ffn would take the batched path.  It calls no hipMalloc, hipFree or other
 * allocating routine.  The first call on a GPU looks the array up and prepares the kernels
 * (synchronous; make it outside a capture).  err_dev: optional device word that receives the
 * flags (bit 0: an activated expert was absent and contributed nothing, bit 1: id out of range);
 * NULL = flags dropped.  All calls on one GPU share the array, whatever their stream: calls that
 * overlap on a GPU race; order them on one stream or with events. */
int moe_expert_ffn_static(int32_t H, int32_t F, int32_t N, int32_t dtype, const void* const* table_dev,
                          const void* x_dev, int B, const int32_t* ids_dev, const float* w_dev, const int32_t* k_dev,
                          float* y_dev, int32_t* err_dev, void* stream);

/* Prefetch for `layer` (Sec. 4.3), ids in rank order.  At most as many of them as the layer
 * owns slots go to its LRU set: resident -> most recently used; absent -> evict LRU if
 * full, start an asynchronous copy on the library's side stream.  The others are copied
 * into landing buffers outside the budget (at most 2*max_B per layer; further ones are
 * left out) and kept until the layer's next demand (moe_demand / moe_layer_step, or a
 * moe_expert_ffn that no moe_demand preceded).  Returns at once. */
int moe_prefetch(adapmoe_ctx* ctx, int layer, const int32_t* ids_host, int n);

/* One layer of Alg.1 for B tokens: gate + predict; (if the layer is not fully
 * bound: bring ids to the host, demand lookup, start copies of missing
 * experts, then the predicted experts of layer+1, on the side stream, and make
 * `stream` wait for the demanded copies only); expert FFNs + combine into y.
 * With B > 1 the demanded set is the union over tokens in token order. */
int moe_layer_step(adapmoe_ctx* ctx, int layer, const void* x_dev, int B, float* y_dev, void* stream);

/* Residual wiring used between blocks by multi-layer runs (not from the paper):
 * h[b] += gamma * y[b] (skipped if y_dev is NULL), then
 * x[b] = h[b] / sqrt(mean(h[b]^2) + 1e-6) stored in the activation type.
 * h [B,H] float, y [B,H] float, x [B,H]. */
int moe_residual_rmsnorm(adapmoe_ctx* ctx, float* h_dev, const float* y_dev, float gamma,
                         void* x_dev, int B, void* stream);

/* One token step through all L layers with the wiring above (not from the
 * paper): for l = 0..L-1: x = norm(h) (h first updated with gamma*y of the layer
 * before), moe_layer_step(l, x) -> y; finally h += gamma*y of the last layer.
 * h [B,H] float is updated in place; x [B,H] (activation type) and y [B,H]
 * float are work buffers owned by the caller.  Sets the trace token to `token`. */
int moe_stack_token(adapmoe_ctx* ctx, int token, float* h_dev, void* x_dev, float* y_dev, int B, float gamma, void* stream);

/* Predictive gate for the first layer (Sec. 4.3, Eq.9).  Gpre_dev: device matrix [N,H] in the
 * activation type, borrowed until replaced or the context is destroyed; null switches it off
 * (default: layer 0 is served by its LRU set only).  When set, moe_layer_step on the last layer also
 * applies Gpre to that layer's block input, takes the adaptive decision with layer 0's threshold
 * and prefetches the predicted experts into layer 0's cache for the following token; the decision
 * is reported as the depth-1 prediction of that step.  Training the matrix is the caller's business.
 * A one-layer context has no "last layer of the previous token" distinct from the layer that is
 * running, so the call returns ADAPMOE_ESTATE when L == 1. */
int adapmoe_set_first_layer_predictor(adapmoe_ctx* ctx, const void* Gpre_dev);

/* Tile-wise loading (Sec. 5, Fig.6(b) and Alg.1: tile-wise scheduling).  tiles = 0 or 1: an expert image
 * is one copy and the expert FFN waits for all of it (default).  tiles >= 2 (at most 64): every
 * copy is issued as `tiles` blocks of gate/up row pairs followed by tiles/2 blocks of W2 rows, each
 * with its own event; a single-token moe_layer_step whose expert is still arriving evaluates the
 * experts already in HBM first and then the arriving one block by block, each launch waiting only
 * for the block it reads.  Cache decisions, events and counters are the same in both modes; outputs
 * agree up to the order of the final additions.  Calls with B > 1 wait for whole images. */
int adapmoe_set_tiles(adapmoe_ctx* ctx, int tiles);

/* Expert images in pageable host memory (Alg.1's transfer queue with the host copy as an extra
 * stage; for stacks larger than the process may pin).  buffers >= 2 (at most 16): every load is
 * served by a worker thread of the library, in request order: it copies the registered image into
 * one of `buffers` pinned buffers of one image each (owned by the library; `host_threads` threads
 * share the copy, 0 = 6) and sends it from there to its slot on the side stream, so the host copy of
 * one image runs while the previous one crosses the link; an image that finds the link idle is
 * staged and sent in pieces of 32 MiB instead, so that its transfer starts after the first piece.
 * Cache decisions, events and results are unchanged; tile-wise loading is not used for staged copies.  buffers = 0 switches staging off
 * (images are then read directly and should be pinned).  Call between layer steps. */
int adapmoe_set_staging(adapmoe_ctx* ctx, int buffers, int host_threads);

/* Look-ahead depth of moe_layer_step, 1..3 (default 1) (Sec. 4.3, prefetch beyond the next layer).
 * With depth D the gate launch also applies the routers of layers l+2 .. l+D to the
 * same input.  The prediction for layer l+d (d >= 2) is acted on only when every
 * expert predicted for layer l+d-1 was already resident (its prefetch issued no
 * transfer); the first depth that needs a transfer ends the look-ahead of this step.
 * Returns ADAPMOE_EINVAL outside 1..3. */
int adapmoe_set_lookahead(adapmoe_ctx* ctx, int depth);
/* Prediction of depth d (1..3) of the last moe_layer_step on a non-bound layer. */
int adapmoe_last_lookahead(adapmoe_ctx* ctx, int depth, int32_t* pred_ids, int32_t* pred_k, int B);

/* ---- tuning options -------------------------------------------------------------- */

/* Options that select a code path or a launch shape.  None changes what is computed beyond
 * the order of floating-point additions, except BATCH_TWO_TERMS (precision of the batched
 * path's intermediate activation).  Set between calls, not while work of the context is
 * being captured into a graph. */
enum {
  ADAPMOE_OPT_BATCH_MIN = 0,       /* tokens per call from which bf16 calls take the batched (matrix-core) path; default 3, >= 1 */
  ADAPMOE_OPT_BATCH_TWO_TERMS = 1, /* batched down GEMM multiplies the intermediate activation as hi + lo bfloat16 (1) or rounded
                                      to bfloat16 (0, default) */
  ADAPMOE_OPT_FUSED = 2,           /* 1: single-token steps on fp32/bf16 experts run both GEMVs in one launch joined by a bounded
                                      grid-wide barrier (slower on MI355X, default 0); ADAPMOE_ESTATE if the shape does not fit */
  ADAPMOE_OPT_DYN_PCT = 3,         /* percent of the gate/up GEMV's row passes handed out dynamically, 0..100 (default 20; fp32/bf16
                                      experts only, the quantised kernels assign every row in advance) */
  ADAPMOE_OPT_GATEUP_BLOCKS = 4,   /* workgroups of the gate/up GEMV, 1..65535 */
  ADAPMOE_OPT_DOWN_BLOCKS = 5,     /* workgroups of the fp32/bf16 down GEMV, 1..65535 */
  ADAPMOE_OPT_BATCH_DIRECT = 6,    /* batched gate/up GEMM: 2 (default) one workgroup per compute unit, every wavefront streams
                                      through its row tiles without a break; 1 one row tile per workgroup, wavefronts load their
                                      token operand themselves; 0 one row tile per workgroup, operand staged through LDS.
                                      Same results in all three. */
  ADAPMOE_OPT_POISON_SLOTS = 7     /* debugging aid for the ordering of copies and kernels (default 0): 1 fills a cache slot
                                      with all-ones bytes (not-a-number in every storage type, scales and zeros of the
                                      quantised types included) on the side stream right before each copy into it, so that a
                                      kernel reading the slot before its copy has landed, or a copy starting while a kernel
                                      still reads the slot's previous expert, shows up as non-finite output instead of as
                                      plausible numbers.  Costs one fill per load. */
};
int adapmoe_set_option(adapmoe_ctx* ctx, int option, int value);
int adapmoe_get_option(adapmoe_ctx* ctx, int option, int* value_out);

/* ---- bookkeeping ------------------------------------------------------------- */

int adapmoe_set_token(adapmoe_ctx* ctx, int token);
/* Copies up to cap oldest unread events into buf and removes them from the ring. */
int adapmoe_trace_read(adapmoe_ctx* ctx, adapmoe_event* buf, size_t cap, size_t* n_out);
int adapmoe_counters(adapmoe_ctx* ctx, adapmoe_counters_t* out);
/* Last gate decision brought to the host by moe_layer_step on a non-bound layer
 * (ids [B,2], k [B], pred_ids [B,2], pred_k [B]); any pointer may be NULL. */
int adapmoe_last_decision(adapmoe_ctx* ctx, int32_t* ids, int32_t* k, int32_t* pred_ids, int32_t* pred_k, int B);
/* Decision log (tracing aid; the gate results of steps that make no host round trip are
 * otherwise not visible): while log_dev is non-NULL every moe_layer_step (also inside
 * moe_stack_token) appends one record of 6*max_B int32 to the caller's device buffer
 * log_dev, which holds `capacity` records: ids [B,2], k [B], then the prediction for the
 * next layer pred_ids [B,2], pred_k [B] (Sec. 4.3) when the step computed one (steps on
 * layers whose experts and whose successor's experts are all bound compute none and leave
 * that part unspecified); the first 6*B entries are used.  The copy is enqueued on the
 * step's stream after the gate.  Appending stops when the buffer is full.  Setting the log
 * (or NULL) restarts at record 0.  Not to be used while a stream is being captured into a
 * graph (the record position is decided on the host). */
int adapmoe_set_decision_log(adapmoe_ctx* ctx, int32_t* log_dev, int capacity);

/* Waits for all work of the context (both streams given so far) and reports
 * device-side flags: ADAPMOE_ENORES if an FFN met a non-resident expert. */
int adapmoe_check(adapmoe_ctx* ctx, void* stream);

/* Kernel timing with HIP events on the launch stream: when on, every launch of
 * the gate and expert-FFN kernels carries a pair of events tied to its own
 * dispatch, so the durations are the kernels' execution times (what a profiler's
 * kernel trace reports), without the dispatch gaps that events recorded around a
 * launch would include; the fused kernel and tile-wise launches are bracketed by
 * event records.  Not to be switched on while a stream is being captured into a
 * graph.  adapmoe_profile_read
 * synchronises and returns, per kernel class (0 = gate/up GEMV, 1 = down GEMV,
 * 2 = gate), the number of launches and their summed duration in ms, then resets.
 * Further classes: 3 bucket/gather, 4 grouped gate/up GEMM, 5 grouped down GEMM
 * (batched path), 6 fused single-token FFN (gate/up + down in one launch). */
int adapmoe_profile(adapmoe_ctx* ctx, int on);
int adapmoe_profile_read(adapmoe_ctx* ctx, int kernel_class, uint64_t* launches, double* total_ms);

/* Measurement aid: what the memory system delivers for the access pattern of a kernel, without the
 * kernel's arithmetic.  Launches `reps` load-only kernels over the matrix buf_dev (device memory,
 * nrows rows of row_bytes) on `stream`, timed with a pair of events, and returns the average duration
 * of one pass in microseconds.  A wavefront reads units of rows_per_unit consecutive rows, chunk_bytes
 * of each row per step, with two 16 KiB register buffers in flight as the expert kernels have:
 * (rows_per_unit 2, chunk_bytes = row_bytes) is the single-token gate/up GEMV reading a row pair,
 * (32, 512) the grouped GEMM of the batched path.  chunk_bytes is 512 or equal to row_bytes (a multiple of
 * 1024 up to 16384); rows_per_unit * chunk_bytes must be a multiple of 16384 and nrows of
 * rows_per_unit; workgroups (256 threads) in 1..65535.  Reads only; ADAPMOE_EINVAL otherwise. */
int adapmoe_stream_probe(const void* buf_dev, int64_t nrows, int row_bytes, int rows_per_unit, int chunk_bytes,
                         int workgroups, int reps, double* us_per_pass_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ADAPMOE_H */
