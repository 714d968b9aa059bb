/*
 * libkvp — time-to-first-token path of KV Prediction (arXiv 2410.08391) on one MI355X (gfx950).
 *
 * The path (Sec. 4.1, Algorithm "KV Prediction Inference", first four statements):
 *     a, KV_A <- A(I)            auxiliary transformer, causal pass over the whole prompt
 *     KV^_B   <- P(KV_A)         per-base-layer linear maps of the auxiliary cache (Sec. 4.2)
 *     b       <- B(I[-1], KV^_B) one base-model step on the last prompt token, attending over
 *                                the predicted cache instead of the base model's own K/V
 *     first   <- argmax(b)
 *
 * Conventions
 *   - Plain C ABI.  No call aborts, prints or throws; every call returns a status
 *     (0 = KVP_OK, negative = error) and kvp_last_error() gives a thread-local message.
 *   - "device" pointers are HIP device memory of the current device, owned by the caller,
 *     and must stay valid until the stream work that uses them has finished.  "host"
 *     pointers are ordinary memory read during the call only.
 *   - Work is enqueued on the caller's HIP stream; calls return without synchronising.  (The
 *     bf16 path may run part of the work on an internal stream that forks from and joins back
 *     into the caller's stream inside the call; nothing outlives the join.  KVP_NO_OVERLAP=1 in
 *     the environment at kvp_load_weights time disables this.)
 *   - Device memory: kvp_load_weights allocates the few small tables a handle owns (two rotary
 *     tables of max_seq x head_dim / 2 float2 each, one flag word, the predictor's pointer and
 *     layer-map tables) and kvp_free releases them.  No other call allocates or frees device
 *     memory: all per-call scratch comes in as `workspace` (or, for kvp_generation_step_static,
 *     lives in a static array inside the library).
 *   - Matrices are row-major [out_features, in_features] (y = W x), element type per
 *     kvp_config.dtype: float (KVP_DTYPE_F32) or bfloat16 (KVP_DTYPE_BF16).
 *   - Transformer block (fixed by the benchmark configurations, the paper only says
 *     "transformer"): pre-norm RMSNorm (eps inside the root), rotary embedding in the
 *     rotate-half pairing (dim d pairs with d + head_dim/2, angle pos * theta^(-2d/head_dim)),
 *     grouped-query softmax attention scaled by 1/sqrt(head_dim) with query head h reading
 *     kv head h / (n_q_heads / n_kv_heads), SwiGLU feed-forward, no biases.
 */
#ifndef KVP_H
#define KVP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVP_OK 0
#define KVP_ERR_NULL (-1)                /* a required pointer was NULL */
#define KVP_ERR_BAD_CONFIG (-2)          /* shapes the kernels cannot serve, bad layer map */
#define KVP_ERR_BAD_SHAPE (-3)           /* B, T, T_cap out of range for this handle */
#define KVP_ERR_WORKSPACE_TOO_SMALL (-4)
#define KVP_ERR_HIP (-5)                 /* a HIP runtime call failed; message has the code */
#define KVP_ERR_UNIMPLEMENTED (-6)

#define KVP_DTYPE_F32 0
#define KVP_DTYPE_BF16 1

/* Bits of the device-side flag word, read with kvp_check_flags. */
#define KVP_FLAG_TOKEN_CLAMPED 1u  /* a token id outside [0, vocab) was clamped into range */

/* Size of the static scratch array behind kvp_generation_step_static (8 MiB per GPU). */
#define KVP_STATIC_SCRATCH_BYTES (8u << 20)

/* Stages of the path, for kvp_run_stages. */
#define KVP_STAGE_AUX 1u       /* auxiliary prefill -> auxiliary cache in the workspace      */
#define KVP_STAGE_PREDICT 2u   /* predictor: auxiliary cache -> caller's base cache          */
#define KVP_STAGE_BASE 4u      /* base step over the base cache -> logits, argmax           */
#define KVP_STAGE_ALL 7u
/* The same base step with the predictor absorbed into its attention (Sec. 4.2 "Predictor
 * Networks": the maps are linear, so q . (W_K k_A) = (W_K^T q) . k_A and
 * sum_u p_u W_V v_A,u = W_V sum_u p_u v_A,u): it reads the AUXILIARY cache in the workspace and
 * needs no predicted cache, so the first token does not wait for KVP_STAGE_PREDICT.  Equal to
 * KVP_STAGE_BASE in exact arithmetic, rounded in another order.  Give it in place of
 * KVP_STAGE_BASE (never both); with KVP_STAGE_AUX | KVP_STAGE_PREDICT in the same call the cache
 * is written beside the last base layers, for the generation loop.  k_cache / v_cache may be
 * NULL when KVP_STAGE_PREDICT is not asked for.  Serves auxiliary widths n_kv_heads * head_dim
 * that are a power of two in [16, 512], base query groups up to 8 and head_dim up to 256;
 * KVP_ERR_UNIMPLEMENTED otherwise. */
#define KVP_STAGE_BASE_ABSORBED 8u

/* Kernel classes, for the per-class timers (kvp_profile_*). */
enum {
  KVP_KC_EMBED_NORM = 0, /* embedding gather, RMSNorm, rotary, SiLU*mul when run as own kernels */
  KVP_KC_AUX_GEMM = 1,   /* auxiliary QKV / O / gate-up / down projections                     */
  KVP_KC_AUX_ATTN = 2,   /* causal grouped-query flash attention                               */
  KVP_KC_PREDICTOR = 3,  /* predictor GEMMs writing the base cache                             */
  KVP_KC_BASE_GEMV = 4,  /* base-step projections and LM head (weight streaming)               */
  KVP_KC_DECODE_ATTN = 5,/* base-step attention over the predicted cache (+ split combine)     */
  KVP_KC_ARGMAX = 6,
  KVP_KC_COUNT = 7
};

typedef struct kvp_handle kvp_handle;

/* One decoder stack. head_dim must be even; n_q_heads % n_kv_heads == 0.
 * Layers of different width (OpenELM's layer-wise scaling; the paper's models, Sec. 4.2
 * "Architectural Details"): optional HOST arrays of n_layers entries each, copied by
 * kvp_load_weights; NULL = every layer has the scalar width.  When given, layer l has
 * layer_n_q_heads[l] query heads, layer_n_kv_heads[l] key/value heads and a feed-forward width of
 * layer_ffn_dim[l], its matrices have exactly those shapes, and the scalar fields must be the
 * maxima over the layers (they size buffers and caches).  Give all three arrays or none. */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim;
  const int32_t* layer_n_q_heads;
  const int32_t* layer_n_kv_heads;
  const int32_t* layer_ffn_dim;
} kvp_model_shape;

typedef struct {
  kvp_model_shape base, aux;
  int32_t vocab;            /* shared by both models */
  int32_t dtype;            /* KVP_DTYPE_* : element type of weights, activations and caches */
  float rope_theta;
  float rms_eps;
  const int32_t* layer_map; /* host, [base.n_layers]; layer_map[i] = j_i in [0, aux.n_layers): the
                               auxiliary layer whose cache feeds base layer i (Sec. 4.2, Table 1).
                               Copied by kvp_load_weights. */
  int32_t max_batch, max_seq; /* upper bounds for B and T of later calls */
} kvp_config;

/* Weights of one stack.  Per-layer members are HOST arrays of n_layers DEVICE pointers.  Every
 * device pointer (here, the predictor's, and the caches / logits of the calls below) must be
 * 16-byte aligned: KVP_ERR_BAD_CONFIG from kvp_load_weights, KVP_ERR_BAD_SHAPE from the calls.
 *   embed [vocab, d_model]            attn_norm, ffn_norm [d_model]
 *   wq [n_q*hd, d_model]   wk, wv [n_kv*hd, d_model]   wo [d_model, n_q*hd]
 *   w_gate, w_up [ffn, d_model]       w_down [d_model, ffn]
 *   final_norm [d_model]   lm_head [vocab, d_model]
 * The auxiliary stack's final_norm / lm_head are never read (its logits are unused at
 * inference, Sec. 4.3) and may be NULL; the base stack's wk / wv are not read by this path
 * (the predicted cache replaces them, Sec. 4.1) and may be NULL. */
typedef struct {
  const void* embed;
  const void* final_norm;
  const void* lm_head;
  const void* const* attn_norm;
  const void* const* wq;
  const void* const* wk;
  const void* const* wv;
  const void* const* wo;
  const void* const* ffn_norm;
  const void* const* w_gate;
  const void* const* w_up;
  const void* const* w_down;
  /* Optional query / key normalisation (the OpenELM trait that Sec. 7 "Analysis" refers to; the
   * paper gives no formula, the reading is OpenELM's): RMSNorm over head_dim of every query and
   * key head, gains [head_dim] per layer, applied before the rotary embedding.  Both NULL: the
   * stack has no such norm.  A stack has it for all layers or for none.  The auxiliary stack
   * needs both arrays; the base stack's k_norm is read only by kvp_reference_prefill and
   * kvp_generation_step and may be NULL for kvp_prefill_predict. */
  const void* const* q_norm;
  const void* const* k_norm;
} kvp_model_weights;

typedef struct {
  kvp_model_weights base, aux;
  /* Predictor F_i (Sec. 4.2): HOST arrays of base.n_layers DEVICE pointers, each
   * [base.n_kv*hd, aux.n_kv*hd]; pred_wk maps post-rotary auxiliary keys, pred_wv values. */
  const void* const* pred_wk;
  const void* const* pred_wv;
} kvp_weights;

/* Cache layout with layers of different width: the cache is base.n_layers blocks of
 * B * base.n_kv_heads * T_cap * head_dim elements (n_kv_heads = the maximum); block i starts with
 * the dense array [B][layer_n_kv_heads[i]][T_cap][head_dim] of layer i and the rest of the block is
 * not touched.  With one width per stack this is the plain [L][B][n_kv][T_cap][hd] array. */

/* Validates the configuration, records the (borrowed) device pointers and builds the launch
 * plan.  Copies nothing large; the weights must outlive the handle.  Allocates, on the current
 * device, the small tables the handle owns (rotary tables, flag word, predictor pointer tables:
 * a few MB for max_seq = 8192) and synchronises the device once; later calls on this handle
 * must run with the same device current.
 * Errors: KVP_ERR_NULL, KVP_ERR_BAD_CONFIG, KVP_ERR_HIP.  On error *out is set to NULL. */
int kvp_load_weights(const kvp_config* cfg, const kvp_weights* weights, kvp_handle** out);

/* Bytes of device scratch kvp_prefill_predict needs for a B x T prompt batch (auxiliary cache,
 * activations, split-attention partials).  0 if the handle is NULL or B/T are out of range.
 * For a fixed B the value does not decrease with T, so a buffer sized for T also serves shorter
 * prompts of B sequences; it is NOT monotone in B (the number of attention splits per sequence
 * shrinks as the batch grows): a buffer meant for several batch sizes takes the maximum over them. */
size_t kvp_workspace_bytes(const kvp_handle* h, int32_t B, int32_t T);

/* The whole path (Algorithm "KV Prediction Inference", statements 1-4) for B prompts of T tokens.
 *   tokens     device int32 [B, T]; ids outside [0, vocab) are clamped into range, and the clamp is
 *              recorded in the handle's flag word (kvp_check_flags): a range check on the host
 *              would need the ids there, which costs a synchronisation the path avoids.
 *   k_cache,
 *   v_cache    device, element type per config, [base.n_layers][B][base.n_kv][T_cap][head_dim];
 *              receives the predicted keys / values for positions 0..T-1; slots T..T_cap-1 are
 *              left untouched (room for a later generation loop).
 *   logits     device float [B, vocab], first-token logits b; may be NULL.
 *   argmax     device int32 [B], greedy first token (lowest index among equal maxima); may be
 *              NULL only if logits is not.
 *   workspace  device, >= kvp_workspace_bytes(h, B, T) bytes, 256-byte aligned.
 *   hip_stream a hipStream_t (NULL = the default stream).
 * Errors: KVP_ERR_NULL, KVP_ERR_BAD_SHAPE (B < 1, T < 1, B > max_batch, T > max_seq, T > T_cap),
 * KVP_ERR_WORKSPACE_TOO_SMALL, KVP_ERR_HIP.  Nothing is enqueued when an error is returned
 * before the first launch.
 * The call allocates nothing, synchronises nothing and enqueues kernels only (plus event record /
 * wait between hip_stream and the handle's internal stream), so it may be captured into a HIP
 * graph through hip_stream; one handle serves one call at a time (its internal stream and events,
 * and the workspace, are shared). */
int kvp_prefill_predict(kvp_handle* h, const int32_t* tokens, int32_t B, int32_t T,
                        void* k_cache, void* v_cache, int64_t T_cap,
                        float* logits, int32_t* argmax,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* Same as kvp_prefill_predict but runs only the stages in `stages` (KVP_STAGE_* bits), reading
 * what earlier stages of a previous call left in the workspace / caches.  For tests and for
 * timing the stages separately. */
int kvp_run_stages(kvp_handle* h, uint32_t stages, const int32_t* tokens, int32_t B, int32_t T,
                   void* k_cache, void* v_cache, int64_t T_cap,
                   float* logits, int32_t* argmax,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/* Where the auxiliary cache KV_A (Sec. 4.2) lives inside the workspace after KVP_STAGE_AUX:
 * byte offsets of two arrays [aux.n_layers][B*T][aux.n_kv*head_dim] (token-major, feature =
 * kv_head*head_dim + dim; keys post-rotary), element type per config.  With layers of different
 * width each layer's block has the widest layer's size and starts with that layer's dense
 * [B*T][layer_n_kv_heads[l]*head_dim] array. */
int kvp_aux_cache_offsets(const kvp_handle* h, int32_t B, int32_t T, size_t* k_offset, size_t* v_offset);

/* Ordinary inference of ONE of the two models, on the same kernels: the reference points of the
 * paper's timing experiments (Sec. 6.3 "Timing Experiments": time to first token of the base model, and of the
 * small model alone; T_B(N) and T_A(N) of Sec. 4.4).  A causal pass of the whole stack over the
 * prompt, every layer complete, then final norm and LM head on the last position.
 *   model      KVP_MODEL_BASE or KVP_MODEL_AUX.  That stack's wk / wv, final_norm and lm_head
 *              must have been given to kvp_load_weights (KVP_ERR_NULL otherwise).
 *   k_cache,
 *   v_cache    device, [n_layers][B][n_kv][T_cap][head_dim] of THAT model, or both NULL: the
 *              model's own keys (post-rotary) / values for positions 0..T-1.
 *   logits / argmax / workspace / hip_stream: as for kvp_prefill_predict, workspace >=
 *              kvp_reference_workspace_bytes(h, model, B, T).
 * Runs on the caller's stream only.  Errors as kvp_prefill_predict. */
#define KVP_MODEL_BASE 0
#define KVP_MODEL_AUX 1
size_t kvp_reference_workspace_bytes(const kvp_handle* h, int32_t model, int32_t B, int32_t T);
int kvp_reference_prefill(kvp_handle* h, int32_t model, const int32_t* tokens, int32_t B, int32_t T,
                          void* k_cache, void* v_cache, int64_t T_cap,
                          float* logits, int32_t* argmax,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* The handle's device-side flag word (KVP_FLAG_* bits, set by kernels of earlier calls on this
 * handle; Sec. 4.1's algorithm takes token ids I as given, so an id outside the vocabulary is the
 * caller's error, reported here instead of read out of bounds).  Copies 4 bytes to the host with
 * a blocking copy: synchronise the stream(s) the calls were enqueued on first, or bits of work
 * still in flight are missed.  clear != 0 resets the word after reading.  Not for use during
 * graph capture.
 *   flags_out  host uint32.
 * Errors: KVP_ERR_NULL, KVP_ERR_HIP. */
int kvp_check_flags(kvp_handle* h, uint32_t* flags_out, int32_t clear);

/* One pass of the generation loop that follows the first token (Sec. 4.1 "Inference", Algorithm
 * "KV Prediction Inference": p, y <- B(y, KV)): the base model alone processes, for every sequence,
 * the token it produced last.  Unlike the first-token step it computes its OWN key and value for
 * that token, rotates the key to position pos and appends both to the cache, so the cache holds the
 * predicted entries of the prompt followed by true base entries.
 *   tokens     device int32 [B]: the token fed at this step (position pos), e.g. the previous argmax.
 *   pos        entries already in the cache (T after kvp_prefill_predict, then T + 1, ...);
 *              pos + 1 <= max_seq and pos + 1 <= T_cap.
 *   k_cache,
 *   v_cache    as for kvp_prefill_predict; slot pos of every layer is written, 0..pos are read.
 *   logits / argmax: as for kvp_prefill_predict (the distribution of the token after position pos).
 *   workspace  >= kvp_generation_workspace_bytes(h, B, pos + 1) bytes, 256-byte aligned (the base
 *              step's activations, split partials and logits only: a few MB; it does not shrink
 *              as pos grows, so size it for the longest total length once).  It may be the
 *              buffer kvp_prefill_predict used: the step then overwrites the start of what that
 *              call left there, the auxiliary cache included.
 * Needs base.wk / base.wv (KVP_ERR_NULL if they were not given).  Caller's stream only. */
size_t kvp_generation_workspace_bytes(const kvp_handle* h, int32_t B, int32_t T_total);
int kvp_generation_step(kvp_handle* h, const int32_t* tokens, int32_t B, int32_t pos,
                        void* k_cache, void* v_cache, int64_t T_cap,
                        float* logits, int32_t* argmax,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* kvp_generation_step for callers that cannot allocate or pass scratch memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and errors as kvp_generation_step, bit for bit, without the workspace: the scratch is a static
 * device array of KVP_STATIC_SCRATCH_BYTES inside the library (each GPU the library runs on holds
 * it until the process ends; its address on the handle's device is looked up by kvp_load_weights).
 * The call allocates nothing, frees nothing, synchronises nothing and enqueues kernels only.
 *   - KVP_ERR_WORKSPACE_TOO_SMALL when kvp_generation_workspace_bytes(h, B, pos + 1) exceeds
 *     KVP_STATIC_SCRATCH_BYTES (the five benchmark configurations need 0.02 - 3.7 MB);
 *   - KVP_ERR_BAD_CONFIG when the current device is not the one the handle was loaded on;
 *   - KVP_ERR_BAD_SHAPE while the per-class timers are enabled (they create events).
 * Every call on a GPU shares that GPU's array, whatever the handle: calls that overlap in time on
 * one GPU (two streams, two handles, two threads) race on it.  Nothing in it has to start at zero:
 * each kernel of the step writes what the next one reads. */
size_t kvp_static_scratch_bytes(void);
int kvp_generation_step_static(kvp_handle* h, const int32_t* tokens, int32_t B, int32_t pos,
                               void* k_cache, void* v_cache, int64_t T_cap,
                               float* logits, int32_t* argmax, void* hip_stream);

/* The workspace plan of a B x T call to kvp_prefill_predict / kvp_run_stages, for tests and
 * tools: every region the library carves out of the workspace, in address order.  Runs entirely on
 * the host (no device, no weights needed): the same planner the calls use, applied to `cfg`.
 *   regions        host array of `capacity` entries, may be NULL to query the count only.
 *   n_regions      host: number of regions of the plan (also when it exceeds capacity).
 *   total_bytes    host: what kvp_workspace_bytes returns for this shape.
 * A region's `bytes` is what the planner reserved; `bytes_touched` is what the kernels of such a
 * call read or write there according to the launch-side shape rules (number of attention splits
 * and the like).  Regions never overlap and bytes_touched <= bytes; a test checks both over a
 * grid of shapes.  Errors: KVP_ERR_NULL, KVP_ERR_BAD_CONFIG, KVP_ERR_BAD_SHAPE. */
typedef struct {
  char name[24];
  uint64_t offset, bytes, bytes_touched;
} kvp_plan_region;
int kvp_debug_plan(const kvp_config* cfg, int32_t B, int32_t T, kvp_plan_region* regions, int32_t capacity,
                   int32_t* n_regions, uint64_t* total_bytes);

/* Test aid.  The attention kernels of the bf16 prefill keep one softmax reference per query row,
 * fixed by the row's first key tile, and re-reference a tile (raise the reference to the tile's
 * maximum, rescale, recompute) only when the sum of its probabilities in a lane exceeds a guard
 * value, 2^20 by default.  This sets the guard for the whole process (limit <= 0 restores the
 * default); a tiny value sends every tile through the re-referencing path, which tests use to
 * check that path against the oracle.  Results are correct for any positive value. */
void kvp_debug_flash_guard(float limit);

/* Achievable-peak probes (measurement aids, not part of the path): plain kernels of known work
 * whose rate is what this chip sustains on the two roofs the path's kernels are priced against.
 * Both only enqueue one kernel on hip_stream; the caller times it (HIP events on that stream).
 * kvp_probe_mfma: a register-resident loop of the matrix-core instruction all GEMM and attention
 *   kernels here use (v_mfma_f32_32x32x16_bf16), no memory traffic; *flops_out (host) receives the
 *   floating-point operations the launch performs; sink: device, >= 4 bytes, never written in
 *   practice.
 * kvp_probe_stream: kind 0 reads `bytes` from src (contiguous share per block, non-temporal loads:
 *   the fastest way found to stream from memory on this chip), 1 copies src -> dst, 2 fills dst;
 *   src / dst device, 16-byte aligned, `bytes` long (kind 0 writes nothing but needs dst != NULL).
 * Errors: KVP_ERR_NULL, KVP_ERR_BAD_SHAPE, KVP_ERR_HIP (kvp_last_error is not set). */
int kvp_probe_mfma(float* sink, int32_t iters, double* flops_out, void* hip_stream);
int kvp_probe_stream(int32_t kind, const void* src, void* dst, size_t bytes, void* hip_stream);

/* Per-kernel-class timers.  While enabled, one HIP event is recorded on the caller's stream after
 * every launch (a decode-attention split + merge pair counts as one); the time between consecutive
 * events is charged to the class of the later launch (this perturbs end-to-end time a little: use
 * a separate pass).  kvp_profile_read synchronises on the recorded events and returns, per class,
 * the summed device milliseconds and launch count since the last kvp_profile_reset.
 * ms, launches: host arrays [KVP_KC_COUNT]. */
int kvp_profile_enable(kvp_handle* h, int32_t on);
int kvp_profile_reset(kvp_handle* h);
int kvp_profile_read(kvp_handle* h, double* ms, int64_t* launches);

/* Releases the handle: host metadata, the internal stream and events, profiling events, and the
 * device tables kvp_load_weights allocated (rotary tables, flag word, predictor pointer tables).
 * Synchronises the internal stream first.  NULL is allowed. */
void kvp_free(kvp_handle* h);

/* Message of the last error on this thread ("" if none); storage is thread-local and static. */
const char* kvp_last_error(void);

/* Library version string. */
const char* kvp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVP_H */
