/*
 * po.h -- C ABI of libpo: single-output-token ("prefill-only") transformer inference on
 * one AMD MI355X (gfx950).
 *
 * The operation (paper Sections 1, 2.2, 4): a request is a token sequence plus a short
 * list of acceptable output tokens; the engine runs ONLY the prefill phase, in one
 * forward pass, and returns the next-token distribution at the last position, either
 * as logits over the vocabulary or as log-probabilities restricted to the acceptable
 * tokens (whose probabilities sum to 1).  Because nothing is decoded, only the K/V of
 * the layer currently being computed is kept (abstract, Section 1); the position-wise
 * layers run chunk by chunk over tokens so their intermediates stay small while
 * attention runs over the whole sequence in one call ("hybrid prefilling", Section 4.2);
 * chunk outputs are written straight into preallocated buffers and same-shape outputs
 * overwrite their inputs (Section 4.3).  Requests run one at a time (Section 6.1).
 *
 * Model: a Llama-style pre-norm decoder (RMSNorm, rotary embedding with the rotate-half
 * pairing (i, i + head_dim/2) and angle pos * theta^(-2i/head_dim), causal grouped-query
 * attention with query head h reading KV head h / (n_q_heads / n_kv_heads), SwiGLU MLP,
 * untied LM head, optional QKV bias).  Position of token i is i.
 *
 * Conventions
 *   - every call returns a po_status; nothing is written to outputs on error.
 *   - pointers are HOST pointers unless the name starts with dev_.
 *   - the caller owns every buffer it passes, including the two device arenas
 *     (dev_weights, dev_workspace) which must stay alive and untouched by others for
 *     the life of the context; the library owns only the po_ctx.
 *   - all device work of a context is issued on the HIP stream given to po_create;
 *     po_prefill returns after that stream has been synchronised.
 *   - a context is not re-entrant: one call at a time per context.
 *   - weights are given in the checkpoint layout [out_features, in_features], row-major,
 *     in the model's storage dtype (float for PO_F32; bf16 bit patterns for PO_BF16).
 */
#ifndef PO_H_
#define PO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PO_OK = 0,
    PO_ERR_INVALID_ARG = 1,        /* NULL pointer, non-positive size, bad enum value      */
    PO_ERR_BAD_CONFIG = 2,         /* model shape the kernels do not support               */
    PO_ERR_NOT_LOADED = 3,         /* po_prefill before every tensor was loaded            */
    PO_ERR_TOO_LONG = 4,           /* len > max_input_len given to po_create               */
    PO_ERR_TOKEN_RANGE = 5,        /* a token or candidate id outside [0, vocab_size)      */
    PO_ERR_WORKSPACE_TOO_SMALL = 6,/* an arena smaller than po_workspace_bytes reports     */
    PO_ERR_OOM = 7,                /* host allocation failed                               */
    PO_ERR_DEVICE = 8              /* a HIP call failed (message via po_last_device_error) */
} po_status;

/* PO_BF16_FP8: a bf16 model (weights are given, and activations stored, as bf16) whose decoder-block
 * linear layers (Q/K/V, O, gate/up, down) run FP8-dynamic: weights quantised to E4M3 per output channel
 * when they are loaded, their input activations per token when they are used (see po_op_quantize_rows);
 * embedding, norms, rotary embedding, attention and the LM head stay bf16. */
typedef enum { PO_F32 = 0, PO_BF16 = 1, PO_BF16_FP8 = 2 } po_dtype;

/* Tensor kinds for po_load_tensor.  Per-layer kinds take layer in [0, n_layers);
 * global kinds (EMBED, FINAL_NORM, LM_HEAD) take layer = -1. */
typedef enum {
    PO_T_EMBED = 0,       /* [vocab, d_model]                    */
    PO_T_ATTN_NORM = 1,   /* [d_model]   gain of the norm before attention */
    PO_T_WQ = 2,          /* [n_q_heads*head_dim, d_model]       */
    PO_T_WK = 3,          /* [n_kv_heads*head_dim, d_model]      */
    PO_T_WV = 4,          /* [n_kv_heads*head_dim, d_model]      */
    PO_T_BQ = 5,          /* [n_q_heads*head_dim]   (qkv_bias=1) */
    PO_T_BK = 6,          /* [n_kv_heads*head_dim]  (qkv_bias=1) */
    PO_T_BV = 7,          /* [n_kv_heads*head_dim]  (qkv_bias=1) */
    PO_T_WO = 8,          /* [d_model, n_q_heads*head_dim]       */
    PO_T_MLP_NORM = 9,    /* [d_model]   gain of the norm before the MLP */
    PO_T_WG = 10,         /* [ffn_dim, d_model]   gate projection */
    PO_T_WU = 11,         /* [ffn_dim, d_model]   up projection   */
    PO_T_WD = 12,         /* [d_model, ffn_dim]   down projection */
    PO_T_FINAL_NORM = 13, /* [d_model]                            */
    PO_T_LM_HEAD = 14,    /* [vocab, d_model]                     */
    PO_T_COUNT = 15
} po_tensor_kind;

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab_size;
    float rms_eps, rope_theta;
    int32_t dtype;     /* po_dtype: storage and activation type; accumulation is fp32 */
    int32_t qkv_bias;  /* 0 | 1 */
} po_model_config;

/* Kernel classes whose time po_get_stats splits out when phase timing is on. */
typedef enum {
    PO_K_ATTENTION = 0,   /* causal GQA attention, one launch per layer                     */
    PO_K_QKV = 1,         /* QKV projection (+ rotary embedding, transposed V)              */
    PO_K_RESIDUAL = 2,    /* O-projection and MLP down projection (+ residual add)          */
    PO_K_GATE_UP = 3,     /* MLP gate/up projection (+ SiLU-multiply)                       */
    PO_K_COUNT = 4
} po_kernel_class;

typedef struct {
    double last_prefill_ms;               /* device time of the last po_prefill (HIP events on its stream) */
    double kernel_ms[PO_K_COUNT];         /* ... of which each kernel class (0 unless phase timing is on)  */
    int64_t kernel_launches[PO_K_COUNT];  /* launches of each class in the last po_prefill                 */
    uint64_t weights_bytes;               /* size of the weight arena in use                               */
    uint64_t workspace_bytes;             /* size of the activation arena in use (peak; static)            */
    int64_t last_len;                     /* tokens in the last request                                    */
    int64_t split_launches;               /* GEMM / attention launches of the last request that ran split
                                             (po_set_few_rows_split); 0 on the default path               */
} po_stats;

typedef struct po_ctx po_ctx;

/* Sizes of the two device arenas for a model, a maximum input length and a chunk size
 * (Section 3: the user declares the maximum input length up front and memory is sized
 * from it).  Closed form; needs no GPU.  workspace = residual stream + Q/O + ONE layer
 * of K/V + one chunk of position-wise intermediates + rotary table + logits. */
po_status po_workspace_bytes(const po_model_config* cfg, int64_t max_input_len, int32_t mlp_chunk,
                             size_t* weights_bytes, size_t* workspace_bytes);

/* Largest maximum input length whose two arenas fit in hbm_budget_bytes (the quantity the
 * paper's evaluation calls maximum input length, Section 7.2 / its MIL table): the largest
 * N with weights_bytes + workspace_bytes(N) <= budget, found by bisection on the closed
 * form above; needs no GPU.  PO_ERR_OOM if not even one token fits; *max_len is capped at
 * the longest sequence the kernels address (2^24 tokens, or less for wide KV rows). */
po_status po_max_input_len(const po_model_config* cfg, int32_t mlp_chunk, size_t hbm_budget_bytes,
                           int64_t* max_len);

/* Creates a context over caller-provided device memory (256-byte aligned) and a HIP
 * stream (hipStream_t passed as void*; NULL = the default stream).  mlp_chunk is the
 * number of tokens per chunk of the position-wise layers (Section 4.2), >= 1. */
po_status po_create(const po_model_config* cfg, int64_t max_input_len, int32_t mlp_chunk,
                    void* dev_weights, size_t weights_bytes,
                    void* dev_workspace, size_t workspace_bytes,
                    void* hip_stream, po_ctx** out);

/* Copies one tensor from host memory into the weight arena (re-laid out for the
 * kernels).  bytes must equal the tensor's size in the model dtype.  Synchronous. */
po_status po_load_tensor(po_ctx* ctx, int32_t tensor_kind, int32_t layer,
                         const void* host_data, size_t bytes);

/* A whole model in host memory: tensor[kind] points at the tensor of a global kind
 * (PO_T_EMBED, PO_T_FINAL_NORM, PO_T_LM_HEAD), or at an array of n_layers pointers, one per
 * layer, for a per-layer kind (the three bias kinds may be NULL when qkv_bias == 0).  Every
 * tensor has the size and layout po_load_tensor expects. */
typedef struct {
    const void* tensor[PO_T_COUNT];
} po_host_weights;

/* po_load_tensor for every tensor of the model.  Stops at the first error; tensors loaded
 * before it stay loaded. */
po_status po_load_weights(po_ctx* ctx, const po_host_weights* weights);

/* 1 when every tensor the configuration needs has been loaded, else 0. */
int32_t po_is_loaded(const po_ctx* ctx);

/* One prefill-only request.  tokens[len] int32 in [0, vocab); cand_ids[n_cand] are the
 * acceptable tokens (may be NULL/0).  out_logits (fp32 [vocab]) and out_cand_logprobs
 * (fp32 [n_cand], log-softmax restricted to the candidates) may each be NULL.  Ranges
 * are validated on the host before any launch. */
po_status po_prefill(po_ctx* ctx, const int32_t* tokens, int64_t len,
                     const int32_t* cand_ids, int32_t n_cand,
                     float* out_logits, float* out_cand_logprobs);

/* n_req independent requests run one after another (Section 6.1: no batching);
 * tokens_concat holds them back to back, lens[n_req] their lengths.  Outputs are
 * [n_req, vocab] and [n_req, n_cand].  Bit-identical to n_req po_prefill calls. */
po_status po_prefill_batch(po_ctx* ctx, const int32_t* tokens_concat, const int64_t* lens,
                           int32_t n_req, const int32_t* cand_ids, int32_t n_cand,
                           float* out_logits, float* out_cand_logprobs);

/* The same n_req requests with their tokens packed into one buffer for the position-wise
 * layers.  A variant beside the paper's design: Section 6.1 runs requests one at a time
 * because a long prefill already saturates the GPU; short requests do not fill whole
 * rounds of GEMM tiles, so here consecutive requests are laid one after the other (each
 * starting on a multiple of 64 rows, as many as max_input_len rows hold), norms and linear
 * layers run over all their rows at once, attention runs per request, every request
 * restarts at position 0, and each request's last row goes through the final norm and LM
 * head.  Same arguments, outputs and validation as po_prefill_batch, and bit-identical
 * results: no kernel's result for a row depends on which other rows share its launch. */
po_status po_prefill_packed(po_ctx* ctx, const int32_t* tokens_concat, const int64_t* lens,
                            int32_t n_req, const int32_t* cand_ids, int32_t n_cand,
                            float* out_logits, float* out_cand_logprobs);

/* Profile run (Section 3: at start-up the engine forwards a fake request of the declared
 * maximum input length and sizes what is left of the GPU from it).  Fills the activation
 * arena with a byte pattern, runs one request of `len` copies of token 0 (len <= the
 * context's max_input_len; weights must be loaded), and reports the device time of that
 * request and the measured high-water mark of the arena: the offset one past the highest
 * byte the run changed.  The footprint is static, so the mark must come out as the closed
 * form of po_workspace_bytes for the context's max_input_len, less the unused tail of the
 * candidate buffers at the arena's end (sized for the largest candidate list; the fake
 * request uses two); that is what this call lets a caller check.  Synchronous; overwrites
 * the arena (the rotary table, the only content that outlives a request, is rebuilt). */
po_status po_profile(po_ctx* ctx, int64_t len, double* elapsed_ms, size_t* touched_bytes);

/* Prefix K/V cache (Section 5.1, suffix KV cache discarding: the K/V of a request's prefix
 * tokens is kept on the GPU for later requests that share the prefix, the K/V of its suffix
 * is discarded with each layer as before).  The cache is caller-provided device memory
 * (256-byte aligned) of po_kv_cache_bytes(cfg, prefix_capacity) bytes: per layer the K rows
 * and the V rows (stored transposed for bf16) of up to prefix_capacity positions, i.e.
 * 2 * n_layers * n_kv_heads * head_dim elements per position.  dev_cache = NULL detaches. */
po_status po_kv_cache_bytes(const po_model_config* cfg, int64_t prefix_capacity, size_t* bytes);
po_status po_attach_kv_cache(po_ctx* ctx, void* dev_cache, size_t bytes, int64_t prefix_capacity);

/* The same with n_slots entries of prefix_capacity positions each (bytes >= n_slots times
 * what po_kv_cache_bytes reports).  A request reuses the entry with which it shares the
 * longest prefix.  The prefix it asks to keep: if that entry already contains it, nothing
 * is stored and the entry stays as long as it is; if the request shares everything the
 * entry holds, or at least half of it, the entry is cut to the shared part and grows in
 * place (requests that differ only in their tails keep one entry and rewrite the tail);
 * otherwise (a hit on less than half of the entry, or none) the prefix replaces an empty or
 * else the least recently used of the OTHER entries, so that a short partial hit does not
 * destroy a long entry (with one entry it replaces that one).  "Used" = reused by a request
 * or written. */
po_status po_attach_kv_cache_slots(po_ctx* ctx, void* dev_cache, size_t bytes, int64_t prefix_capacity,
                                   int32_t n_slots);

/* What the cache would spare a request: the longest common prefix of tokens[0 .. len) with
 * any entry, at most len - 1 (0 without a cache).  Host only. */
po_status po_kv_cache_match(const po_ctx* ctx, const int32_t* tokens, int64_t len, int64_t* cached_len);

/* The token ids whose K/V entry `slot` holds: *n_tokens receives their number, tokens_out
 * (may be NULL; capacity >= *n_tokens otherwise) the ids.  Host only. */
po_status po_kv_cache_slot(const po_ctx* ctx, int32_t slot, int32_t* tokens_out, int64_t capacity,
                           int64_t* n_tokens);

/* po_prefill with the prefix cache.  The longest common prefix of tokens[] with the tokens
 * whose K/V the cache holds (at most len - 1 positions) is NOT recomputed: embedding,
 * projections and MLP run on the remaining positions only, and attention reads the cached
 * K/V of the prefix next to the fresh K/V of the rest (rectangular block for the prefix keys,
 * causal block for the rest).  *reused_prefix_len (may be NULL) reports that length.
 * keep_prefix > 0: afterwards some entry of the cache holds the K/V of tokens[0 .. keep_prefix)
 * (see po_attach_kv_cache_slots for which; keep_prefix <= len and <= prefix_capacity, else PO_ERR_TOO_LONG);
 * keep_prefix = 0 leaves the cache as it is; keep_prefix = PO_KEEP_ALL keeps as much of the
 * request as an entry holds, min(len, prefix_capacity).  The outputs are bit-identical to po_prefill
 * on the same tokens (a row's result does not depend on which other rows are computed; in
 * few-rows mode, see po_set_few_rows_split, equal within tolerance instead).
 * PO_ERR_INVALID_ARG without an attached cache. */
#define PO_KEEP_ALL (-1)
po_status po_prefill_prefix(po_ctx* ctx, const int32_t* tokens, int64_t len, int64_t keep_prefix,
                            const int32_t* cand_ids, int32_t n_cand,
                            float* out_logits, float* out_cand_logprobs, int64_t* reused_prefix_len);

/* Profiles how the job completion time varies with (n_input, n_cached) (Section 6.3: pairs that
 * cover the maximum input length at a granularity of `step` tokens, 1000 in the paper; the
 * scheduler's linear model is fitted on them, see po_sched_fit_jct_model).  Runs one fake request
 * of pseudo-random token ids for every n_input in {step, 2 step, ..., max_len} and every
 * n_cached in {0, step, ...} below n_input and within the cache's capacity, through the same
 * path as po_prefill_prefix with that many positions reused, and reports the device time of
 * each in milliseconds.  *n_samples receives the number of pairs; with all three output arrays
 * NULL nothing runs (size query), otherwise capacity must be at least that number.  Needs an
 * attached cache (PO_ERR_INVALID_ARG without) and loaded weights; max_len <= the context's.
 * Synchronous; afterwards the cache is empty. */
po_status po_profile_jct(po_ctx* ctx, int64_t max_len, int64_t step, int64_t* n_input_out,
                         int64_t* n_cached_out, double* jct_ms_out, int32_t capacity, int32_t* n_samples);

/* Request scheduling on the host (Section 6.3, Algorithm 1: shortest-remaining-job-first with
 * continuous JCT calibration).  The scheduler keeps the waiting requests (copies of their
 * tokens); every pick recomputes, for each of them, n_cached = the length of its common
 * prefix with the tokens the prefix cache holds at that moment (at most len - 1) and
 * score = jct(n_input, n_cached) - lambda * (now - arrival_time), and returns the request
 * with the lowest score (the earliest pushed on ties), removing it from the queue.
 * jct is the paper's default proxy n_input - n_cached, or, once set or fitted, the linear
 * model c0 + c_input * n_input + c_cached * n_cached (the paper fits it by linear regression
 * on profiled (n_input, n_cached) pairs; coef[3] receives c0, c_input, c_cached, may be NULL;
 * at least 3 non-collinear samples).  lambda (>= 0; the paper uses 500 with JCT in tokens
 * and time in seconds) trades average for worst-case latency.  po_sched_pick on an empty
 * queue returns PO_OK with *id = -1.  No GPU is involved. */
typedef struct po_sched po_sched;
po_status po_sched_create(double lambda, po_sched** out);
void po_sched_destroy(po_sched* s);
po_status po_sched_set_jct_model(po_sched* s, double c0, double c_input, double c_cached);
po_status po_sched_fit_jct_model(po_sched* s, const int64_t* n_input, const int64_t* n_cached,
                                 const double* jct, int32_t n, double coef[3]);
po_status po_sched_push(po_sched* s, int64_t id, const int32_t* tokens, int64_t len, double arrival_time);
/* The same with the request's own acceptable output tokens (a request is a token sequence plus that
 * list, Section 2.2); po_engine_step uses them when it is given none. */
po_status po_sched_push_request(po_sched* s, int64_t id, const int32_t* tokens, int64_t len, const int32_t* cand_ids,
                                int32_t n_cand, double arrival_time);
int64_t po_sched_size(const po_sched* s);
/* Takes the request with this id out of the queue without running it (PO_ERR_INVALID_ARG if there is none). */
po_status po_sched_remove(po_sched* s, int64_t id);
po_status po_sched_pick(po_sched* s, const int32_t* cached_tokens, int64_t n_cached_tokens, double now,
                        int64_t* id, int64_t* n_cached_hit);
/* The same against a cache of several entries: n_cached of a request is the best any entry
 * offers it (cached_tokens[e] / n_cached_tokens[e], e < n_entries). */
po_status po_sched_pick_multi(po_sched* s, const int32_t* const* cached_tokens, const int64_t* n_cached_tokens,
                              int32_t n_entries, double now, int64_t* id, int64_t* n_cached_hit);

/* One step of the serving loop (Section 3: the scheduler hands the executor one request per
 * step; Section 6.3: which one).  Scores every waiting request of `s` as po_sched_pick does,
 * n_cached being what ctx's prefix cache would spare it at this moment (po_kv_cache_match; 0
 * without a cache), removes the one with the lowest score from the queue and runs it: with a
 * cache attached through po_prefill_prefix with keep_prefix = PO_KEEP_ALL, otherwise through
 * po_prefill.  The acceptable output tokens are cand_ids[0 .. n_cand) for whichever request
 * runs, or, with cand_ids = NULL, the list the request was pushed with (po_sched_push_request;
 * possibly none).  out_cand_logprobs (may be NULL) holds cand_capacity floats; a longer list is
 * PO_ERR_INVALID_ARG and leaves the queue as it is.  *n_cand_used (may be NULL) receives the
 * number of log-probs written.  Other outputs as in po_prefill; *id receives the request's id
 * (-1, and nothing runs, when the queue is empty), *len and *reused_prefix_len (both may be
 * NULL) its length and the positions it did not compute.  A request leaves the queue only once it
 * has run: if the context refuses it (PO_ERR_TOO_LONG, PO_ERR_TOKEN_RANGE, ...) or its run fails, the
 * error is returned with *id set and the request is still queued; drop it with po_sched_remove, or the
 * next step picks it again. */
po_status po_engine_step(po_ctx* ctx, po_sched* s, double now, const int32_t* cand_ids, int32_t n_cand,
                         float* out_logits, float* out_cand_logprobs, int32_t cand_capacity, int64_t* id,
                         int64_t* len, int64_t* reused_prefix_len, int32_t* n_cand_used);

/* Last-layer shortcut, on by default.  A prefill-only request produces one token (Section 1),
 * so nothing reads the last layer's output except at the last position: with the shortcut
 * the last layer still forms K and V for every position, but runs attention only for the
 * row block that holds the last position and the O-projection and MLP only for that row.
 * Logits and log-probs are bit-identical with the shortcut on and off. */
po_status po_set_lazy_last_layer(po_ctx* ctx, int32_t on);

/* Few-rows mode, off by default (bf16 and FP8-dynamic contexts; fp32 ignores it).  A request that computes few
 * positions -- a short one, or the suffix behind a long cached prefix, the paper's post
 * recommendation case (Sections 2.2, 5.1) -- gives the QKV, O- and MLP down projections too
 * few output tiles, and attention too few query tiles, to occupy the chip.  With the mode on,
 * launches of those GEMMs whose tiles would fill at most half the compute units split their
 * reduction over K between workgroups, and attention over at most 1024 query rows splits each
 * query tile's keys between workgroups (fp32 partial results in the free part of the chunk
 * buffer, merged in a fixed order by a second kernel: deterministic; the footprint
 * po_workspace_bytes reports is unchanged).  A split sum is rounded differently
 * from the single running sum of the default path: results stay within the library's
 * tolerance against the definition but are no longer bit-identical to the default path's,
 * nor between a request run alone and the same rows computed as part of a larger chunk. */
po_status po_set_few_rows_split(po_ctx* ctx, int32_t on);

/* Float32 contexts only (PO_ERR_BAD_CONFIG otherwise); off by default.  When on, every tensor the forward pass keeps
 * between two operators -- both normalised activations, the rotated Q and K, V, the attention output, the gated MLP
 * intermediate, the residual stream after each update, the normalised last row -- is rounded to the nearest bf16 value
 * (ties to even) as soon as it is written; arithmetic inside an operator and the logits stay float32.  This is what a
 * bf16 model's storage does to the definition's result with no other source of error, measured by comparing a run
 * with the mode on against one with it off: the yardstick for the bf16 path at configurations too large for a
 * float64 CPU run (Section 4.2 of the paper claims only that chunking changes nothing; storage precision is the
 * model's own).  Host call, takes effect from the next request. */
po_status po_set_storage_rounding(po_ctx* ctx, int32_t on);

/* When on, po_prefill brackets the attention and GEMM launches with HIP events on its stream
 * so that po_get_stats can split the time per kernel class (adds event overhead; off by
 * default). */
po_status po_set_phase_timing(po_ctx* ctx, int32_t on);

po_status po_get_stats(const po_ctx* ctx, po_stats* out);

void po_destroy(po_ctx* ctx);

const char* po_strerror(po_status s);

/* Text of the last HIP error seen by this thread ("" if none). */
const char* po_last_device_error(void);

/* ------------------------------------------------------------------------------------
 * Single-kernel entry points.  Each runs ONE step of the path on DEVICE buffers the
 * caller owns, asynchronously on `hip_stream`, so a step can be checked against its
 * definition and timed at the exact shapes the full path uses.  dtype is a po_dtype
 * (activation and weight storage; all reductions accumulate in fp32).
 * ---------------------------------------------------------------------------------- */

/* y[r, :] = x[r, :] * rsqrt(mean(x[r,:]^2) + eps) * g   (rows x d). */
po_status po_op_rmsnorm(int32_t dtype, const void* dev_x, const void* dev_g, void* dev_y,
                        int64_t rows, int32_t d, float eps, void* hip_stream);

/* Position-wise linear layer of Section 4: C[M, N] = A[M, K] * W[N, K]^T (+ residual).
 * dev_residual may be NULL, or a [M, N] tensor added before the store (may alias dev_c). */
po_status po_op_linear(int32_t dtype, const void* dev_a, const void* dev_w, void* dev_c,
                       const void* dev_residual, int64_t M, int32_t N, int32_t K, void* hip_stream);
/* The few-rows form of po_op_linear with a residual (bf16 only; see po_set_few_rows_split): C = A W^T + R with
 * the reduction over K split between workgroups, fp32 partial sums in dev_scratch (scratch_bytes; 256-byte
 * aligned).  *splits_used receives the number of splits; 0 or 1 means the shape is not worth splitting or the
 * scratch is too small, and then NOTHING was computed. */
po_status po_op_linear_split(const void* dev_a, const void* dev_w, void* dev_c, const void* dev_residual,
                             void* dev_scratch, size_t scratch_bytes, int64_t M, int32_t N, int32_t K,
                             void* stream, int32_t* splits_used);

/* Gate/up projection with the SiLU-multiply of the MLP (Section 4.1's MLP figure):
 * H[M, F] = silu(A Wg^T) * (A Wu^T); dev_wgu is [2F, K] in the library's interleaved
 * order (see po_op_pack_gate_up); dev_scratch must hold M*2F elements for PO_F32 and may
 * be NULL for PO_BF16. */
po_status po_op_gate_up_silu(int32_t dtype, const void* dev_a, const void* dev_wgu, void* dev_h,
                             void* dev_scratch, int64_t M, int32_t F, int32_t K, void* hip_stream);

/* Packs Wg [F, K] and Wu [F, K] (device) into the interleaved [2F, K] order the gate/up
 * kernel reads. */
po_status po_op_pack_gate_up(int32_t dtype, const void* dev_wg, const void* dev_wu, void* dev_wgu,
                             int32_t F, int32_t K, void* hip_stream);

/* Causal grouped-query attention over one whole sequence (Section 4.2: attention is not
 * chunked).  q [N, Hq, hd] (already rotated), k [N, Hkv, hd] (rotated), v [N, Hkv, hd];
 * o [N, Hq, hd] may alias q.  dev_scratch (256-byte aligned): PO_BF16 needs
 * round_up(2*Hkv*hd*round_up(N,64), 256) + 4*Hq*ceil(N/256) bytes (a transposed copy of V, then one word
 * per 256-row query tile and head in which the kernel marks tiles whose scores outgrow its fixed reference
 * exponent; those are recomputed with a running maximum, so the result is softmax for every finite input);
 * PO_F32 needs none (NULL).
 * q_prescaled (0 | 1; PO_BF16 only): 1 = dev_q holds the queries times log2(e) / sqrt(head_dim), which is how the
 * full path hands them over (po_op_qkv_rope's q_scale applies the factor in fp32 before Q's one rounding): the
 * kernel then exponentiates K Q^T as it comes out of the matrix pipe, with no multiply-add per score and no
 * reference exponent; rows whose probabilities would leave the float range that way (scores beyond about +-60
 * nats as a whole row) are recomputed with a running maximum, like overflowing ones with q_prescaled = 0. */
po_status po_op_attention(int32_t dtype, const void* dev_q, const void* dev_k, const void* dev_v,
                          void* dev_o, void* dev_scratch, int64_t N, int32_t n_q_heads,
                          int32_t n_kv_heads, int32_t head_dim, int32_t q_prescaled, void* hip_stream);
/* The few-rows form of po_op_attention (bf16 only; see po_set_few_rows_split): rows [q_row0, N) of the causal
 * attention, each query tile's keys divided between workgroups and merged by a second kernel.  dev_scratch_vt as
 * dev_scratch there; dev_scratch_part (part_bytes, 256-byte aligned) takes the fp32 partial results.  Rows below
 * q_row0 of dev_o are left as they are.  *splits_used receives the number of key splits; 0 or 1 means too few keys
 * or rows too many (> 1024) or the scratch too small, and then NOTHING was computed. */
po_status po_op_attention_split(const void* dev_q, const void* dev_k, const void* dev_v, void* dev_o,
                                void* dev_scratch_vt, void* dev_scratch_part, size_t part_bytes, int64_t N,
                                int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int64_t q_row0,
                                void* hip_stream, int32_t* splits_used);

/* Rotary embedding in place on x [N, H, hd] for positions 0..N-1 (angles formed in
 * double precision). */
po_status po_op_rope(int32_t dtype, void* dev_x, int64_t N, int32_t n_heads, int32_t head_dim,
                     float theta, void* hip_stream);

/* po_op_rope for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same arithmetic and bit-identical results, but the
 * rotary table lives in a device array inside the library (8 MiB per GPU, held until the process ends) instead
 * of a buffer allocated and freed per call, and the call does not synchronise: it is asynchronous on
 * hip_stream.  N * head_dim * 4 bytes of table must fit: N * head_dim <= 2 097 152 (e.g. 16 384 positions of
 * head_dim 128), else PO_ERR_WORKSPACE_TOO_SMALL and nothing is launched.  The table is rewritten in full by
 * every call before it is read.  All calls on one GPU share that GPU's array: calls that overlap on one GPU
 * (different streams, different threads) race; calls on different GPUs do not. */
po_status po_op_rope_static(int32_t dtype, void* dev_x, int64_t N, int32_t n_heads, int32_t head_dim,
                            float theta, void* hip_stream);

/* cos/sin tables, fp32 [n, head_dim/2] each, of pos * theta^(-2i/head_dim) for positions
 * 0..n-1 (angles formed in double precision). */
po_status po_op_rope_table(float* dev_cos, float* dev_sin, int64_t n, int32_t head_dim, float theta,
                           void* hip_stream);

/* PO_BF16 only.  Builds the packed QKV weight [(Hq+2Hkv)*hd, K] (and bias, if the three bias
 * pointers are given) the fused projection reads, from Wq [Hq*hd, K], Wk, Wv [Hkv*hd, K]:
 * rows are concatenated and, inside every Q and K head, reordered so that the two halves of
 * a rotary pair land in one accumulator lane. */
po_status po_op_pack_qkv(const void* dev_wq, const void* dev_wk, const void* dev_wv, void* dev_wqkv,
                         const void* dev_bq, const void* dev_bk, const void* dev_bv, void* dev_bqkv,
                         int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t K, void* hip_stream);

/* PO_BF16 only.  The fused step before attention for M consecutive tokens starting at
 * sequence position pos0: [Q|K|V] = A Wqkv^T (+bias), rotary embedding applied to Q and K in
 * fp32 before rounding; q [M, Hq*hd] and k [M, Hkv*hd] are written row-major, V is written
 * transposed into columns pos0..pos0+M-1 of vt [Hkv*hd][ldv] (the layout the attention
 * kernel reads).  dev_bqkv may be NULL.  q_scale (> 0): factor on the rotated Q values, applied in fp32 before
 * they are rounded; 1 gives the rotated queries themselves, log2(e) / sqrt(head_dim) what po_op_attention
 * expects with q_prescaled = 1 (the full path's choice).  K and V are never scaled. */
po_status po_op_qkv_rope(const void* dev_a, const void* dev_wqkv, const void* dev_bqkv, void* dev_q, void* dev_k,
                         void* dev_vt, int64_t ldv, const float* dev_cos, const float* dev_sin, int64_t pos0,
                         int64_t M, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t K,
                         float q_scale, void* hip_stream);

/* ---- FP8-dynamic variant of the decoder's linear layers (Section 7.1 names FP8-dynamic
 * checkpoints; the scheme is the public convention: OCP E4M3 codes, one float32 scale per
 * output channel of a weight and per token of an activation).  A bf16 row x with
 * amax = max|x_k| becomes codes e4m3(x_k * (448 / amax)), round to nearest even, and the
 * scale amax / 448 (amax == 0: codes 0, scale 1); single float32 operations throughout, so
 * codes and scales are reproducible bit for bit. */

/* codes [M, K] (one byte each) and scales [M] of the bf16 rows x [M, K].  K % 8 == 0,
 * K <= 28672.  dev_codes may be dev_x itself (a row's codes then occupy the first half of
 * the row). */
po_status po_op_quantize_rows(const void* dev_x, void* dev_codes, float* dev_scales, int64_t M, int32_t K,
                              void* hip_stream);

/* The same of bf16(rmsnorm(x; g)), the normalised row formed exactly as po_op_rmsnorm
 * forms it (d % 8 == 0, d <= 8192). */
po_status po_op_rmsnorm_quantize(const void* dev_x, const void* dev_g, void* dev_codes, float* dev_scales,
                                 int64_t rows, int32_t d, float eps, void* hip_stream);

/* C = (Qa Qw^T) * sa[row] * sw[col], products accumulated in fp32, result bf16.
 * epilogue 0: C [M, N]; 1: C = ... + residual [M, N] (added in fp32, may alias C);
 * 2: Qw rows in the interleaved gate/up order of po_op_pack_gate_up (and dev_w_scales in the
 * same order), C [M, N/2] = silu(gate) * up.  K % 128 == 0, N % 64 == 0. */
po_status po_op_linear_fp8(int32_t epilogue, const void* dev_a_codes, const float* dev_a_scales,
                           const void* dev_w_codes, const float* dev_w_scales, void* dev_c,
                           const void* dev_residual, int64_t M, int32_t N, int32_t K, void* hip_stream);

/* po_op_qkv_rope with FP8 operands: dev_w_codes / dev_w_scales hold the packed QKV weight rows
 * (the order po_op_pack_qkv produces), dev_bqkv (bf16, packed order) may be NULL. */
po_status po_op_qkv_rope_fp8(const void* dev_a_codes, const float* dev_a_scales, const void* dev_w_codes,
                             const float* dev_w_scales, const void* dev_bqkv, void* dev_q, void* dev_k, void* dev_vt,
                             int64_t ldv, const float* dev_cos, const float* dev_sin, int64_t pos0, int64_t M,
                             int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t K, float q_scale,
                             void* hip_stream);

/* ---- Micro-peaks of the machine, for the benchmark to report beside the nominal peaks (measurement only; the
 * paper's claim that the workload is compute-bound, Section 2.3, is priced against what the board sustains).
 * po_op_mfma_peak: every wavefront of a chip-filling grid (1024 workgroups of 256 * waves_per_simd threads)
 * multiplies one pair of bf16 fragments, read once from dev_operands (32 bytes per thread: operand_bytes >=
 * 1024 * 256 * waves_per_simd * 32; give it random data, the clock under matrix load depends on the operands),
 * `iters` times into independent accumulators with kind 0: v_mfma_f32_32x32x16_bf16, 1: v_mfma_f32_16x16x32_bf16;
 * nothing but the matrix pipe works inside the loop.  *flop receives the flop executed; dev_sink is one float
 * (never written in practice).  Asynchronous on hip_stream; time it with events.
 * po_op_stream_copy: dev_dst[0 .. bytes) = dev_src[0 .. bytes), 16 bytes per lane, bytes % 16 == 0. */
po_status po_op_mfma_peak(int32_t kind, int32_t waves_per_simd, int32_t iters, const void* dev_operands,
                          size_t operand_bytes, void* dev_sink, void* hip_stream, double* flop);
po_status po_op_stream_copy(const void* dev_src, void* dev_dst, size_t bytes, void* hip_stream);

/* Last-position LM head: logits[V] = x[d] . W[V, d]^T  (fp32 output). */
po_status po_op_lm_head(int32_t dtype, const void* dev_x, const void* dev_w, float* dev_logits,
                        int32_t V, int32_t d, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PO_H_ */
