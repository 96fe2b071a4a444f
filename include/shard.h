/*
 * libshard - forward pass of one EdgeShard shard on one MI355X (gfx950).
 *
 * A shard is a contiguous range [layer_lo, layer_hi) of a model's decoder layers placed on
 * one device; the device receives the previous range's output activations, runs its
 * layers over a KV cache it pre-allocated, and hands its own output activations on
 * (EdgeShard Sec. 3 "Collaborative inference"; Sec. 4 "System Model": layer i has an
 * activation size O_i and a memory need Req_i).  Inference has two phases: prefill
 * consumes the whole prompt at once, the autoregressive phase consumes one token per
 * iteration and reuses the cached keys/values (Sec. 2 "Generative LLM Inference").
 *
 * The layer is the Llama 2 decoder layer (the model family of Sec. 5.1): pre-norm
 * RMSNorm (eps inside the root, gain after), bias-free Q/K/V/O projections, rotary
 * position embedding on ADJACENT element pairs (2i, 2i+1) of every q/k head with angle
 * pos * theta^(-2i/head_dim), causal softmax attention scaled by 1/sqrt(head_dim) where
 * query head h reads KV head h / (n_heads / n_kv_heads), residual add, RMSNorm,
 * SwiGLU feed-forward silu(Wg h) * (Wu h) -> Wd, residual add.
 *
 * Conventions for every entry point
 *  - Return value: SHARD_OK or a negative SHARD_E_* code; shard_last_error() gives a
 *    thread-local human-readable message for the last failure on the calling thread.
 *    Nothing throws or aborts across this boundary.  Validation happens before any
 *    launch; a call that fails validation leaves the shard unchanged.
 *  - "device pointer" = memory of the current HIP device; "host pointer" = ordinary
 *    host memory.  The library never takes ownership of caller memory.
 *  - hip_stream is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *    enqueued on it and the call returns without waiting; the caller synchronises.
 *  - State: a call that fails - at validation or at a kernel launch - leaves the sequences'
 *    lengths and pages as they were before it.
 *  - Range of the 16-bit path (weight_dtype SHARD_BF16): activations fed to the matrix cores
 *    (the half copy of the residual stream, the SwiGLU output) and the KV cache are IEEE half,
 *    largest finite value 65504.  Every kernel that rounds such a value to half tests it; a
 *    value beyond the range (or a NaN) raises a sticky flag in host-visible memory, and from
 *    then on shard_prefill / shard_decode / shard_decode_static return SHARD_E_RANGE before
 *    they launch anything (the flag is seen once the offending kernel has run, so at the
 *    latest by the call after the caller's next synchronisation).  shard_overflow reads and
 *    optionally clears it.  The fp32 path has no such limit.
 *  - A shard handle is not thread-safe; use one thread per handle at a time.
 *  - Several streams: calls issued (from that one thread) on different streams may overlap on
 *    the device when they carry different sequences - micro-batches of a pipeline stage, for
 *    instance.  The shard keeps SHARD_MAX_STREAMS workspace sets (all of them large enough for
 *    a prefill of max_batch_tokens when such a set is below 256 MB, otherwise only one) and
 *    orders its own reuse of them with events, so any pattern of streams is safe; up to
 *    SHARD_MAX_STREAMS streams run without waiting for each other.  The caller orders calls that touch the SAME sequence
 *    (its decode after its prefill, step after step), as on a single stream.
 */
#ifndef SHARD_H
#define SHARD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct shard shard_t; /* opaque; created by shard_create, freed by shard_destroy */

enum {
    SHARD_OK = 0,
    SHARD_E_INVAL = -1,   /* bad argument or configuration */
    SHARD_E_NOMEM = -2,   /* device or host allocation failed */
    SHARD_E_KV_FULL = -3, /* sequence would exceed max_seq_len, or no free sequence slot */
    SHARD_E_STATE = -4,   /* unknown seq_id, decode on an empty sequence, duplicate seq_id */
    SHARD_E_HIP = -5,     /* a HIP runtime call failed */
    SHARD_E_RANGE = -6    /* a 16-bit activation or cache value left the range of IEEE half */
};

enum { SHARD_F32 = 0, SHARD_BF16 = 1 };

/* Largest number of sequences one shard_prefill / shard_decode call may carry. */
#define SHARD_MAX_BATCH 64
/* Workspace sets a shard keeps, i.e. streams whose shard_decode calls can overlap. */
#define SHARD_MAX_STREAMS 4

typedef struct {
    int32_t d_model;      /* width of the hidden state */
    int32_t n_heads;      /* query heads Hq */
    int32_t n_kv_heads;   /* key/value heads Hkv; must divide n_heads */
    int32_t head_dim;     /* dh: 32, 64 or 128 */
    int32_t ffn_dim;      /* SwiGLU inner width F */
    float rms_eps;
    float rope_theta;
    int32_t weight_dtype; /* dtype of the matrices handed to shard_create.
                             SHARD_F32: KV cache and all arithmetic fp32.
                             SHARD_BF16: the matrices are converted ONCE, at create, to IEEE half
                             (same 2 bytes per element; every bf16 value of magnitude 6.1e-5 ..
                             65504 converts exactly, smaller ones round onto half's subnormal grid,
                             absolute error <= 3e-8; a larger one makes shard_create fail with
                             SHARD_E_INVAL).  The RMSNorm gains are multiplied into the converted
                             wq/wk/wv/w_gate/w_up (W (g * x_hat) = (W diag g) x_hat; one more
                             rounding to half per weight, and the product must stay within
                             65504 too).  The KV cache and the activations fed to the matrix
                             cores are half as well (8x finer rounding than bf16); accumulation and
                             the residual stream are fp32. */
    int32_t act_dtype;    /* dtype of x_in / x_out at the boundary; only SHARD_F32 is supported:
                             the paper runs full precision, and an fp32 hand-off keeps shard
                             composition exact.  The residual stream inside is always fp32. */
} shard_model_cfg;

typedef struct {
    int32_t max_seqs;         /* sequences that can be live at once (>= 1) */
    int32_t max_seq_len;      /* tokens per sequence the cache can hold (>= 1) */
    int32_t page_size;        /* tokens per KV page (>= 1; 16 is the tuned value);
                                 max_seq_len * page_size must be below 2^32 */
    int32_t max_batch_tokens; /* largest B*T of one shard_prefill call; 0 = max_seq_len */
} shard_kv_cfg;

/* One layer's parameters.  Matrices are [out, in] row-major in weight_dtype (bf16 as raw
 * 16-bit patterns): wq [Hq*dh, d], wk/wv [Hkv*dh, d], wo [d, Hq*dh], w_gate/w_up [F, d],
 * w_down [d, F].  Gains g_attn, g_ffn are float32 [d]. */
typedef struct {
    const void *wq, *wk, *wv, *wo, *w_gate, *w_up, *w_down;
    const float *g_attn, *g_ffn;
} shard_layer_weights;

/* What offline profiling records per layer (Sec. 3 "Profiling": execution time of each
 * layer for the prefill and the autoregressive stage and their average; activation size;
 * memory consumption).  Times are seconds per call of that layer. */
typedef struct {
    double t_prefill_s;         /* mean time of the layer in a prefill of (B, T_prefill) */
    double t_decode_s;          /* mean time of the layer in one decode step at batch B */
    double t_avg_s;             /* mean time per generated token over 1 prefill + n_decode steps:
                                   (t_prefill_s + n_decode * t_decode_s) / (1 + n_decode) */
    uint64_t act_bytes_prefill; /* O_i for the profiled prefill: B * T_prefill * d * 4 */
    uint64_t act_bytes_decode;  /* O_i for one decode step: B * d * 4 */
    uint64_t weight_bytes;      /* Req_i, parameter part */
    uint64_t kv_bytes_per_token;/* Req_i, cache part per cached token: 2 * Hkv * dh * sizeof(dtype) */
} shard_layer_profile;

/* Build a shard for layers [layer_lo, layer_hi) (0 <= layer_lo < layer_hi; the indices
 * only label the range - `w` holds layer_hi - layer_lo entries, entry 0 being layer_lo).
 * Copies (and repacks) all weights into library-owned device memory and pre-allocates the
 * KV page pool (max_seqs * ceil(max_seq_len / page_size) pages per layer for K and V) and
 * all workspace (Sec. 3: the KV cache is pre-allocated on each participating device);
 * the caller may free its weight buffers when the call returns.
 * weights_on_device: 0 = the pointers in `w` are host pointers, 1 = device pointers.
 * Blocks until the upload is complete.  On failure *out is NULL. */
int shard_create(shard_t **out, const shard_model_cfg *model, const shard_kv_cfg *kv,
                 int32_t layer_lo, int32_t layer_hi, const shard_layer_weights *w,
                 int32_t weights_on_device);

/* Wait for the shard's outstanding work and release everything it owns.  NULL is OK. */
int shard_destroy(shard_t *s);

/* Reserve a sequence slot (an empty KV cache row); *seq_id receives its id.
 * SHARD_E_KV_FULL when max_seqs are live. */
int shard_seq_alloc(shard_t *s, int32_t *seq_id);

/* Return a sequence's pages to the pool.  Work already enqueued that uses the sequence
 * must have completed.  SHARD_E_STATE for an id that is not live. */
int shard_seq_free(shard_t *s, int32_t seq_id);

/* Tokens currently cached for a live sequence, or a negative error code. */
int32_t shard_seq_len(shard_t *s, int32_t seq_id);

/* Prefill phase (Sec. 2): append T tokens to each of the B distinct sequences seq_ids[0..B)
 * (host pointer) and produce the range's output activation for every token.
 * x_in, x_out: device pointers, float32 [B, T, d_model] row-major; x_out may alias x_in.
 * Sequence b's tokens take positions P_b .. P_b+T-1 where P_b is its current length, so a
 * non-empty sequence is legal (chunked prefill).  1 <= B <= SHARD_MAX_BATCH,
 * B*T <= max_batch_tokens, P_b + T <= max_seq_len (else SHARD_E_KV_FULL). */
int shard_prefill(shard_t *s, const int32_t *seq_ids, int32_t B, int32_t T,
                  const void *x_in, void *x_out, void *hip_stream);

/* Autoregressive phase (Sec. 2): one new token for each of the B distinct sequences, each
 * of which must already hold at least one token (SHARD_E_STATE otherwise); lengths may
 * differ between sequences.  x_in, x_out: device pointers, float32 [B, d_model]. */
int shard_decode(shard_t *s, const int32_t *seq_ids, int32_t B,
                 const void *x_in, void *x_out, void *hip_stream);

/* shard_decode for callers that cannot allocate device memory or must know that no library
 * call does: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and same results as shard_decode, but every
 * intermediate buffer of the step (normalised activations, q, attention output and its
 * context-slice partials, the SwiGLU output) is carved from one array of
 * SHARD_STATIC_SCRATCH_BYTES that lives in the library's device image (one copy per GPU, held
 * until the process ends) instead of the workspace shard_create allocated; the call makes no
 * hipMalloc / hipFree and creates no events.  A step whose buffers would not fit
 * (roughly B * (3 d_model + 2 Hq dh + ffn_dim) * 4 bytes plus the attention partials) is
 * refused with SHARD_E_INVAL and a message that states both sizes; so is a call while
 * shard_timing_enable is on (timing creates events).  All calls on one GPU, from any shard,
 * share that array: calls that overlap on the device (different streams or shards) race -
 * order them on one stream or with events.  Nothing in the array needs to start at zero. */
#define SHARD_STATIC_SCRATCH_BYTES (8u << 20)
int shard_decode_static(shard_t *s, const int32_t *seq_ids, int32_t B,
                        const void *x_in, void *x_out, void *hip_stream);

/* Whether a value rounded to IEEE half by this shard's kernels has left half's range since
 * the shard was created (or since the flag was last cleared): *overflowed = 0 or 1, for the
 * work that has completed on the device.  clear != 0 resets the flag; the KV cache of the
 * sequences that were running may hold infinities - free them.  Always 0 for SHARD_F32. */
int shard_overflow(shard_t *s, int32_t clear, int32_t *overflowed);

/* Offline profiling of this device's column of the planner's inputs (Sec. 3 "Profiling"):
 * on scratch sequences and zero-free synthetic activations, time every layer of the range
 * with HIP events in a prefill of (B, T_prefill) and in n_decode following decode steps,
 * averaged over `iters` repetitions, and report activation and memory sizes.
 * Needs B free sequence slots; blocks until done; `out` is a host array of
 * layer_hi - layer_lo entries. */
int shard_profile(shard_t *s, int32_t B, int32_t T_prefill, int32_t n_decode, int32_t iters,
                  shard_layer_profile *out);

/* Kernel timing for roofline reports.  While enabled, every kernel dispatch carries a HIP
 * event pair that reads the kernel's own start and end (no launch gaps, the figure a
 * profiler's kernel trace gives); shard_timing_read waits for the stream work recorded so
 * far and returns kernel launches and total kernel seconds per class since enable.  The
 * classes are the steps of the layer, separately for the autoregressive and the prefill
 * phase; a class may hold more than one kernel per layer (attention + its merge; the
 * one-off cast of x_in to half on the batched 16-bit decode path counts with the QKV class). */
enum {
    SHARD_K_DECODE_QKV = 0,     /* RMSNorm + QKV projection + RoPE + KV append */
    SHARD_K_DECODE_ATTN = 1,
    SHARD_K_DECODE_O = 2,       /* O projection + residual */
    SHARD_K_DECODE_GATEUP = 3,  /* RMSNorm + gate/up projection + SwiGLU */
    SHARD_K_DECODE_DOWN = 4,    /* down projection + residual */
    SHARD_K_PREFILL_NORM = 5,   /* both RMSNorms */
    SHARD_K_PREFILL_QKV = 6,    /* QKV GEMM + RoPE + KV append */
    SHARD_K_PREFILL_ATTN = 7,
    SHARD_K_PREFILL_O = 8,
    SHARD_K_PREFILL_GATEUP = 9,
    SHARD_K_PREFILL_DOWN = 10,
    SHARD_K_COUNT = 11
};
int shard_timing_enable(shard_t *s, int32_t on);
int shard_timing_read(shard_t *s, int64_t launches[SHARD_K_COUNT], double seconds[SHARD_K_COUNT]);

/* ---- The ends of a model around its decoder layers -------------------------------------
 * The N layers the paper places include the token embedding and the output projection next
 * to the decoder layers (Sec. 4 "System Model"), and the first of them, which sees the raw
 * input tokens, is pinned to the source node (Eq. 4).  A shard maps hidden states to hidden
 * states; these entry points supply what comes before the first shard and after the last:
 * the token embedding lookup, and the final RMSNorm + output projection ("LM head") with a
 * greedy choice of the next token, so that a whole token loop can run on library calls.
 * The vocabulary size is the model's (32000 for Llama 2; not stated in the paper).
 * An ends object holds whichever of the two ends it was given; same conventions as above. */
typedef struct shard_ends shard_ends_t;

/* tok_embeddings [vocab, d_model] and lm_head [vocab, d_model] are row-major in
 * model->weight_dtype (bf16 as raw 16-bit patterns, converted once to IEEE half like the
 * layer matrices); g_final is float32 [d_model].  tok_embeddings may be NULL (no embedding
 * end), and so may g_final together with lm_head (no output end); at least one end must be
 * given.  Copies everything; blocks until the upload is complete.  max_tokens >= 1 is the
 * largest n of one shard_ends_embed call. */
int shard_ends_create(shard_ends_t **out, const shard_model_cfg *model, int32_t vocab, int32_t max_tokens,
                      const void *tok_embeddings, const float *g_final, const void *lm_head,
                      int32_t weights_on_device);
int shard_ends_destroy(shard_ends_t *e);

/* x_out[i, :] = tok_embeddings[token_ids[i], :] as float32, i < n.  token_ids: HOST pointer
 * (the ids are validated here: an id outside [0, vocab) is SHARD_E_INVAL and nothing is
 * enqueued).  x_out: device pointer, float32 [n, d_model]. */
int shard_ends_embed(shard_ends_t *e, const int32_t *token_ids, int32_t n, void *x_out, void *hip_stream);

/* logits[i, :] = lm_head . rmsnorm(x[i, :]; g_final), i < n, 1 <= n <= SHARD_MAX_BATCH.
 * x: device float32 [n, d_model] (the last shard's output for the tokens whose successor is
 * wanted); logits: device float32 [n, vocab]. */
int shard_ends_logits(shard_ends_t *e, const void *x, int32_t n, void *logits, void *hip_stream);

/* token_ids_out[i] = argmax_j logits[i, j] (greedy decoding; the lowest index among equal
 * maxima).  logits: device float32 [n, vocab]; token_ids_out: device int32 [n]. */
int shard_ends_argmax(shard_ends_t *e, const void *logits, int32_t n, int32_t *token_ids_out, void *hip_stream);

/* Message for the most recent failure on this thread ("" if none). */
const char *shard_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SHARD_H */
