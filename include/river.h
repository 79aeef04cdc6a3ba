/*
 * river.h -- C ABI of the MI355X (gfx950) early-exit decode library.
 *
 * The library runs the batch-1 autoregressive decode step of a decoder-only
 * transformer with token-level early exit as River-LLM defines it (method
 * section: "KV-Shared Exit Layer" and "Inference with Seamless Exit", Eq. 1):
 * after backbone block l the cosine similarity between the block's input and
 * output hidden state is compared with tau; once a token exits, the remaining
 * blocks run as 4-bit weight-only twins (the Exit River) that read and write the
 * SAME KV-cache slots as the backbone blocks they replace, and the original
 * final norm + LM head produce the logits.
 *
 * Conventions
 *  - Every pointer is marked HOST or DEVICE.  Device memory is allocated by the
 *    caller (for example through torch) and handed over.  The one exception:
 *    the first river_create on a device allocates 128 KiB of uncached device
 *    memory for the counters of the device-wide barrier (2 KiB per live
 *    context, at most 64 contexts per device); it is kept until the process
 *    ends.  The context borrows weights and workspace: they must outlive it.
 *  - All calls return RIVER_OK (0) or a negative RIVER_E* code, never throw and
 *    never abort.  river_last_error() gives a text for the last failure.
 *  - Matrices are [out, in] row-major (nn.Linear orientation).  dtype selects
 *    the storage type of weights and KV cache; the residual stream, all
 *    accumulation, softmax and the similarity are fp32.
 *  - A context is single-threaded.  All work is enqueued on the hipStream_t
 *    given at creation.
 *  - Blocks are numbered 1..L; the exit position e of a token is the number of
 *    backbone blocks it executed (caption of the paper's exit-position table);
 *    e = L means no exit; river twins run blocks e+1..L.
 */
#ifndef RIVER_H
#define RIVER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct river_ctx river_ctx; /* opaque */

enum {
  RIVER_OK = 0,
  RIVER_EINVAL = -1, /* bad configuration, null pointer, value out of range */
  RIVER_ENOSPC = -2, /* max_seq or workspace exceeded */
  RIVER_ESTATE = -3, /* call out of order (decode before prefill, ...) */
  RIVER_EHIP = -4    /* HIP runtime failure or a device-side wait that timed out */
};

enum { RIVER_F32 = 0, RIVER_BF16 = 1 };

/* Storage type of the KV cache: the weight dtype, or IEEE half (the paper keeps the cache in
 * FP16; "KV-Shared Exit Layer" subsection).  RIVER_KV_F16 needs RIVER_BF16 weights. */
enum { RIVER_KV_SAME = 0, RIVER_KV_F16 = 1 };

/* How one decode step is issued.  Both run the same device code.
 * KERNELS: one launch per phase (6 + 5 per block), no cross-workgroup waiting.
 * PERSISTENT: one launch per token; workgroups meet at device-wide barriers
 * whose waits are bounded by spin_limit.  Offered for RIVER_BF16 only:
 * river_create and river_workspace_bytes refuse it for RIVER_F32. */
enum { RIVER_EXEC_KERNELS = 0, RIVER_EXEC_PERSISTENT = 1 };

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_base; /* theta_i = rope_base^(-2i/head_dim), rotate-half pairing (i, i+head_dim/2) */
  float rms_eps;
  int32_t dtype;          /* RIVER_F32 or RIVER_BF16: weights, river scale/zero, KV cache */
  int32_t max_batch;      /* sequences the context holds, 1..32.  1: the batch-1 decode path
                             (river_decode_step).  > 1: a batched context (river_decode_batch); needs RIVER_BF16
                             and d_model, d_ffn, river_group multiples of 64 */
  int32_t max_seq;        /* KV-cache capacity in positions */
  int32_t min_exit_layer; /* L_s: smallest allowed exit position ("predefined entry layer") */
  float tau;              /* Eq. 1 threshold, strict '>' ; tau >= 1 never exits */
  int32_t river_bits;     /* must be 4 */
  int32_t river_group;    /* consecutive input elements per quantisation group, multiple of 32 */
  int32_t exec_mode;      /* RIVER_EXEC_* */
  int32_t spin_limit;     /* PERSISTENT: polls before a barrier wait gives up (0 = default) */
  int32_t prefill_gemm_min_tokens; /* prompts of at least this many tokens are prefilled with MFMA GEMMs
                                      (RIVER_BF16, d_model, d_ffn and river_group multiples of 64); shorter
                                      ones, and all other configurations, run the decode kernels per prompt
                                      position.  0 = default (32); negative = never */
  int32_t batch_exit_rule; /* batched contexts, when Eq. 1 decides: 0 = every sequence for itself
                              (s_b > tau); 1 = Eq. 1 as printed: the whole batch leaves the backbone together at
                              the first block with min over the batch of s_b > tau */
  int32_t kv_dtype;        /* RIVER_KV_* */
} river_config;

/* Backbone weights.  DEVICE pointers in HOST arrays of length n_layers.  "DEVICE" includes
 * pinned host memory that the device can address (hipHostMalloc): the paper's Backbone
 * Offloading keeps deep, rarely reached backbone blocks out of VRAM while the river stays
 * resident; a caller does that by handing such pointers for those blocks' matrices, which the
 * kernels then read in place over the host link only when a token reaches them. */
typedef struct {
  const void *tok_emb;    /* [vocab, d_model] */
  const void *final_norm; /* [d_model] */
  const void *lm_head;    /* [vocab, d_model] */
  const void *const *attn_norm, *const *wq, *const *wk, *const *wv, *const *wo;
  const void *const *ffn_norm, *const *w_gate, *const *w_up, *const *w_down;
} river_weights;

/*
 * River twin of the seven matrices of each block, order wq wk wv wo w_gate w_up
 * w_down.  For a [rows, cols] matrix: codes [rows, cols/2] bytes, two 4-bit codes
 * per byte with the even column in the low nibble; scale and zero
 * [rows, ceil(cols/group)] in `dtype`; weight = (code - zero) * scale.  Norm gains
 * are shared with the backbone.  DEVICE pointers in HOST arrays of length
 * n_layers; entries of blocks that never run as twins (l <= L_s) may be NULL.
 */
typedef struct {
  const void *const *codes[7];
  const void *const *scale[7];
  const void *const *zero[7];
} river_qweights;

/*
 * River construction ("KV-Shared Exit Layer": the twin inherits the block's
 * parameters, then 4-bit weight-only PTQ).  Asymmetric round-to-nearest per
 * group of `group` consecutive input elements of one row (last group shorter
 * if group does not divide cols), fp32 arithmetic:
 *   scale = (max-min)/15 (1 if max == min), zero = -min/scale, both stored in
 *   `dtype`; code = clamp(rint(w/scale + zero), 0, 15) with the stored values.
 * w, codes, scale, zero: DEVICE.  Asynchronous on `hip_stream`.
 * Requires cols % 16 == 0 and group % 32 == 0.
 */
int river_quantize_w4(const void *w, int64_t rows, int64_t cols, int32_t group, int32_t dtype,
                      void *codes, void *scale, void *zero, void *hip_stream);

/* Bytes of DEVICE workspace river_create needs for this configuration (KV cache,
 * RoPE table, activations, partial results, step records); 0 if cfg is invalid.
 * A batched context (max_batch > 1) also keeps, in the workspace, a second copy of
 * every block matrix (bf16 and 4-bit) and of the LM head in the order its GEMM
 * streams them, written by river_create: about the size of the model again. */
size_t river_workspace_bytes(const river_config *cfg);

/*
 * Creates a context.  cfg, w, q: HOST structs (copied).  q may be NULL if
 * tau >= 1 and no forced exit below L will be requested.  workspace: DEVICE,
 * 256-byte aligned, at least river_workspace_bytes(cfg) bytes; the library
 * initialises it.  hip_stream: a hipStream_t (NULL = the null stream).
 */
int river_create(const river_config *cfg, const river_weights *w, const river_qweights *q,
                 void *workspace, size_t workspace_bytes, void *hip_stream, river_ctx **out);

/*
 * river_create for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc).  Same arguments and
 * behaviour as river_create, and the workspace must have the same size, but the call
 * allocates nothing: the step-transient part of the workspace (activations, partial
 * results, counters, step records, descriptor tables) and the counters of the device-wide
 * barrier live in a static device array of 8 MiB inside the library, which every GPU the
 * library runs on holds until the process ends; the KV cache, the RoPE table and the packed
 * river scales stay in the caller's workspace.  RIVER_ENOSPC if the configuration needs more
 * than the 8 MiB (the 8B shape needs 4.5 MiB).  The array is shared by every call on a device
 * and keeps the last context's contents; the call clears what must start at zero.  At most one
 * context created this way can be live per device (RIVER_ESTATE otherwise: two would race on
 * the array); contexts from river_create are not affected.  The barrier counters are then in
 * ordinary device memory and polled with device-coherent vector loads, a few percent slower
 * per token than river_create's uncached pool; results are identical.
 */
int river_create_static(const river_config *cfg, const river_weights *w, const river_qweights *q,
                        void *workspace, size_t workspace_bytes, void *hip_stream, river_ctx **out);

/*
 * Prefill phase ("Inference with Seamless Exit", list of phases: the prompt is
 * processed by sequence-level exit, all prompt tokens leaving the backbone at one
 * unified depth).  prefill_exit_layer is that depth e_p: every prompt position runs
 * backbone blocks 1..e_p and river twins e_p+1..L, filling the shared KV cache for
 * positions 0..n_tokens-1 of every block.  e_p must lie in [L_s, L]; negative or L =
 * the full backbone depth (then no river weights are needed).  How e_p is chosen the
 * paper leaves open: it is the caller's.  Restarts the sequence at position 0.
 * seq: the sequence (0 unless the context is batched).  tokens: HOST [n_tokens].  out_token: HOST, the greedy token after
 * the last prompt position (nullable).  out_logits: DEVICE fp32 [vocab], the logits of
 * the last prompt position (nullable).  Synchronises the stream.
 */
int river_prefill(river_ctx *ctx, int32_t seq, const int32_t *tokens, int32_t n_tokens,
                  int32_t prefill_exit_layer, int32_t *out_token, float *out_logits);

/*
 * Generation phase, one token-level-exit decode step (Eq. 1).
 * in_token:    HOST, the token to consume; NULL = the token the previous step (or
 *              the prefill) produced, taken on the device without a host round trip.
 * forced_exit: HOST; NULL = Eq. 1 decides with cfg.tau.  Otherwise *forced_exit is
 *              the exit position to impose: in [L_s, L] (L = run the whole
 *              backbone), or 0 when L_s == 0.  The similarities are still computed.
 * out_token, out_exit_layer: HOST; if out_token is NULL nothing is copied back and
 *              the call does not synchronise (steps can be queued back to back; read
 *              the results later with river_read_records).
 * out_sims:    HOST [n_layers], nullable: s(l) for executed backbone blocks, NaN for
 *              river blocks.
 * Advances the sequence by one position.  RIVER_ENOSPC if the cache is full.
 */
int river_decode_step(river_ctx *ctx, const int32_t *in_token, const int32_t *forced_exit,
                      int32_t *out_token, int32_t *out_exit_layer, float *out_sims);

/*
 * One decode step of a batched context (max_batch > 1) for sequences 0..n_seq-1, each at
 * its own position and with its own exit depth ("Inference with Seamless Exit"; Eq. 1 is
 * stated over a batch B).  Every sequence must have been prefilled (river_prefill with its
 * seq index).  Per block the rows still in the backbone run the bf16 matrices and the rows
 * that have left it the 4-bit twins, both as MFMA GEMMs that write K/V to the sequence's
 * own slot of the shared cache; which side a row is on is decided on the device after each
 * backbone block by cfg.batch_exit_rule, or imposed by forced_exit.
 * in_tokens:   HOST [n_seq] or NULL (= the tokens the previous step / prefill produced).
 * forced_exit: HOST [n_seq] or NULL; entry b < 0 lets Eq. 1 decide for sequence b, else
 *              the exit position to impose, in [L_s, L] (or 0 when L_s == 0).
 * out_tokens, out_exit_layers: HOST [n_seq]; out_sims: HOST [n_seq][n_layers] (NaN for
 *              blocks run as river twins); all nullable; if out_tokens is NULL the call
 *              does not synchronise (read results with river_read_batch_records).
 * Advances every sequence by one position.
 */
int river_decode_batch(river_ctx *ctx, int32_t n_seq, const int32_t *in_tokens, const int32_t *forced_exit,
                       int32_t *out_tokens, int32_t *out_exit_layers, float *out_sims);

/* Synchronises and copies tokens and exit positions of the last n_steps batched steps (at most
 * 1024, oldest first) for sequences 0..n_seq-1.  tokens, exit_layers: HOST [n_steps][n_seq]. */
int river_read_batch_records(river_ctx *ctx, int32_t n_steps, int32_t n_seq, int32_t *tokens,
                             int32_t *exit_layers);

/* Synchronises and copies the records of the last n decode steps (n <= 4096, oldest
 * first).  tokens, exit_layers: HOST [n]; sims: HOST [n][n_layers], nullable. */
int river_read_records(river_ctx *ctx, int32_t n, int32_t *tokens, int32_t *exit_layers,
                       float *sims);

/* Moves sequence seq back to new_len positions (0 <= new_len <= current length) so
 * that steps can be replayed; cache contents are left as they are. */
int river_rewind(river_ctx *ctx, int32_t seq, int32_t new_len);

/* Number of positions currently in the cache, or a negative error. */
int river_position(const river_ctx *ctx);
int river_seq_position(const river_ctx *ctx, int32_t seq); /* the same for sequence seq of a batched context */

enum {
  RIVER_DBG_HIDDEN = 0, /* fp32 [n_layers+1][d_model]: h(0..L) of the last token processed */
  RIVER_DBG_LOGITS = 1, /* fp32 [vocab] of the last step that ran the head */
  RIVER_DBG_KCACHE = 2, /* cache storage type [max_batch][n_layers][max_seq][n_kv_heads*head_dim] */
  RIVER_DBG_VCACHE = 3,
  RIVER_DBG_TRACE = 4,  /* uint64 [5*n_layers][2][workgroups] then [64]: 100 MHz device clock at which each
                           workgroup arrived at / was released from each device-wide barrier of the last
                           launch, then 64 marks inside the phases (PERSISTENT mode of a library built
                           with -DRIVER_TRACE; zeros otherwise); bytes = (5*n_layers*2*workgroups + 64)*8 */
  RIVER_DBG_BATCH_HIDDEN = 5, /* batched context: fp32 [n_layers+1][max_batch][d_model] of the last step */
  RIVER_DBG_BATCH_LOGITS = 6  /* batched context: fp32 [max_batch][vocab] of the last step */
};
/* Synchronises and copies a device buffer to dst (HOST, `bytes` must equal its size). */
int river_get_debug(river_ctx *ctx, int32_t what, void *dst, size_t bytes);

/* Overwrites the whole KV cache with the byte `value` (tests use a NaN pattern as a
 * canary for slots that are read before they are written).  Asynchronous. */
int river_fill_cache(river_ctx *ctx, int32_t value);

const char *river_last_error(const river_ctx *ctx); /* ctx may be NULL: last create error */
int river_destroy(river_ctx *ctx);                  /* NULL is a no-op */

#ifdef __cplusplus
}
#endif
#endif /* RIVER_H */
