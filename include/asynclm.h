/*
 * libasynclm - the inference process of asynchronous LLM function calling (arXiv 2412.07017)
 * on one AMD MI355X (gfx950): autoregressive decoding that keeps running while function calls
 * execute, plus in-flight injection of interrupt tokens into the live K/V cache.
 *
 * What the calls mean follows the paper's statement of the problem:
 *   - Sec. 5 / Fig. 4: the system intercepts the model's autoregressive token generation; one
 *     iteration is "forward over the newest token(s) -> next-token distribution -> pick a token".
 *   - Sec. 3.2: when a call returns, an interrupt block is inserted at the end of the token stream
 *     (the LLM context) and generation resumes after the block.
 *   - Sec. 5.3: queued interrupts are appended to the generated tokens and processed by the model
 *     in its next forward pass; this never happens in the middle of a step.
 *   - Sec. 5.5: the stateless alternative recomputes the whole context per interrupt; both see the
 *     same context, so after any successful call the logits of a sequence equal those of a
 *     from-scratch pass of the decoder over that sequence's whole token stream.
 * The control plane of the paper (CML grammar, token monitor, executor, interrupt queue, critical
 * sections, trap handling) sits above this interface and only hands it integer token ids.
 *
 * Model: Llama-style decoder (RMSNorm with eps inside the root, rotary embedding on half-split
 * pairs (i, i+head_dim/2) with angle pos * theta^(-2i/head_dim), grouped-query causal attention
 * scaled by 1/sqrt(head_dim), SwiGLU feed-forward, no biases, separate output head).
 *
 * Conventions
 *   - Every function returns 0 on success or a negative ASYNCLM_E_* code.  A failed call leaves the
 *     sequence (length, cache, logits) unchanged, except ASYNCLM_E_DEVICE which poisons the context.
 *   - "device pointer" = memory of the GPU that was current when asynclm_create ran; "host pointer"
 *     = ordinary process memory.  The library never frees or writes caller memory other than the
 *     documented outputs.
 *   - One caller thread per context.  Work is enqueued on the HIP stream given at create; calls
 *     that return data to the host synchronise that stream, the others may return before the GPU
 *     has finished.
 *   - All memory the library needs (K/V cache, rotary table, activations, logits, pinned staging, the captured
 *     graphs of the decoding steps for every context length up to max_positions) is allocated in asynclm_create.
 *     Of the other calls only asynclm_set_option allocates (options that change the launch geometry of a decoding
 *     step build its graphs again) and asynclm_profile_step (events).
 */
#ifndef ASYNCLM_H
#define ASYNCLM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ASYNCLM_OK           0
#define ASYNCLM_E_INVAL     -1   /* null pointer, bad sequence index, token id outside [0, vocab), count <= 0, bad shape */
#define ASYNCLM_E_STATE     -2   /* decode / inject / logits on an empty sequence; prefill on a non-empty one */
#define ASYNCLM_E_CAPACITY  -3   /* the call would grow a sequence beyond max_positions (checked before any change) */
#define ASYNCLM_E_NOMEM     -4   /* device or host allocation failed in asynclm_create */
#define ASYNCLM_E_DEVICE    -5   /* a HIP call failed; the context is unusable afterwards */

#define ASYNCLM_DTYPE_FP32 0
#define ASYNCLM_DTYPE_BF16 1

/* Storage of cached keys and values.
 * AUTO: fp32 for fp32 models; for bf16 models a PAIR of bf16 planes, hi = bf16(x) and
 *       lo = bf16(x - hi) (about 16 mantissa bits, 4 bytes per element), which keeps the logits within
 *       the bf16 parity tolerance of an fp32 reference at any depth.  Models that the matrix-core append path
 *       serves (bf16, head_dim 128, d_model and ffn multiples of 128) keep the values only transposed and tiled
 *       (the operand order of that path's attention, which also serves their decoding steps).
 * BF16: bf16 models only: the hi plane alone (2 bytes per element).  Halves cache size and traffic; the
 *       rounding of K and V then moves logits by several 1e-2 on N(0, 0.02)-initialised models.
 * PAIR_ROWS: as AUTO, and the values are kept row by row as well (half as much cache again): the layout that the
 *       single-row attention kernel reads, which the options "attn_mfma_min" = 0, "fused" and "pipeline" need on
 *       models of the append path (they are ignored there without it). */
#define ASYNCLM_KV_AUTO 0
#define ASYNCLM_KV_BF16 1
#define ASYNCLM_KV_PAIR_ROWS 2

typedef struct asynclm_ctx asynclm_ctx;   /* opaque; owned by the library */

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    float   rms_eps, rope_theta;
    int32_t dtype;           /* ASYNCLM_DTYPE_*: storage type of all matrices and of the K/V cache */
    int32_t max_seqs;        /* number of independent sequences (>= 1) */
    int32_t max_positions;   /* K/V capacity per sequence, in tokens */
    int32_t kv_format;       /* ASYNCLM_KV_* */
} asynclm_config;
/* Shape limits: head_dim in {64, 128}; n_q_heads a multiple of n_kv_heads with ratio <= 8;
 * d_model, ffn multiples of 8; everything > 0. */

/* Device pointers, borrowed: they must stay valid and unchanged until asynclm_destroy.
 * Matrices are row-major [out, in] in `dtype`; norm gains are fp32 whatever `dtype` is.
 * The six per-layer members are HOST arrays of n_layers device pointers (read during create). */
typedef struct {
    const void *embed;        /* [vocab, d_model] */
    const float *final_norm;  /* [d_model] */
    const void *lm_head;      /* [vocab, d_model] */
    const float *const *attn_norm;  /* each [d_model] */
    const void *const *wqkv;        /* each [(n_q_heads + 2 n_kv_heads) head_dim, d_model]: query rows, key rows, value rows */
    const void *const *wo;          /* each [d_model, n_q_heads head_dim] */
    const float *const *ffn_norm;   /* each [d_model] */
    const void *const *wgate_up;    /* each [2 ffn, d_model]: gate rows, then up rows */
    const void *const *wdown;       /* each [d_model, ffn] */
} asynclm_weights;

/* Create a context on the current HIP device.  `hip_stream` is a hipStream_t (NULL = the null
 * stream) on which all work is enqueued; it is borrowed.  On failure *out is NULL. */
int asynclm_create(asynclm_ctx **out, const asynclm_config *cfg, const asynclm_weights *w, void *hip_stream);

/* Waits for outstanding work, frees everything the library allocated.  NULL is allowed. */
int asynclm_destroy(asynclm_ctx *ctx);

/* Start a sequence: process n >= 1 prompt tokens (host pointer) into the empty sequence `seq`.
 * Afterwards the logits predict the token that follows the prompt. */
int asynclm_prefill(asynclm_ctx *ctx, int32_t seq, const int32_t *tokens, int32_t n);

/* One decoding step (Fig. 4): choose the next token - `forced_token` if >= 0, else the greedy
 * argmax of the current logits, lowest index on ties, computed on the device - append it to the
 * sequence and run one forward pass, leaving the logits for the token after it.
 * token_out (host pointer, may be NULL): receives the chosen token.  The call waits only until the
 * token has been chosen (the first kernel of the step), not for the forward pass, which is still
 * running when it returns: the caller (the token monitor of Sec. 5.1) works on the token while
 * the device computes, and the next call queues behind the running step.  (With the "fused"
 * option the call waits for the whole step.)  NULL: nothing is waited for. */
int asynclm_decode_step(asynclm_ctx *ctx, int32_t seq, int32_t forced_token, int32_t *token_out);

/* In-flight interrupt injection (Sec. 3.2, 5.3): append the k >= 1 tokens (host pointer) to the end
 * of the live context of `seq` without touching the cached prefix, and leave the logits for the
 * token after the block.  Legal between any two decoding steps of a non-empty sequence. */
int asynclm_inject_interrupt(asynclm_ctx *ctx, int32_t seq, const int32_t *tokens, int32_t k);

/* One batched iteration over several sequences with ONE pass over the weights (Sec. 5.3: the interrupts that are
 * queued when a step ends are appended to the just-generated tokens and processed in the next forward pass).
 * For i in [0, nseq): sequence seqs[i] (all distinct, non-empty) gets the rows
 *     [chosen token] ++ intr_tokens[intr_offsets[i] .. intr_offsets[i+1])
 * where the chosen token is forced[i] if forced != NULL and forced[i] >= 0, else the greedy argmax of the
 * sequence's current logits (device side).  All rows of all sequences go through the layers together (each
 * row attends to its own sequence only); afterwards every sequence has valid logits for its next token.
 * seqs, forced, intr_tokens, intr_offsets (nseq + 1 ascending entries; NULL = no interrupts) are host pointers.
 * tokens_out (host, may be NULL): tokens_out[i] receives the token chosen for seqs[i]; NULL avoids the stream
 * synchronisation.  More rows than one pass holds (512) are processed in several passes.
 * Everything is validated before any state changes (ASYNCLM_E_INVAL / _STATE / _CAPACITY as for the
 * single-sequence calls; a sequence may appear only once). */
int asynclm_step_batch(asynclm_ctx *ctx, int32_t nseq, const int32_t *seqs, const int32_t *forced,
                       const int32_t *intr_tokens, const int32_t *intr_offsets, int32_t *tokens_out);

/* Device half of the token monitor (Sec. 5.1: the monitor keeps tokens such as the interrupt marker out of the
 * next-token distribution): every later greedy choice of `seq` skips the n <= 31 token ids in `ids` (host pointer;
 * n = 0 clears the list).  Applies to the tokens chosen by asynclm_decode_step and asynclm_step_batch when no token
 * is forced, starting with the very next one; the logits themselves are returned unmasked.  The list survives
 * asynclm_reset. */
int asynclm_set_banned_tokens(asynclm_ctx *ctx, int32_t seq, const int32_t *ids, int32_t n);

/* The token the next unforced asynclm_decode_step / asynclm_step_batch would choose for `seq` (greedy over the ids
 * that are not banned), without changing anything.  The host-side interrupt manager needs it: whether queued
 * interrupts may ride with the next token (Sec. 5.3) depends on that token (a token that opens a call block
 * starts a critical section, Sec. 3.2).  Synchronises the stream. */
int asynclm_peek_token(asynclm_ctx *ctx, int32_t seq, int32_t *token_out);

/* asynclm_peek_token's choice for callers that cannot allocate and have no context: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Picks the greedy token (maximum, lowest index on ties, the
 * n_banned ids in banned_dev skipped) of logits_dev[0..n) and stores it to *token_out_dev, with the same kernel as
 * asynclm_peek_token; the kernel's scratch (per-block maxima, a counter: about 2.3 KB) is a static array in device
 * memory, one copy per GPU, held until the process ends, instead of a workspace of a context.  All three pointers are
 * DEVICE pointers owned by the caller; the work is enqueued on hip_stream (a stream of the current device) and the
 * call does not wait for it.  No hipMalloc, hipFree or other allocating call is made.
 * Limits: 1 <= n <= ASYNCLM_STATIC_MAX_VOCAB, 0 <= n_banned <= 31, else ASYNCLM_E_INVAL and nothing is enqueued.
 * Every call on a GPU uses that GPU's one scratch array: calls that overlap on one GPU (two streams, two threads)
 * race; calls on one stream are ordered.  The array keeps the last call's contents; the call clears what it needs. */
#define ASYNCLM_STATIC_MAX_VOCAB (1 << 24)
int asynclm_greedy_token_static(const float *logits_dev, int32_t n, const int32_t *banned_dev, int32_t n_banned,
                                int32_t *token_out_dev, void *hip_stream);

/* Trap handling support (Sec. 5.4): while a sequence is paused its K/V state can be kept in place, dropped and
 * recomputed later (asynclm_reset + asynclm_prefill of the whole stream: time grows faster than linearly with the
 * context), or swapped to host memory and back (linear).  These calls are the swap; they synchronise the stream.
 *   asynclm_kv_bytes     size of the host image of `seq` at its current length
 *   asynclm_kv_swap_out  writes the image (cached rows of all layers, current logits, pending greedy token) to
 *                        host_buf[0..capacity) (host pointer; pinned memory copies fastest); ASYNCLM_E_CAPACITY if it
 *                        does not fit.  The sequence stays valid; asynclm_reset then frees its slot.
 *   asynclm_kv_swap_in   restores an image into the EMPTY sequence `seq` (any slot of a context created with the
 *                        same configuration; the image carries its own description and is checked).  Afterwards the
 *                        sequence is exactly as it was at swap-out: same logits, same next greedy token. */
int asynclm_kv_bytes(asynclm_ctx *ctx, int32_t seq, uint64_t *bytes);
int asynclm_kv_swap_out(asynclm_ctx *ctx, int32_t seq, void *host_buf, uint64_t capacity);
int asynclm_kv_swap_in(asynclm_ctx *ctx, int32_t seq, const void *host_buf, uint64_t bytes);

/* Copy the current next-token logits of `seq` (fp32) to out_host[0..n); n must equal vocab.
 * Synchronises the stream. */
int asynclm_logits(asynclm_ctx *ctx, int32_t seq, float *out_host, int32_t n);

/* Device address of the same fp32[vocab] logits (valid until destroy; contents change with every
 * call on `seq`, in stream order). */
int asynclm_logits_device(asynclm_ctx *ctx, int32_t seq, const float **out_dev);

/* Number of tokens in the context of `seq` (prompt + generated + injected). */
int asynclm_seq_len(asynclm_ctx *ctx, int32_t seq, int32_t *len);

/* Forget the sequence: length 0, cache rows reusable. */
int asynclm_reset(asynclm_ctx *ctx, int32_t seq);

/* Block until all enqueued work of this context has finished. */
int asynclm_synchronize(asynclm_ctx *ctx);

/* Tuning knobs; all have working defaults.  Unknown names give ASYNCLM_E_INVAL.
 *   "chunk"        rows processed per forward pass by prefill / inject (1 .. 512); 1 = token by token
 *                  through the decode kernels.  Default 512 where the matrix-core append path applies
 *                  (bf16 model, paired cache, head_dim 128, d_model and ffn multiples of 128), else 1.
 *   "chunk_split"  0 = split-K factors of the append path's products chosen from the shapes and the number
 *                  of compute units, 1..8 = force one
 *   "fused"        1 = run a decoding step as one persistent cooperative kernel (where the device and the
 *                  model shape allow it; ignored otherwise), 0 = one kernel per operation (default)
 *   "graph"        (per-operation kernels only) 1 = replay decoding steps as a captured HIP graph,
 *                  0 = launch kernels one by one
 *   "pipeline"     (per-operation kernels only) 1 = run a decoding step with its kernels alternating between the
 *                  caller's stream and a second stream of the library's, neighbouring kernels overlapping and handing
 *                  over through counters in device memory instead of kernel boundaries (contexts up to 2048 tokens,
 *                  models of which two workgroups per kernel fit a compute unit; ignored otherwise); 0 (default) = one
 *                  stream.  Same arithmetic per kernel (bf16 models take the single-row attention kernel here, so their
 *                  logits agree with the default within rounding).  Measured slower than the default on the 8B shape.
 *   "gemv_grid"    workgroups per matrix-vector kernel (default: the number of compute units).  For experiments; the
 *                  value is shared by every context of the process.
 *   "step_stamps"  1 = the kernels of decoding steps of the default (one-stream) kind whose attention runs on the
 *                  matrix cores leave time stamps for asynclm_profile_trace (measurement only; the step graphs are
 *                  instantiated again when the option changes).
 *   "attn_split"   0 = choose the number of sequence splits of decode attention from the length,
 *                  1..128 = always use n (at most 64 apply to the single-row attention kernel, at most 128,
 *                  rounded up to a multiple of 4, to its matrix-core variant)
 *   "attn_mfma_min" context length from which a decoding step runs its attention on the matrix cores (models
 *                  with the append path only); 0 = never.  Default 1: measured faster than the single-row
 *                  attention kernel at every context length on the 8B shape. */
int asynclm_set_option(asynclm_ctx *ctx, const char *name, int32_t value);

/* Per-kernel-class GPU time of ONE decoding step (forced token), measured with HIP events around
 * every launch (graphs off for this step).  The step is a real step: the sequence grows by one.
 * names_out: receives a pointer to a static array of class names; ms_out[0..n_classes) receives the
 * summed milliseconds and launches_out[0..n_classes) the number of launches per class.
 * Returns the number of classes (>= 0) or a negative error.  Pass cap = capacity of the arrays. */
int asynclm_profile_step(asynclm_ctx *ctx, int32_t seq, int32_t forced_token, const char *const **names_out,
                         float *ms_out, int32_t *launches_out, int32_t cap);

/* Raw time stamps.  After a decoding step that ran on two streams ("pipeline"): n_workgroups = 2 and, for kernel k
 * of the step (per layer: QKV, attention, O, gate/up, down; then the output head), out_host[(3 k + j) * 2 + w] is the
 * 100 MHz device clock at j = 0 kernel start, 1 hand-over from the previous kernel seen, 2 done, of w = 0 the first
 * workgroup (done: the workgroup that finished first), w = 1 the last one (done: the one that finished last).
 * After a one-stream decoding step in stamp mode ("step_stamps"): the same layout with six kernels per layer (QKV,
 * attention, merge of its key splits, O, gate/up, down; then the output head) and j = 1 = input vector staged in LDS
 * (unused for the two attention kernels).
 * Otherwise, of the last asynclm_profile_step that ran as the fused kernel: out_host[i * n_workgroups + w]
 * is the 100 MHz device clock of workgroup w at phase boundary i (per layer: end of QKV, barrier passed, end of
 * attention, barrier, end of merge, barrier, end of O, barrier, end of gate/up, barrier, end of down, barrier;
 * stamp 0 is the first barrier, the last two are the output head and its barrier).  Call with out_host = NULL
 * to get the sizes; cap is the capacity of out_host in elements. */
int asynclm_profile_trace(asynclm_ctx *ctx, uint64_t *out_host, int32_t cap, int32_t *n_stamps, int32_t *n_workgroups);

/* Text for an error code; never NULL. */
const char *asynclm_strerror(int code);

/* Library version, e.g. "0.1.0". */
const char *asynclm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ASYNCLM_H */
