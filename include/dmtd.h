/*
 * dmtd.h - C ABI of the MI355X (gfx950) decode path for Direct Multi-Token Decoding.
 *
 * The library runs cycle-based greedy decoding of a Qwen3-style decoder-only
 * transformer: each cycle starts with one pass through all layers and continues with
 * tau-1 passes through only the last n_late ("decoding") layers; the tokens that
 * skipped the front (encoding + thinking) layers have their front-layer KV entries
 * refilled by the next cycle's full pass (paper Sec. 2.2, Fig. 3; Eq. 4 for what the
 * late layers read; Eq. 5 for the LM head; Eq. 7 for the layer count per token).
 *
 * Conventions
 *  - Every pointer is labelled HOST or DEVICE.  The library never allocates or frees
 *    device memory: the weight blob and the workspace are the caller's, and must stay
 *    valid and unmodified by others until dmtd_destroy.  Host buffers are borrowed
 *    only for the duration of a call.
 *  - All work is enqueued on the one HIP stream given at creation; calls that return
 *    host data synchronise that stream before returning.  A context is not thread-safe.
 *  - Every call returns 0 (DMTD_OK) or a negative code.  Arguments and state are checked
 *    before anything is enqueued: a call that fails with DMTD_EINVAL, DMTD_ESTATE or
 *    DMTD_ECAPACITY leaves the context's state unchanged, on the host and on the device.
 *    After DMTD_EHIP (a launch, capture or copy failed midway) the host-side state and the
 *    device's position counters are those before the call, but token-history and cache
 *    entries written by steps that did complete remain (forced input tokens included):
 *    repeating the same call gives what it would have given without the failure; before
 *    any other use call dmtd_reset.  dmtd_last_error gives a message for the last failure.
 *  - A batch of sequences shares one cycle phase (and, unless dmtd_prefill_ragged is used, one prompt length),
 *    except through dmtd_decode_per_seq.
 *  - Positions are 0-based absolute token positions.
 *
 * Weight blob (DEVICE, element type per config.dtype, matrices row-major [out, in],
 * tensors contiguous in this order): token table [vocab, hidden]; for each layer
 * attn_norm[hidden], q[n_q_heads*head_dim, hidden], k[n_kv_heads*head_dim, hidden],
 * v[n_kv_heads*head_dim, hidden], q_norm[head_dim], k_norm[head_dim],
 * o[hidden, n_q_heads*head_dim], mlp_norm[hidden], gate[intermediate, hidden],
 * up[intermediate, hidden], down[hidden, intermediate]; final_norm[hidden];
 * lm_head[vocab, hidden] only when tied_embeddings == 0.
 */
#ifndef DMTD_H
#define DMTD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DMTD_OK          0
#define DMTD_EINVAL     -1   /* null pointer, bad shape, tau < 1, n_late outside [1, L], token id >= vocab, batch mismatch */
#define DMTD_ESTATE     -2   /* decode/logits before prefill; prefill twice without reset; n_late changed while tokens await refill */
#define DMTD_ECAPACITY  -3   /* sequence would exceed max_seq_len; workspace or output buffer too small */
#define DMTD_EHIP       -4   /* HIP runtime failure (message in dmtd_last_error) */

#define DMTD_DTYPE_F32   0
#define DMTD_DTYPE_BF16  1

typedef struct dmtd_ctx dmtd_ctx;   /* opaque host object owned by the library */

typedef struct dmtd_config {
  int32_t n_layers;            /* L */
  int32_t hidden;              /* d, multiple of 8 */
  int32_t n_q_heads;           /* multiple of n_kv_heads */
  int32_t n_kv_heads;
  int32_t head_dim;            /* 64 or 128 */
  int32_t intermediate;        /* SwiGLU width, multiple of 8 */
  int32_t vocab;
  float   rms_eps;
  float   rope_theta;
  int32_t tied_embeddings;     /* 1: the LM head is the token table */
  int32_t dtype;               /* DMTD_DTYPE_*: storage type of weights and KV cache */
  int32_t max_batch;
  int32_t max_seq_len;         /* prompt + generated tokens per sequence */
  int32_t full_pos_add_embed;  /* 0: late layers read the front output at full positions (tau=1 is ordinary
                                  decoding); 1: literal Eq. 4, h_emb + h_think at full positions */
  int32_t use_graphs;          /* 1: each decode step is replayed from a captured hipGraph */
  int32_t dry_run;             /* 1: no device work at all; only the cycle scheduler runs (host tests) */
  void*   stream;              /* hipStream_t; NULL = the default stream */
} dmtd_config;

/* Bytes of DEVICE workspace dmtd_create needs for this configuration (KV caches of all
 * layers, activations, logits, attention partials, token history, counters).
 * Returns 0 if the configuration is invalid. */
size_t dmtd_workspace_bytes(const dmtd_config* cfg);

/* Create a context.  weights_dev: DEVICE weight blob of weights_bytes bytes (layout
 * above), 16-byte aligned.  workspace_dev: DEVICE, 256-byte aligned, at least
 * dmtd_workspace_bytes(cfg).  With cfg->dry_run both may be NULL.  On success *out
 * receives the context.  Errors: DMTD_EINVAL (shape, size or alignment), DMTD_ECAPACITY
 * (workspace too small), DMTD_EHIP. */
int dmtd_create(const dmtd_config* cfg, const void* weights_dev, size_t weights_bytes,
                void* workspace_dev, size_t workspace_bytes, dmtd_ctx** out);

/* Prefill (Sec. 2.2): all prompt tokens of every sequence pass through all layers,
 * filling every layer's KV cache for positions 0..prompt_len-1; the last position's
 * logits give the first generated token, which is the first token of cycle 1.
 * tokens: HOST int32 [batch, prompt_len] row-major.  first_tokens: HOST int32 [batch],
 * may be NULL.  n_late is used only under full_pos_add_embed (the embedding is added
 * again where the late layers start); pass 0 otherwise.
 * Errors: DMTD_EINVAL, DMTD_ESTATE (already prefilled), DMTD_ECAPACITY. */
int dmtd_prefill(dmtd_ctx* ctx, const int32_t* tokens, int32_t batch, int32_t prompt_len,
                 int32_t n_late, int32_t* first_tokens);

/* Prefill for prompts of different lengths (the paper's speed test uses one static length, Sec. 3.4; this is the batch
 * of its evaluation runs).  tokens: HOST int32 [batch, prompt_len] row-major, sequence b's prompt in its first lengths[b]
 * entries (the rest is ignored); lengths: HOST int32 [batch], each in [1, prompt_len], the largest equal to prompt_len.
 * Every sequence's first generated token comes from its own last prompt position, cycles are anchored at the end of
 * each sequence's own prompt, and all sequences then decode in lockstep (same phase): sequence b's positions trail the
 * longest sequence's by prompt_len - lengths[b].  dmtd_get_state and max_seq_len refer to the longest sequence;
 * dmtd_read_kv rows of sequence b are valid up to its own length.  Errors as dmtd_prefill. */
int dmtd_prefill_ragged(dmtd_ctx* ctx, const int32_t* tokens, int32_t batch, int32_t prompt_len, const int32_t* lengths,
                        int32_t n_late, int32_t* first_tokens);

/* Run decode steps of cycle length tau with n_late late layers (Sec. 2.2).  If the
 * current cycle is complete (tau tokens emitted, counting the token prefill emitted
 * for cycle 1) the call starts a new cycle with a full step: the pending in-cycle
 * tokens and the newest token pass through the first L - n_late layers together
 * (refilling those layers' KV), and only the newest continues through the late
 * layers.  It then runs late-only steps (the newest token's embedding is the late
 * layers' input, Eq. 4) until the cycle has tau tokens or max_new steps have run in
 * this call (max_new <= 0: no cap).  So the first call after prefill emits tau-1
 * tokens and later calls emit tau; tau = 1 is ordinary decoding.
 * forced_inputs: HOST int32 [batch, n_forced] or NULL.  Step i of this call (i <
 * n_forced) consumes forced_inputs[b, i] as its input token instead of the previous
 * step's argmax (teacher forcing); out_tokens still reports every step's argmax.
 * out_tokens: HOST int32 [batch, out_stride], step i of sequence b at b*out_stride+i;
 * out_stride must be >= the number of steps the call runs (at most tau).
 * n_emitted: HOST, receives the number of steps run.
 * Errors: DMTD_EINVAL, DMTD_ESTATE (no prefill; n_late changed while tokens await
 * refill), DMTD_ECAPACITY (max_seq_len, out_stride). */
int dmtd_decode_cycle(dmtd_ctx* ctx, int32_t tau, int32_t n_late, int32_t max_new,
                      const int32_t* forced_inputs, int32_t n_forced,
                      int32_t* out_tokens, int32_t out_stride, int32_t* n_emitted);

/* Cycles back to back (Sec. 2.2): exactly n_steps decode steps (1 <= n_steps <= 64), with the
 * same steps, in the same order and with the same results as repeated dmtd_decode_cycle calls
 * with max_new = the steps still to run - a full step wherever a cycle of tau tokens is
 * complete, late-only steps otherwise - but enqueued as one piece of GPU work: the tokens are
 * selected on the device, so the host is not needed between cycles and synchronises once, at
 * the end of the call (a decode loop that looks at its tokens every few cycles only).  The call
 * may end inside a cycle; the next call, of either kind, continues it.
 * forced_inputs, out_tokens, out_stride (>= n_steps), n_emitted: as for dmtd_decode_cycle.
 * Nothing runs unless all n_steps steps fit (all-or-nothing).
 * Errors: as dmtd_decode_cycle; DMTD_EINVAL for n_steps outside [1, 64]. */
int dmtd_decode(dmtd_ctx* ctx, int32_t tau, int32_t n_late, int32_t n_steps,
                const int32_t* forced_inputs, int32_t n_forced,
                int32_t* out_tokens, int32_t out_stride, int32_t* n_emitted);

/* Cycles per sequence (Sec. 2.2 applied to each sequence of a batch on its own; the evaluation of Sec. 3.7 varies the cycle
 * length at inference): exactly n_steps decode steps (1 <= n_steps <= 64) in which sequence b decodes in cycles of tau[b]
 * tokens, so the sequences of one batch may be at different points of their cycles - a sequence starts a new cycle (its
 * pending tokens and its newest token pass the front layers, refilling its own front-layer KV entries) at the step after
 * its own cycle is complete, whatever the others do.  In such a step the sequences that start a cycle pass the front layers
 * (one weight pass per distinct number of pending rows among them), and ALL sequences' newest tokens then share one pass
 * through the late layers and the LM head.  tau: HOST int32 [batch], each in [1, 64]; the lengths may change from call to
 * call (a sequence whose cycle already holds tau[b] or more tokens starts a new one at the call's first step).
 * forced_inputs, out_tokens, out_stride (>= n_steps), n_emitted: as for dmtd_decode.  All-or-nothing like dmtd_decode.
 * While the sequences differ in phase or in pending tokens, dmtd_decode_cycle, dmtd_decode and dmtd_decode_cycle_noalloc
 * return DMTD_ESTATE, dmtd_get_state reports sequence 0 (its counters[] follow sequence 0's schedule) and
 * dmtd_get_seq_state any sequence; once they agree again the other calls work as before.  Not available in the ExDy
 * variant (DMTD_ESTATE).
 * Errors: DMTD_EINVAL, DMTD_ESTATE (no prefill; ExDy; n_late changed while tokens await refill), DMTD_ECAPACITY
 * (max_seq_len, out_stride, more than 16 pending rows for a sequence), DMTD_EHIP. */
int dmtd_decode_per_seq(dmtd_ctx* ctx, const int32_t* tau, int32_t n_late, int32_t n_steps,
                        const int32_t* forced_inputs, int32_t n_forced,
                        int32_t* out_tokens, int32_t out_stride, int32_t* n_emitted);

/* Scheduler state of sequence b after dmtd_decode_per_seq: n_front (in the coordinates of dmtd_get_state's n_tok, i.e.
 * n_tok - n_front of its tokens await refill) and phase (tokens of its current cycle already emitted).  Either pointer may
 * be NULL.  Errors: DMTD_EINVAL (b outside the batch). */
int dmtd_get_seq_state(const dmtd_ctx* ctx, int32_t b, int32_t* n_front, int32_t* phase);

/* dmtd_decode_cycle for callers that cannot allocate or synchronise: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same steps, same kernels and same results as dmtd_decode_cycle, with these differences:
 *  - forced_inputs_dev and out_tokens_dev are DEVICE buffers (int32 [batch, n_forced] and [batch, out_stride], row-major;
 *    forced_inputs_dev may be NULL); nothing is copied to or from the host.  Forced ids outside the vocabulary cannot be
 *    seen by the host and are clamped into it on the device.
 *  - the call allocates nothing (no hipMalloc / hipFree, no graph instantiation, no staging copies) and does not
 *    synchronise: it enqueues the steps' kernels on the context's stream, one by one (use_graphs is ignored), and returns;
 *    out_tokens_dev and dmtd_logits are valid once the stream has reached the end of that work.
 *  - the steps' partial results (attention key ranges, selection keys of the LM head, K-split sums of the tiled
 *    projection kernel) live in a 16 MiB array the library holds on each GPU it runs on, not in the workspace.  A call
 *    whose partial results need more (they grow with batch x refill rows per sequence; a 4B-shaped model at batch 1 and
 *    tau <= 4 needs 4.1 MiB) is refused with DMTD_ECAPACITY before anything runs.  All contexts on one GPU share the
 *    array: two such calls whose GPU work overlaps on one GPU race; calls ordered on one stream do not.
 * n_emitted: HOST, the number of steps enqueued (at most tau).  The host-side state (dmtd_get_state) advances at once.
 * After DMTD_EHIP (a launch failed) the device state is undefined: call dmtd_reset.
 * Errors: as dmtd_decode_cycle, plus DMTD_ECAPACITY for the scratch limit. */
int dmtd_decode_cycle_noalloc(dmtd_ctx* ctx, int32_t tau, int32_t n_late, int32_t max_new,
                              const int32_t* forced_inputs_dev, int32_t n_forced,
                              int32_t* out_tokens_dev, int32_t out_stride, int32_t* n_emitted);

/* Copy the logits (Eq. 5) of the most recent step: HOST float32 [batch, vocab],
 * out_elems >= batch * vocab.  Errors: DMTD_ESTATE before prefill, DMTD_ECAPACITY. */
int dmtd_logits(dmtd_ctx* ctx, float* out, size_t out_elems);

/* Scheduler state (Sec. 2.2).  n_tok: tokens that have entered the late layers' caches; n_front:
 * tokens in the front layers' caches (n_tok - n_front await refill); phase: tokens of
 * the current cycle already emitted; counters[4] (HOST int64): layers traversed by
 * token-emitting rows, layers traversed by refill rows, tokens emitted by decode
 * steps, decode steps that were full steps.  counters[0] / (counters[2] * n_layers) is the
 * percentage of layers per token of Eq. 7 (over whole cycles: (L + (tau-1) L_d) / (tau L));
 * counters[0] + counters[1] is the total load, that of ordinary decoding once every token is
 * refilled (Sec. 2.2).  Any pointer may be NULL. */
int dmtd_get_state(const dmtd_ctx* ctx, int32_t* n_tok, int32_t* n_front, int32_t* phase,
                   int64_t* counters);

/* Schedule trace since the last reset, in the form of the walk-through of Fig. 3 (which tokens pass which layer group in
 * which forward pass): one record of 4 int32 per (pass, layer group):
 * pass number (1 = prefill), group (0 = front layers; with n_early > 0: the thinking layers, 1 = late layers, 2 = encoding layers of the ExDy variant), first
 * position, number of consecutive positions.  buf: HOST, cap_records records.
 * n_records receives the total number available (which may exceed cap_records). */
int dmtd_get_trace(const dmtd_ctx* ctx, int32_t* buf, int32_t cap_records, int32_t* n_records);

/* Copy one layer's KV cache rows for positions [0, n_pos) of sequence b to the host as
 * float32 [2 (K,V), n_kv_heads, n_pos, head_dim] (for cache-indexing tests). */
int dmtd_read_kv(dmtd_ctx* ctx, int32_t layer, int32_t b, int32_t n_pos, float* out, size_t out_elems);

/* Measurement aid: launch one kernel kind of the decode path back to back, once per layer
 * (the LM head: once per repetition), reps times over, with `rows` activation rows, on the
 * context's stream between two HIP events, and return the average duration of one launch
 * in microseconds.  Activations are whatever the workspace holds; caches, token history and
 * scheduler state are not modified (the residual stream scratch is).  kind: DMTD_K_*.
 * Needs a prefilled context (attention reads the current context length).
 * Errors: DMTD_EINVAL (kind, rows outside [1, 16] for attention (rows per sequence) or [1, 16 * max_batch] for the projections (total rows), reps < 1), DMTD_ESTATE, DMTD_EHIP. */
#define DMTD_K_QKV     0   /* RMSNorm + fused QKV projection (Sec. 3.1 model; hot-path step a2) */
#define DMTD_K_OPROJ   1   /* O projection + residual */
#define DMTD_K_GATEUP  2   /* RMSNorm + gate/up projections + SwiGLU */
#define DMTD_K_DOWN    3   /* down projection + residual */
#define DMTD_K_LMHEAD  4   /* final RMSNorm + LM head (Eq. 5) + argmax partials */
#define DMTD_K_ATTN    5   /* split-K GQA decode attention over the current context */
/* Kinds that only read: one launch per layer of a kernel that streams exactly the weight bytes of that projection
 * (as stored) and does nothing else; `rows` is ignored (pass 1).  bf16 models only (DMTD_EINVAL otherwise).  What a
 * plain read of the same bytes costs on the chip, to set beside the kernel that does the work. */
#define DMTD_K_READ_QKV    6
#define DMTD_K_READ_OPROJ  7
#define DMTD_K_READ_GATEUP 8
#define DMTD_K_READ_DOWN   9
int dmtd_time_kernel(dmtd_ctx* ctx, int32_t kind, int32_t rows, int32_t reps, float* avg_us);

/* ExDy variant (Sec. 2.1, the paragraph before Eq. 5; layer allocations of Sec. 3.3): the in-cycle tokens
 * reuse the first n_early (encoding) layers as well as the last n_late (decoding) layers, i.e. h_masked is built
 * from h_enc instead of h_emb.  A late-only step then runs layers [0, n_early) and [L - n_late, L) on its token
 * and keeps the encoding output; the next full step refills only the thinking layers [n_early, L - n_late) from
 * the stored outputs.  n_early = 0 (the default) is the plain method; the setting survives dmtd_reset.
 * Allowed before prefill or whenever no token awaits refill (under the literal Eq. 4 reading only before prefill).
 * dmtd_decode_cycle then requires n_early + n_late <= n_layers (DMTD_EINVAL).
 * Errors: DMTD_EINVAL (n_early outside [0, n_layers - 1]), DMTD_ESTATE. */
int dmtd_set_n_early(dmtd_ctx* ctx, int32_t n_early);

/* Token selection.  The paper generates without post-verification and names no sampling rule (Sec. 3.2); greedy
 * selection is the default here.  With temperature > 0 every later prefill and decode step draws its token from
 * softmax(z / temperature) restricted to the top_k largest logits (top_k = 0: no restriction; logits equal to the
 * k-th largest all stay in; top_k = 1 or temperature <= 0: greedy).  The draw for the row at position p of sequence
 * b is argmax_v z_v / temperature - log(-log(u_v)) (Gumbel-max), u_v = (m + 0.5) / 2^23 with m the top 23 bits of a
 * counter-based SplitMix64 value keyed by (seed, b * 2^32 + p, v): it does not depend on batch order, graph replay
 * or earlier draws.  dmtd_logits still returns the unperturbed logits; the setting survives dmtd_reset.
 * Errors: DMTD_EINVAL (temperature not finite, top_k < 0), DMTD_EHIP. */
int dmtd_set_sampling(dmtd_ctx* ctx, float temperature, int32_t top_k, uint64_t seed);

/* Whole-sequence masked forward (Sec. 2.1, Eqs. 1-5) and next-token loss (Eq. 6): the form the method is trained in, and
 * a teacher-forced scorer.  Every position of every sequence passes the encoding and thinking layers (the first
 * n_layers - n_late layers); the decoding layers read, at position i, the thinking output where mask[i] != 0 (a full
 * position) and the raw token embedding elsewhere (Eq. 4; with n_early > 0 the encoding layers' output; with
 * full_pos_add_embed the literal sum); the LM head (Eq. 5) follows at every position.  With
 * mask[i] = (i mod tau == 0) this is Eq. 3; with the mask cycle decoding realises (all prompt positions, then every
 * tau-th) the logits equal those of dmtd_prefill + teacher-forced dmtd_decode_cycle at the same positions.
 * tokens: HOST int32 [batch, n] row-major.  mask: HOST uint8 [n], shared by the sequences.
 * nll: HOST float32 [batch, n] or NULL: nll[b, i] = CrossEntropy(z_i, tokens[b, i+1]) for i < n-1, 0 for i = n-1.
 * best: HOST int32 [batch, n] or NULL: argmax of z_i (lowest index among equal maxima).
 * logits: HOST float32 [batch, n, vocab] or NULL (logits_elems >= batch*n*vocab): every position's logits.
 * loss: HOST float32 [batch] or NULL: Eq. 6, the mean of nll[b, 0..n-2].
 * Needs an empty context (fresh or reset) and n <= max_seq_len; uses the KV caches as scratch and leaves the context empty.
 * Errors: DMTD_EINVAL, DMTD_ESTATE (context holds a sequence; dry run), DMTD_ECAPACITY, DMTD_EHIP. */
int dmtd_masked_forward(dmtd_ctx* ctx, const int32_t* tokens, int32_t batch, int32_t n, const uint8_t* mask, int32_t n_late,
                        float* nll, int32_t* best, float* logits, size_t logits_elems, float* loss);

/* Back to the state right after dmtd_create (caches are treated as empty). */
int dmtd_reset(dmtd_ctx* ctx);

void dmtd_destroy(dmtd_ctx* ctx);

/* Message for the last failed call on ctx (or, with ctx == NULL, the last failed
 * dmtd_create on this thread).  Never NULL. */
const char* dmtd_last_error(const dmtd_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* DMTD_H */
