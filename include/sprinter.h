/*
 * sprinter.h - C ABI of the batched SPRINTER decode step for one MI355X (gfx950).
 *
 * SPRINTER ("Speeding up Speculative Decoding via Sequential Approximate
 * Verification", Sec. 3 "Algorithm", Alg. 1; detailed listing: Alg. 2 in the
 * appendix "Full SPRINTER Algorithm") decodes with three models: a small draft
 * LM M_q, a large target LM M_p and a tiny verifier classifier V.  Per token the
 * draft samples x ~ q(.|prefix); the verifier scores a latent feature of the
 * draft; if the score clears the threshold tau the token is kept, otherwise the
 * target is run once for that position and its sample replaces the draft token
 * (Fig. 2(a)).  This library runs that loop for B independent rows in lock step:
 *
 *   draft single-token forward (B rows) -> fused LM head + Gumbel-max sample
 *   -> verifier MLP + sigmoid + threshold -> stable compaction of rejected rows
 *   -> target single-token forward on the R rejected rows -> LM head + sample
 *   -> scatter the replacements back, advance per-row state.
 *
 * Everything is enqueued on the caller's HIP stream and all decisions are taken
 * on the device.  The host learns one number per step, the count R of rejected
 * rows: the calling thread waits a few microseconds inside sprinter_step (it
 * polls a pinned host word the decide kernel writes) and then launches the
 * target pass for exactly R rows, or none.  A step can therefore not be
 * recorded into a HIP graph, and one thread drives a context at a time.
 * sprinter_prefill drains the stream every 4 passes; sprinter_get_stats and
 * sprinter_destroy wait for it.  The library never allocates device memory: the
 * caller hands over one workspace.  sprinter_create allocates 256 bytes of
 * pinned host memory (that polled word), freed by sprinter_destroy.
 *
 * Conventions
 *   - "dev" pointers are device memory, "host" pointers host memory.
 *   - every call returns 0 (SPRINTER_OK) or a negative SPRINTER_E_* code; the
 *     text of the last error is available from sprinter_last_error().  A call
 *     that fails validation enqueues no device work.
 *   - matrices are row-major [out, in] ("y = W x"), in the element type chosen
 *     by sprinter_cfg.dtype; every 1-D parameter (bias, norm gain/offset) and
 *     the whole verifier are float32.
 *   - arithmetic of SPRINTER_BF16: weights and both KV caches hold bfloat16
 *     values; the matrix products take float16 operands - the weights converted
 *     once when they are packed (exact above 2^-14, rounded to the float16
 *     subnormal grid below), the activations rounded to float16 (11 significant
 *     bits; magnitudes above 65504 become infinities) - and accumulate in
 *     float32; the residual stream, projections, attention scores and logits
 *     are float32.  SPRINTER_F32: float32 throughout.
 */
#ifndef SPRINTER_H
#define SPRINTER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  SPRINTER_OK = 0,
  SPRINTER_E_NULL = -1,      /* a required pointer is NULL */
  SPRINTER_E_CONFIG = -2,    /* unsupported or inconsistent configuration */
  SPRINTER_E_WORKSPACE = -3, /* workspace too small or misaligned */
  SPRINTER_E_WEIGHTS = -4,   /* unknown name, wrong shape, or weights missing */
  SPRINTER_E_RANGE = -5,     /* batch / length outside the configured maxima */
  SPRINTER_E_STATE = -6,     /* call order violated (e.g. generate before prefill) */
  SPRINTER_E_HIP = -7        /* a HIP runtime call failed */
};

enum { SPRINTER_ARCH_GPT = 0, SPRINTER_ARCH_LLAMA = 1 };
enum { SPRINTER_F32 = 0, SPRINTER_BF16 = 1 };
enum { SPRINTER_DRAFT = 0, SPRINTER_TARGET = 1, SPRINTER_VERIFIER = 2 };

/* One decoder-only transformer.
 *   arch 0 (GPT family)  : pre-LN LayerNorm, biases on all linear maps, tanh-GELU
 *                          two-matrix FFN, learned absolute positions, LM head tied
 *                          to the token embedding.
 *   arch 1 (LLaMA family): RMSNorm, no biases, rotary positions on pairs
 *                          (i, i + d_head/2), SwiGLU three-matrix FFN, grouped-query
 *                          attention (n_kv_head divides n_head), separate LM head.
 * d_head = d_model / n_head must be 64 or 128; d_model and d_ff multiples of 8. */
typedef struct {
  int32_t arch, n_layer, d_model, n_head, n_kv_head, d_ff, vocab, max_pos;
  float norm_eps, rope_theta;
} sprinter_model_cfg;

/* The triple (M_q, M_p, V) and the sampling parameters (inputs of Alg. 1/2:
 * "M_p, M_q, V, Prefix, prediction threshold tau").
 *   ver_d_hidden  0: V = sigmoid(w2 . hf + b2), the single layer of Sec. 3.2;
 *                >0: V = sigmoid(w2 . relu(W1 hf + b1) + b2).
 *   hf is the draft's final hidden state after the last norm (the LM-head input).
 *   accept <=> V >= tau (the comparison of Alg. 2), taken in float32.
 *   temperature 0 selects greedy decoding; otherwise tokens are drawn by
 *   Gumbel-max with Philox4x32-10 noise keyed by (seed; vocab index, position,
 *   row, stream), so a run is reproducible from (seed, prompts) alone.
 *   target_ctx_mode 0 (own history): the target's cache holds the prompt plus
 *   one entry per earlier target call of that row (each with its true position
 *   id), so a target call is a single-token forward (the cost model of
 *   Sec. 3.1(c)).  target_ctx_mode 1 (full prefix): before it scores the
 *   rejected position the target first consumes every committed token of that
 *   row it has not seen, so its distribution is conditioned on the whole
 *   prefix (Sec. 2, Alg. 2 "Run M_p Once" on Prefix); a rejected row then
 *   brings one work-list entry per unseen token and the target pass runs over
 *   the list in chunks of at most max_batch (rounded up) entries.  In this
 *   mode sprinter_step does not produce target_logits / target_hidden (they
 *   must be NULL).  Other values are rejected.
 *   reject_mode 0 (replace): on a rejection the target's sample replaces the
 *   draft token (Fig. 2(a)).  reject_mode 1 (p/q correction, Sec. 2 Eq. (1)
 *   and the coin of Alg. 2): the draft token x is kept with probability
 *   min(1, p(x)/q(x)) (coin: Philox stream 2 of the row and position),
 *   otherwise the token is drawn from the normalised residual max(0, p - q)
 *   (Gumbel-max with the target stream's noise); q and p are the softmax of
 *   logits / temperature, so temperature must be > 0.  A rejected position
 *   whose committed token equals its draft token was kept by the coin.
 *   sd_gamma > 0 reserves the buffers of sprinter_sd_generate (standard
 *   speculative decoding on the same models) for windows of up to sd_gamma
 *   draft tokens: two arrays of (sd_gamma + 1) * max_batch * vocab floats.
 *   0 <= sd_gamma <= 16.
 *   chunk_rows: rows of the activation buffers = entries one pass over the
 *   weights takes in a multi-entry forward (prefill, full-prefix work lists,
 *   speculative-decoding windows).  0 = default (bf16: 4096; float32: 16); else a
 *   multiple of 64 in [64, 4096].  Never below max_batch rounded up. */
typedef struct {
  sprinter_model_cfg draft, target;
  int32_t ver_d_in, ver_d_hidden;
  int32_t dtype;
  int32_t max_batch, max_seq;
  float tau, temperature;
  uint64_t seed;
  int32_t target_ctx_mode;
  int32_t reject_mode;
  int32_t sd_gamma;
  int32_t chunk_rows;
} sprinter_cfg;

/* Optional per-step outputs of sprinter_step; every field is a device pointer
 * or NULL.  B = batch of the last prefill, R = number of rejected rows.
 *   draft_tok[B]      token sampled from the draft (Alg. 2 "x ~ q_r")
 *   score[B]          verifier output in (0,1)
 *   accept[B]         1 iff score >= tau
 *   rej_idx[B]        first R entries: rejected rows in ascending order
 *   n_rej[1]          R
 *   committed_tok[B]  token appended to the row (draft token or target sample)
 *   draft_logits[B,V] draft_hidden[B,d_q]   float32, before noise / after last norm
 *   target_logits[B,V] target_hidden[B,d_p] rows 0..R-1 in rej_idx order */
typedef struct {
  int32_t* draft_tok;
  float* score;
  uint8_t* accept;
  int32_t* rej_idx;
  int32_t* n_rej;
  int32_t* committed_tok;
  float* draft_logits;
  float* draft_hidden;
  float* target_logits;
  float* target_hidden;
} sprinter_step_out;

/* Counters since the last prefill (the paper's "Avg Tokens" and the number of
 * target invocations follow from them). */
typedef struct {
  int64_t steps;              /* decode steps executed */
  int64_t steps_with_target;  /* steps in which at least one row was rejected */
  int64_t sum_rejected;       /* total target row-invocations = sum over steps of R */
  int32_t batch;
  int32_t coin_kept;          /* reject_mode 1: rejected positions whose draft token survived the p/q coin */
} sprinter_stats;

typedef struct sprinter_ctx sprinter_ctx;

/* Bytes of device workspace sprinter_create needs for cfg: everything the loop
 * of Alg. 2 keeps between tokens for the inputs "M_p, M_q, V, Prefix" (KV caches
 * of both models for max_batch x max_seq, the committed prefixes), tile-packed
 * weight copies and activations. */
int sprinter_workspace_bytes(const sprinter_cfg* cfg, size_t* out_bytes);

/* Creates a context for one triple (M_q, M_p, V) and threshold tau, the fixed
 * inputs of Alg. 1 / Alg. 2, on the current device.  dev_workspace (256-byte aligned, at
 * least sprinter_workspace_bytes) stays owned by the caller and must outlive the
 * context; hip_stream is a hipStream_t (NULL = the default stream) on which all
 * later work is enqueued.  The library allocates no device memory; create
 * allocates 256 bytes of pinned host memory (the word the host polls for the
 * number of rejected rows), freed by sprinter_destroy.  Errors: NULL pointers,
 * unsupported cfg (see field comments), workspace too small. */
int sprinter_create(const sprinter_cfg* cfg, void* dev_workspace, size_t workspace_bytes,
                    void* hip_stream, sprinter_ctx** out_ctx);

/* sprinter_create for callers that cannot allocate device memory at all (code that runs while a
 * HIP graph is being captured elsewhere in the process, tight serving loops, harnesses that forbid
 * hipMalloc): the workspace is a static array inside the library, SPRINTER_STATIC_WORKSPACE_BYTES
 * (64 MiB) on every GPU the library runs on, held until the process ends.  The call allocates
 * nothing, neither device nor pinned host memory, and neither do later calls on the context; a
 * context made here therefore learns the number of rejected rows through a small device-to-host copy
 * and a stream synchronisation per step instead of a polled pinned word (about 10 us more per step).
 * Weights, prompts and outputs are passed to the later calls as for any other context.
 * Errors: cfg whose sprinter_workspace_bytes exceeds the limit (SPRINTER_E_WORKSPACE, both sizes in
 * the message); a second context of this kind on a device while the first is alive
 * (SPRINTER_E_STATE): all such contexts of a device share that one array, so they must not overlap
 * - destroy one before creating the next.  The array keeps the previous context's contents; create
 * clears everything that has to start at zero. */
#define SPRINTER_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)
int sprinter_create_static(const sprinter_cfg* cfg, void* hip_stream, sprinter_ctx** out_ctx);

/* Hands over the parameters of one of the three models of Sec. 3 (draft M_q,
 * target M_p, verifier V of Sec. 3.2).  which: SPRINTER_DRAFT, _TARGET or
 * _VERIFIER.  names[i] / dev_ptrs[i] / shapes[4*i..4*i+3] (unused dims 0) describe
 * tensor i.  Names: "tok_emb" [V,d], "pos_emb" [max_pos,d] (GPT), "lm_head" [V,d]
 * (LLaMA), "normf.g" [d], "normf.b" [d] (GPT) and per layer i "l<i>.norm1.g",
 * "l<i>.norm1.b"*, "l<i>.wqkv" [(H+2KVH)d_h, d] (rows: Q heads, K heads, V heads),
 * "l<i>.bqkv"*, "l<i>.wo" [d, H d_h], "l<i>.bo"*, "l<i>.norm2.g", "l<i>.norm2.b"*,
 * GPT: "l<i>.w1" [ff,d], "l<i>.b1", "l<i>.w2" [d,ff], "l<i>.b2";
 * LLaMA: "l<i>.wg" [ff,d], "l<i>.wu" [ff,d], "l<i>.w2" [d,ff]   (* = GPT only).
 * Verifier: "v.w1" [h,d_in], "v.b1" [h] (h > 0 only), "v.w2" [h or d_in], "v.b2" [1].
 * In bf16 mode matrices are copied into a tile-packed layout inside the workspace
 * (enqueued on the stream; the originals may be freed once the stream has passed
 * this point), except the embedding tables, which are read in place; every other
 * tensor is BORROWED and must stay valid for the life of the context.  The call
 * fails if a name is unknown, a shape is wrong, a pointer is not 16-byte aligned,
 * or a tensor of the model is absent. */
int sprinter_load_weights(sprinter_ctx* ctx, int which, const char* const* names,
                          const void* const* dev_ptrs, const int64_t* shapes, int n);

/* Takes the "Prefix" input of Alg. 1 / Alg. 2 for B independent rows: resets
 * state and counters and fills both KV caches with
 * positions 0 .. P_b-2 of each prompt; the first decode step then feeds the last
 * prompt token at position P_b-1.  All (row, position) pairs go through both
 * models in row-major chunks of cfg.chunk_rows tokens per pass over the weights
 * (bf16: matrix-core GEMMs over the whole chunk and causal matrix-core attention
 * over each row's run of positions; float32: the vector kernels, 16 tokens per
 * pass by default).  The
 * stream is drained every 4 passes.  dev_prompt is [B, max_prompt] int32 (padding
 * is never read), host_prompt_len[B] has 1 <= P_b <= max_prompt.  Errors:
 * B > max_batch, P_b out of range, max_prompt > max_seq (or > max_pos), weights
 * not loaded. */
int sprinter_prefill(sprinter_ctx* ctx, const int32_t* dev_prompt, const int32_t* host_prompt_len,
                     int B, int max_prompt);

/* One iteration of the loop of Alg. 2 for every row: "q_r ~ M_q(Prefix)",
 * "x ~ q_r", the test "V(s(x, Prefix)) >= tau", and for the rows that fail it
 * "Run M_p Once" (the steps listed at the top).  out may be NULL.
 * Error if no prefill was done or a row would exceed max_seq / max_pos.
 * The calling thread waits inside the call (a few microseconds of polling on a
 * pinned word the decide kernel writes) until the device has counted the rejected
 * rows, then launches the target pass for exactly that many rows - or none.  The
 * rest of the step is only enqueued.  The call can therefore not be recorded into
 * a HIP graph, and two threads must not drive one context at the same time. */
int sprinter_step(sprinter_ctx* ctx, const sprinter_step_out* out);

/* The whole loop of Alg. 2 for a fixed number of tokens (the paper generates a
 * fixed count per prompt, Sec. 4; there is no end-of-sequence rule): Prefix + t
 * for t = 1 .. n_tokens.  n_tokens decode steps back to back (each with the short wait described at
 * sprinter_step; no stream synchronisation).  Outputs are [B, n_tokens] row-major
 * device arrays; any of them may be NULL: committed tokens, accept flags, verifier
 * scores, draft tokens.  The last step's tail is still running when the call returns. */
int sprinter_generate(sprinter_ctx* ctx, int n_tokens, int32_t* dev_out_tok, uint8_t* dev_out_accept,
                      float* dev_out_score, int32_t* dev_out_draft_tok);

/* Standard speculative decoding (Sec. 2 with Eq. (1)) on the same draft / target
 * pair: the method the paper's speed-ups are measured against.  One round, for
 * every row: the draft model generates gamma tokens one after the other; the
 * target model reads the last committed token and those gamma tokens in one pass
 * (gamma + 1 positions per row); the draft tokens are checked in order, x stays
 * with probability min(1, p(x)/q(x)), the first that does not is replaced by a
 * draw from norm(max(0, p - q)) and ends the window; if all stay, one more token
 * is drawn from the target's last distribution.  A round commits n_acc + 1 tokens
 * of a row, 0 <= n_acc <= gamma.  Random numbers: as in the decode step, keyed by
 * (row, sequence position): draft stream for the window, coin stream for the
 * test, target stream for the residual draw and the extra token.  The verifier
 * is not used.
 * Runs n_rounds rounds.  Outputs (device pointers, each may be NULL):
 *   dev_out_tok [B, tok_stride]   tokens committed by this call, in order;
 *                                 tok_stride >= n_rounds * (gamma + 1)
 *   dev_out_n_tok [B]             how many of them per row
 *   dev_out_n_acc [B, n_rounds]   draft tokens kept per round
 *   dev_out_draft [B, n_rounds, gamma]  every drafted token
 * Needs cfg.sd_gamma >= gamma >= 1 and temperature > 0.  Between two prefills a
 * context runs either decode steps or rounds of this call, not both (error
 * otherwise).  Error if max_prompt + (rounds so far + n_rounds) * (gamma + 1)
 * would exceed max_seq.  The calling thread waits once per round (polling a
 * pinned word, as in sprinter_step) for the size of the next draft pass: after a
 * fully kept window the draft model has one more token to read than otherwise.
 * sprinter_get_stats then counts rounds as steps, rows whose window was cut as
 * sum_rejected and kept draft tokens as coin_kept. */
int sprinter_sd_generate(sprinter_ctx* ctx, int gamma, int n_rounds, int32_t* dev_out_tok, int tok_stride,
                         int32_t* dev_out_n_tok, int32_t* dev_out_n_acc, int32_t* dev_out_draft);

/* Replaces the prediction threshold tau of Alg. 1 / Alg. 2 (the operating point on the
 * verifier's ROC curve, Sec. 3.2); takes effect for steps enqueued afterwards. */
int sprinter_set_tau(sprinter_ctx* ctx, float tau);

/* Waits for the stream and copies the counters to the host: the quantities behind
 * Table 2's "Avg Tokens" (generated tokens per target call) and the cost model of
 * Sec. 3.1(c) (number of target runs).
 * host_target_calls, if not NULL, receives the per-row number of target calls [B]. */
int sprinter_get_stats(sprinter_ctx* ctx, sprinter_stats* host_out, int64_t* host_target_calls);

/* Waits for the stream, frees the context and its pinned word; the workspace stays with the caller. */
void sprinter_destroy(sprinter_ctx* ctx);

/* Text of the last error on ctx (or of the last failed sprinter_create /
 * sprinter_workspace_bytes in this thread when ctx is NULL).  Never NULL. */
const char* sprinter_last_error(const sprinter_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* SPRINTER_H */
