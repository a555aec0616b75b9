// Internal declarations shared by the C-ABI layer (abi.cpp) and the kernel
// launchers (k_*.hip).  Nothing here is part of the public interface.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace sprinter {

// ---- activation / weight tile geometry (bf16 mode) -------------------------
// A GEMM operand tile is what one v_mfma_f32_16x16x32_bf16 consumes from one
// side: 16 rows x 32 k-values = 64 lanes x 8 bf16 = 1 KiB, stored lane-major so
// that a wavefront fetches it with one fully coalesced 16-byte-per-lane load:
//   element (row r, k) of tile -> lane = ((k % 32) / 8) * 16 + (r % 16), slot k % 8.
// Tiles are ordered [row_tile][k_tile].  Weight matrices are repacked into this
// layout once at load time; activations that feed a GEMM are produced in it.
static inline __host__ __device__ int round_up(int x, int m) { return (x + m - 1) / m * m; }

struct RowDesc {       // which rows a model forward works on (all device memory)
  const int* n_rows;   // [1] number of active rows M (<= launch-time maximum)
  const int* b;        // [M] batch row of each active row (KV cache owner, RNG row)
  const int* tok;      // [M] input token
  const int* pos;      // [M] position id of the input token
  const int* slot;     // [M] KV-cache slot the new entry is written to (= entries already cached)
};

struct LayerW {
  const float *n1g, *n1b, *bqkv, *bo, *n2g, *n2b, *b1, *b2;
  const void *wqkv, *wo, *w1, *wg, *wu, *w2;   // dtype matrices (bf16: tile-packed)
};

struct ModelDims {
  int arch, n_layer, d, H, KVH, dh, ff, V, max_pos, dqkv;
  float eps, theta;
};

constexpr int PART_SHARES = 8;   // most K shares launch_gemm_part may use
struct ModelScratch {  // per-model activation buffers, sized for max_batch rows
  float* h;            // [M, d] residual stream, float32
  void* xn;            // [M, d] normalised GEMM input (activation layout)
  float* y;            // [M, dqkv] QKV projection output, float32
  void* ao;            // [M, H*dh] attention output (activation layout)
  void* mid;           // [M, ff] FFN hidden (activation layout)
  float* hf;           // [M, d] final hidden state after the last norm, float32
  void* hfn;           // same values in activation layout (LM-head input)
  float* rope;         // [M, dh/2, 2] cos/sin of the row's position
  float* part;         // [PART_SHARES][M, d] partial O-proj / FFN-down products (bf16 mode), float32
  unsigned long long* am_part;  // [n_lm_wg, Mpad] packed (value, index) arg-max partials
  int n_lm_wg;
};

struct SamplerArgs {
  unsigned seed_lo, seed_hi, stream;
  float inv_temperature;   // 0 = greedy (no noise)
};

// ---- launchers (k_*.hip) ---------------------------------------------------
void launch_pack_bf16(const void* w, void* out, int N, int K, hipStream_t s);
void launch_fill_zero(void* p, size_t bytes, hipStream_t s);

void launch_embed(int dtype, const ModelDims& md, const void* tok_emb, const void* pos_emb,
                  const RowDesc& rd, float* h, float* rope, int max_rows, hipStream_t s);
// An update of the residual stream that is still in pieces (launch_gemm_part): the norm kernel adds
// bias + share 0 + share 1 + ... to the row, writes the row back and normalises the sum.
struct NormPending {
  const float* part; size_t stride; int shares; const float* bias;
};
// pend is honoured by the bf16 kernel only (d a multiple of 8, at most 8192): see norm_takes_pending().
void launch_norm(int dtype, int arch, const float* h, const float* g, const float* b, float eps, int d,
                 const int* n_rows, void* act_out, float* f32_out, int max_rows, hipStream_t s,
                 const NormPending* pend = nullptr);
inline bool norm_takes_pending(int dtype, int d) { return dtype == 1 && d % 8 == 0 && d <= 8192; }
// bf16: part[s] = X[:, K share s] W[:, K share s]^T for s < returned share count (<= max_shares)
int launch_gemm_part(const void* W, const void* X, size_t x_elems, const int* n_rows, int N, int K, float* part,
                     size_t part_stride, int max_shares, int max_rows, hipStream_t s);

enum { EPI_F32 = 0, EPI_RESID = 1, EPI_GELU = 2, EPI_SWIGLU = 3, EPI_PART = 4 /* partial product of one K share */ };
// Y[M,N] = X[M,K] W[N,K]^T (+bias) with epilogue; X in activation layout, W in weight layout.
// x_elems: elements the activation buffer X holds (its row tiles bound what a kernel may fetch).
void launch_gemm(int dtype, int epi, const void* W, const void* W2, const void* X, size_t x_elems,
                 const int* n_rows, int N, int K, const float* bias, float* out_f32, int ldo, void* out_act,
                 int out_K, int max_rows, hipStream_t s);

void launch_attention(int dtype, const ModelDims& md, const float* y, const float* rope, const RowDesc& rd,
                      void* kcache, void* vcache, size_t layer_off, int ctx_bound /* upper bound of the rows' cache lengths */,
                      int max_seq /* slots per (row, KV head) of the caches; bf16: a multiple of 32 */,
                      void* ao, int max_rows, hipStream_t s, int phase = 0);
// phase 0: append the row's new key / value to the cache and attend (rows of one launch own different caches);
// phase 1: append only; phase 2: attend only (the pair serves launches where several rows share a cache).

int lmhead_num_wg(int dtype, int V);
void launch_lmhead(int dtype, const void* W, const void* X, size_t x_elems, const RowDesc& rd, int V, int K,
                   const SamplerArgs& sa, unsigned long long* part, int n_wg, int Mpad,
                   float* logits_out, int max_rows, hipStream_t s);

int verifier_num_chunks(int d_hidden);
void launch_verifier_part(const float* hf, int d, int d_hidden, const float* w1, const float* b1,
                          const float* w2, const int* n_rows, float* part, int max_rows, hipStream_t s);

struct State {           // device-resident per-batch state
  int* last_tok;         // [B] last committed token
  int* len_q;            // [B] entries in the draft cache
  int* len_p;            // [B] entries in the target cache
  long long* n_target_calls;  // [B]
  long long* counters;   // [4] steps, steps_with_target, sum_rejected, gen_idx
  int* prompt_len;       // [B]
  int* hist;             // [B][hist_stride] every committed token by position (prompt included)
  int hist_stride;       // max_seq + 1
};

struct DecideArgs {
  const unsigned long long* am_part; int n_lm_wg; int Mpad;
  const float* ver_part; int n_chunks; const float* b2; const float* tau_ptr;
  int B;
  State st;
  // per-step scratch written here
  int* draft_tok; float* score; unsigned char* accept; int* rej_idx; int* n_rej; int* committed;
  // target row descriptors written here
  int* t_n_rows; int* t_b; int* t_tok; int* t_pos; int* t_slot;
  // optional caller outputs (per-step layout [B])
  int* o_draft_tok; float* o_score; unsigned char* o_accept; int* o_rej_idx; int* o_n_rej;
  // pinned host word the waiting host thread polls: (ticket << 32) | number of rejected rows
  // with ctx_mode 1 word [1] receives the number of work-list entries of the target pass
  unsigned long long* host_word; unsigned ticket;
  // ctx_mode 1 (full prefix): rejected row i brings len_q - len_p + 1 entries (the committed tokens its target
  // cache has not seen, then the step's own input); ent_off[0 .. R] = exclusive prefix sums of those counts
  int ctx_mode; int* ent_off;
};
void launch_draft_decide(const DecideArgs& a, hipStream_t s);

struct FinishArgs {
  const unsigned long long* am_part; int n_lm_wg; int Mpad;
  int B;
  State st;
  const int* draft_tok; const float* score; const unsigned char* accept; const int* rej_idx; const int* n_rej;
  int* committed;
  // next step's draft row descriptors
  int* d_n_rows; int* d_b; int* d_tok; int* d_pos; int* d_slot;
  // optional outputs: per-step [B] (step mode) ...
  int* o_committed;
  // ... and [B, n_tokens] arrays indexed by the device-side generation counter (generate mode)
  int n_tokens; int* g_tok; unsigned char* g_accept; float* g_score; int* g_draft_tok;
  int ctx_mode;     // 1: a rejected row's target cache is complete afterwards
  int pre_merged;   // 1: committed[] already holds the rejected rows' tokens (full-prefix collect / p-over-q correction)
};
void launch_step_finish(const FinishArgs& a, hipStream_t s);

// Full-prefix target context: entries [start, start + n) of the step's work list become the target's row
// descriptors (several entries may belong to one batch row; entry order = ascending row, ascending position).
struct CatchupArgs {
  State st; const int* rej_idx; const int* n_rej; const int* ent_off; int start, n;
  int* t_n_rows; int* t_b; int* t_tok; int* t_pos; int* t_slot; int* t_last;   // t_last[e] = 1: last entry of its row
};
void launch_catchup_chunk(const CatchupArgs& a, hipStream_t s);
// After the chunk's forward: the sampled token of every last entry becomes the row's committed token.
void launch_catchup_collect(const unsigned long long* am_part, int n_lm_wg, int Mpad, const int* n_rows, const int* t_b,
                            const int* t_last, int* committed, int max_rows, hipStream_t s);

// Rejection by the p/q coin and the residual of Eq. (1): one workgroup per row of the target pass.
struct SdArgs {
  const float* dl;            // [batch rows][V] draft logits of the step
  const float* tl;            // [pass rows][V] target logits of the pass
  const int* n_rows; const int* t_b; const int* t_pos; const int* t_last;   // t_last may be NULL (every row counts)
  const int* draft_tok; int V; float inv_temperature; unsigned seed_lo, seed_hi;
  int* committed; int* coin_kept;
};
void launch_sd_correct(const SdArgs& a, int max_rows, hipStream_t s);
void launch_set_i32(int* p, int v, hipStream_t s);

// ---- standard speculative decoding (Sec. 2, Eq. (1)) on the same models: k_sd.hip -------------------
struct RowDescW { int* n_rows; int* b; int* tok; int* pos; int* slot; };   // a writable RowDesc
struct SdBase {
  State st;
  int B, gamma, V;
  int* len_dc;            // [B] entries in the draft cache (one behind len_q after a window that was kept whole)
  int* win;               // [B][gamma] the round's draft tokens
  int* qrow;              // [B][gamma] row of dlw with the draft logits behind win[b][j]
  unsigned char* kept;    // [B][gamma] outcome of the p/q coin
  int* alt;               // [B][gamma + 1] residual draw where the coin failed; [gamma]: the extra token
  // work list of a round's first draft pass: 1 or 2 entries per row (row-major, ascending position)
  int* d0_n; int* d0_b; int* d0_tok; int* d0_pos; int* d0_last;
  float* dlw;             // draft logits: rows [0, 2B) first pass (by entry), then B rows per further pass
  float* tlw;             // target logits by entry b * (gamma + 1) + j
  int* o_cnt;             // [B] tokens written to the caller's array so far
  unsigned seed_lo, seed_hi; float inv_temperature;
  int* coin_kept;
};
// Start of a call: clears the per-call token counts; fresh (first rounds after a prefill): the draft cache is level
// with the target's, one entry per row.
void launch_sd_begin(const SdBase& a, int fresh, hipStream_t s);
// Entries [start, start + n) of the first-pass work list become row descriptors (is_last[i]: last entry of its row).
void launch_sd_take_chunk(const SdBase& a, int start, int n, RowDescW out, int* is_last, hipStream_t s);
// After draft pass j over the rows of `in`: the sampled token of every (last) entry joins the window and the
// token history and becomes the row's input of the next pass (`out`, one entry per batch row).
void launch_sd_draft_next(const SdBase& a, int j, const unsigned long long* am_part, int n_lm_wg, int Mpad, RowDesc in,
                          const int* is_last, int logits_row_base, RowDescW out, int max_rows, hipStream_t s);
// Entries [start, start + n) of the target pass: entry e = b * (gamma + 1) + j reads position len_q[b] + j.
void launch_sd_target_list(const SdBase& a, int start, int n, RowDescW out, hipStream_t s);
// One workgroup per entry of the chunk: the p/q coin and, where it fails, the residual draw; entry gamma of a
// row takes the target's own sample (the extra token).
void launch_sd_window_check(const SdBase& a, int start, int n, const unsigned long long* am_part, int n_lm_wg, int Mpad,
                            hipStream_t s);
struct SdFinishArgs {
  int round, n_rounds, tok_stride;
  int* o_tok; int* o_n_tok; int* o_n_acc; int* o_draft;
  unsigned long long* host_word; unsigned ticket;   // receives (ticket << 32) | entries of the next first draft pass
};
void launch_sd_round_finish(const SdBase& a, const SdFinishArgs& f, hipStream_t s);

void launch_prefill_begin(const int* prompt, int max_prompt, int B, State st, int* rej_idx, int* n_rej, hipStream_t s);
void launch_prefill_finish(const int* prompt, int max_prompt, int B, State st,
                           int* d_n_rows, int* d_b, int* d_tok, int* d_pos, int* d_slot, hipStream_t s);
void launch_reset_gen_idx(long long* counters, hipStream_t s);
void launch_set_f32(float* p, float v, hipStream_t s);
void launch_copy_f32(const float* src, float* dst, const int* n_rows, int row_len, int max_rows, hipStream_t s);

}  // namespace sprinter
