// Internal declarations shared by the C-ABI layer (abi.cpp) and the kernel
// launchers (kernels.hip).  Nothing here is part of the public interface.
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

struct ModelScratch {  // per-model activation buffers, sized for max_batch rows
  float* h;            // [M, d] residual stream, float32
  void* xn;            // [M, d] normalised GEMM input (activation layout)
  float* y;            // [M, dqkv] QKV projection output, float32
  void* ao;            // [M, H*dh] attention output (activation layout)
  void* mid;           // [M, ff] FFN hidden (activation layout)
  float* hf;           // [M, d] final hidden state after the last norm, float32
  void* hfn;           // same values in activation layout (LM-head input)
  float* rope;         // [M, dh/2, 2] cos/sin of the row's position
  unsigned long long* am_part;  // [n_lm_wg, Mpad] packed (value, index) arg-max partials
  int n_lm_wg;
};

struct SamplerArgs {
  unsigned seed_lo, seed_hi, stream;
  float inv_temperature;   // 0 = greedy (no noise)
};

// ---- launchers (kernels.hip) ------------------------------------------------
void launch_pack_bf16(const void* w, void* out, int N, int K, hipStream_t s);
void launch_fill_zero(void* p, size_t bytes, hipStream_t s);

void launch_embed(int dtype, const ModelDims& md, const void* tok_emb, const void* pos_emb,
                  const RowDesc& rd, float* h, float* rope, int max_rows, hipStream_t s);
void launch_norm(int dtype, int arch, const float* h, const float* g, const float* b, float eps, int d,
                 const int* n_rows, void* act_out, size_t plane, float* f32_out, int max_rows, hipStream_t s);

enum { EPI_F32 = 0, EPI_RESID = 1, EPI_GELU = 2, EPI_SWIGLU = 3 };
// Y[M,N] = X[M,K] W[N,K]^T (+bias) with epilogue; X in activation layout, W in weight layout.
// x_plane / out_plane: element distance between the hi and lo planes of a bf16 activation buffer.
void launch_gemm(int dtype, int epi, const void* W, const void* W2, const void* X, size_t x_plane,
                 const int* n_rows, int N, int K, const float* bias, float* out_f32, int ldo, void* out_act,
                 int out_K, size_t out_plane, int max_rows, hipStream_t s);

void launch_attention(int dtype, const ModelDims& md, const float* y, const float* rope, const RowDesc& rd,
                      void* kcache, void* vcache, size_t layer_off, int max_batch, int max_seq,
                      void* ao, size_t ao_plane, int max_rows, hipStream_t s);

int lmhead_num_wg(int dtype, int V);
void launch_lmhead(int dtype, const void* W, const void* X, size_t x_plane, const RowDesc& rd, int V, int K,
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
};
void launch_step_finish(const FinishArgs& a, hipStream_t s);

void launch_prefill_prep(const int* prompt, int max_prompt, int j, int B, const int* prompt_len,
                         int* n_rows, int* rb, int* rtok, int* rpos, int* rslot, hipStream_t s);
void launch_prefill_finish(const int* prompt, int max_prompt, int B, State st,
                           int* d_n_rows, int* d_b, int* d_tok, int* d_pos, int* d_slot, hipStream_t s);
void launch_reset_gen_idx(long long* counters, hipStream_t s);
void launch_set_f32(float* p, float v, hipStream_t s);
void launch_copy_f32(const float* src, float* dst, const int* n_rows, int row_len, int max_rows, hipStream_t s);

}  // namespace sprinter
