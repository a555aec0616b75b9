// HIP kernels of the batched SPRINTER decode step for gfx950: the decisions of Alg. 2 (threshold, compaction,
// commit), prefill row lists, the full-prefix work list and the p/q correction of Sec. 2, Eq. (1).
#include "dev.h"
#include <algorithm>
#include <cstring>

namespace sprinter {

// ====================================== decide: arg-max merge, threshold, compaction
// Single workgroup of 1024 threads (B <= 1024).  accept <=> sigmoid(logit) >= tau in float32.
// Rejected rows are listed in ascending order: ballot + popcount inside each wave,
// wave totals prefix-summed through LDS.
__global__ __launch_bounds__(1024) void k_draft_decide(DecideArgs a) {
  __shared__ int s_tok[1024];
  __shared__ int s_wave_cnt[16];
  __shared__ int s_rej[1024];
  __shared__ u64 s_key[16][64];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int B = a.B;
  // Arg-max merge over the LM head's per-workgroup partials part[workgroup][row]: a lane takes one row of a block
  // of 64, a wave every 16th workgroup, so that a load covers 64 consecutive rows of one workgroup (512 contiguous
  // bytes; with a lane per workgroup every 8-byte load hit its own cache line: 37 us at 64 rows and 512 workgroups),
  // then the 16 waves' results meet in LDS.
  float z = 0.f;                                     // the verifier's output logit: offset + the hidden chunks' shares, in order
  if (tid < B) {                                     // (requested ahead of the merge below)
    z = a.b2[0];
#pragma unroll 8
    for (int c = 0; c < a.n_chunks; ++c) z += a.ver_part[(size_t)c * B + tid];
  }
  for (int rb = 0; rb < B; rb += 64) {
    const int m = rb + lane;
    u64 k = 0;
    if (m < B)
      for (int i0 = w; i0 < a.n_lm_wg; i0 += 128) {            // eight loads in flight per lane, not a chain of single ones
        u64 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int i = i0 + 16 * u;
          v[u] = i < a.n_lm_wg ? a.am_part[(size_t)i * a.Mpad + m] : 0;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) k = umax64(k, v[u]);
      }
    s_key[w][lane] = k;
    __syncthreads();
    if (w == 0 && m < B) {
      u64 kk = s_key[0][lane];
#pragma unroll
      for (int q = 1; q < 16; ++q) kk = umax64(kk, s_key[q][lane]);
      s_tok[m] = key_index(kk);
    }
    __syncthreads();
  }
  bool active = tid < B;
  float score = 0.f;
  bool acc = true;
  if (active) {
    score = 1.0f / (1.0f + expf(-z));
    acc = score >= *a.tau_ptr;
  }
  const bool rej = active && !acc;
  const u64 mask = __ballot(rej);
  const int rank = __popcll(mask & ((1ull << lane) - 1ull));
  if (lane == 0) s_wave_cnt[w] = __popcll(mask);
  __syncthreads();
  int off = 0, total = 0;
  for (int q = 0; q < 16; ++q) {
    int c = s_wave_cnt[q];
    if (q < w) off += c;
    total += c;
  }
  if (rej) s_rej[off + rank] = tid;
  if (active) {
    int dt = s_tok[tid];
    a.draft_tok[tid] = dt;
    a.score[tid] = score;
    a.accept[tid] = acc ? 1 : 0;
    a.committed[tid] = acc ? dt : -1;
    if (a.o_draft_tok) a.o_draft_tok[tid] = dt;
    if (a.o_score) a.o_score[tid] = score;
    if (a.o_accept) a.o_accept[tid] = acc ? 1 : 0;
  }
  __syncthreads();
  if (tid < total) {
    int b = s_rej[tid];
    a.rej_idx[tid] = b;
    if (a.o_rej_idx) a.o_rej_idx[tid] = b;
    a.t_b[tid] = b;
    a.t_tok[tid] = a.st.last_tok[b];
    a.t_pos[tid] = a.st.len_q[b];       // true position id of the input token
    a.t_slot[tid] = a.st.len_p[b];      // next free slot of the row's target cache
  }
  if (a.ctx_mode == 1) {
    // work list of the full-prefix target pass: entries per rejected row, exclusive prefix sums in ascending row order
    __syncthreads();
    int cnt = 0;
    if (tid < total) { const int b = s_rej[tid]; cnt = a.st.len_q[b] - a.st.len_p[b] + 1; }
    int inc = cnt;                                     // inclusive scan inside the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const int up = __shfl_up(inc, o); if (lane >= o) inc += up; }
    if (lane == 63) s_wave_cnt[w] = inc;
    __syncthreads();
    int before = 0, all = 0;
    for (int q = 0; q < 16; ++q) { const int c = s_wave_cnt[q]; if (q < w) before += c; all += c; }
    if (tid < total) a.ent_off[tid] = before + inc - cnt;
    if (tid == 0) {
      a.ent_off[total] = all;
      if (a.host_word) a.host_word[1] = (unsigned long long)(unsigned)all;   // ordered before the release store below
    }
  }
  if (tid == 0) {
    *a.n_rej = total;
    *a.t_n_rows = total;
    if (a.o_n_rej) *a.o_n_rej = total;
    if (a.host_word)    // one 8-byte store into pinned host memory: the host launches the target pass from it
      __hip_atomic_store(a.host_word, ((unsigned long long)a.ticket << 32) | (unsigned)total, __ATOMIC_RELEASE,
                         __HIP_MEMORY_SCOPE_SYSTEM);
  }
}
void launch_draft_decide(const DecideArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(k_draft_decide, dim3(1), dim3(1024), 0, s, a);
}

// ===================== finish: target arg-max merge, scatter back, advance state
__global__ __launch_bounds__(1024) void k_step_finish(FinishArgs a) {
  __shared__ int s_commit[1024];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int B = a.B, R = *a.n_rej;
  if (tid < B) s_commit[tid] = a.committed[tid];
  __syncthreads();
  if (!a.pre_merged) {
    for (int i = w; i < R; i += 16) {
      u64 k = merge_partials(a.am_part, a.n_lm_wg, a.Mpad, i, lane);
      if (lane == 0) s_commit[a.rej_idx[i]] = key_index(k);
    }
  }
  __syncthreads();
  const long long g = a.st.counters[3];
  if (tid < B) {
    int c = s_commit[tid];
    bool acc = a.accept[tid] != 0;
    a.committed[tid] = c;
    a.st.last_tok[tid] = c;
    int lq = a.st.len_q[tid] + 1;
    a.st.len_q[tid] = lq;
    if (!acc) {
      a.st.len_p[tid] = a.ctx_mode == 1 ? lq : a.st.len_p[tid] + 1;
      a.st.n_target_calls[tid] += 1;
    }
    a.st.hist[(size_t)tid * a.st.hist_stride + lq] = c;
    if (a.o_committed) a.o_committed[tid] = c;
    if (a.n_tokens > 0 && g < a.n_tokens) {
      size_t o = (size_t)tid * a.n_tokens + (size_t)g;
      if (a.g_tok) a.g_tok[o] = c;
      if (a.g_accept) a.g_accept[o] = acc ? 1 : 0;
      if (a.g_score) a.g_score[o] = a.score[tid];
      if (a.g_draft_tok) a.g_draft_tok[o] = a.draft_tok[tid];
    }
    // the next step's draft forward: every row, its last token at the next position
    a.d_b[tid] = tid;
    a.d_tok[tid] = c;
    a.d_pos[tid] = lq;
    a.d_slot[tid] = lq;
  }
  if (tid == 0) {
    *a.d_n_rows = B;
    a.st.counters[0] += 1;
    a.st.counters[1] += (R > 0) ? 1 : 0;
    a.st.counters[2] += R;
    a.st.counters[3] = g + 1;
  }
}
void launch_step_finish(const FinishArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(k_step_finish, dim3(1), dim3(1024), 0, s, a);
}

// ================================================================ prefill
// Chunked prefill: the prompts go into the token history, every row's caches count as empty and every row is
// listed, so that the full-prefix work-list kernel (k_catchup_chunk) enumerates the prompt positions 0 .. P_b-2
// in row-major order from the prefix sums the host uploaded.
__global__ __launch_bounds__(1024) void k_prefill_begin(const int* __restrict__ prompt, int max_prompt, int B, State st,
                                                        int* rej_idx, int* n_rej) {
  const int tid = threadIdx.x;
  if (tid < B) {
    const int P = st.prompt_len[tid];
    for (int j = 0; j < P; ++j) st.hist[(size_t)tid * st.hist_stride + j] = prompt[(size_t)tid * max_prompt + j];
    st.len_p[tid] = 0;
    rej_idx[tid] = tid;
  }
  if (tid == 0) *n_rej = B;
}
void launch_prefill_begin(const int* prompt, int max_prompt, int B, State st, int* rej_idx, int* n_rej, hipStream_t s) {
  hipLaunchKernelGGL(k_prefill_begin, dim3(1), dim3(1024), 0, s, prompt, max_prompt, B, st, rej_idx, n_rej);
}

__global__ __launch_bounds__(1024) void k_prefill_finish(const int* __restrict__ prompt, int max_prompt, int B,
                                                         State st, int* d_n_rows, int* d_b, int* d_tok, int* d_pos,
                                                         int* d_slot) {
  const int tid = threadIdx.x;
  if (tid < B) {
    int P = st.prompt_len[tid];
    int last = prompt[(size_t)tid * max_prompt + P - 1];
    st.last_tok[tid] = last;
    st.len_q[tid] = P - 1;
    st.len_p[tid] = P - 1;
    st.n_target_calls[tid] = 0;
    for (int j = 0; j < P; ++j) st.hist[(size_t)tid * st.hist_stride + j] = prompt[(size_t)tid * max_prompt + j];
    d_b[tid] = tid;
    d_tok[tid] = last;
    d_pos[tid] = P - 1;
    d_slot[tid] = P - 1;
  }
  if (tid == 0) {
    *d_n_rows = B;
    st.counters[0] = st.counters[1] = st.counters[2] = st.counters[3] = 0;
  }
}
void launch_prefill_finish(const int* prompt, int max_prompt, int B, State st, int* d_n_rows, int* d_b, int* d_tok,
                           int* d_pos, int* d_slot, hipStream_t s) {
  hipLaunchKernelGGL(k_prefill_finish, dim3(1), dim3(1024), 0, s, prompt, max_prompt, B, st, d_n_rows, d_b, d_tok,
                     d_pos, d_slot);
}

// ============================================ full-prefix target context: work list
// One thread per entry of the chunk: binary search of the entry's rejected row in the prefix sums.
__global__ __launch_bounds__(1024) void k_catchup_chunk(CatchupArgs a) {
  const int R = *a.n_rej;
  for (int i = threadIdx.x; i < a.n; i += 1024) {
    const int e = a.start + i;
    int lo = 0, hi = R - 1;                            // last row index with ent_off[row] <= e
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (a.ent_off[mid] <= e) lo = mid; else hi = mid - 1;
    }
    const int b = a.rej_idx[lo];
    const int pos = a.st.len_p[b] + (e - a.ent_off[lo]);
    a.t_b[i] = b;
    a.t_tok[i] = a.st.hist[(size_t)b * a.st.hist_stride + pos];
    a.t_pos[i] = pos;
    a.t_slot[i] = pos;                                 // in this mode the target cache has no gaps: slot = position
    a.t_last[i] = (e + 1 == a.ent_off[lo + 1]) ? 1 : 0;
  }
  if (threadIdx.x == 0) *a.t_n_rows = a.n;
}
void launch_catchup_chunk(const CatchupArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(k_catchup_chunk, dim3(1), dim3(1024), 0, s, a);
}

__global__ __launch_bounds__(256) void k_catchup_collect(const u64* __restrict__ am_part, int n_lm_wg, int Mpad,
                                                        const int* __restrict__ n_rows, const int* __restrict__ t_b,
                                                        const int* __restrict__ t_last, int* __restrict__ committed) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + wave_index();
  if (i >= *n_rows || !t_last[i]) return;
  const u64 k = merge_partials(am_part, n_lm_wg, Mpad, i, lane);
  if (lane == 0) committed[t_b[i]] = key_index(k);
}
void launch_catchup_collect(const unsigned long long* am_part, int n_lm_wg, int Mpad, const int* n_rows, const int* t_b,
                            const int* t_last, int* committed, int max_rows, hipStream_t s) {
  hipLaunchKernelGGL(k_catchup_collect, dim3((max_rows + 3) / 4), dim3(256), 0, s, am_part, n_lm_wg, Mpad, n_rows, t_b,
                     t_last, committed);
}

// ===================================== rejection by p/q coin + residual (Sec. 2, Eq. (1))
// One workgroup per row of the target pass.  q = softmax(draft logits / T), p = softmax(target logits / T):
// three sweeps over the vocabulary (maxima, sums of exponentials, and - only if the coin rejects - the
// Gumbel-max draw from max(0, p - q), on ln(p - q) + noise of the target stream).  float32 throughout.
__global__ __launch_bounds__(256) void k_sd_correct(SdArgs a) {
  __shared__ float s4[4];
  __shared__ u64 s_key[4];
  const int i = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = wave_index();
  if (i >= *a.n_rows) return;
  if (a.t_last && !a.t_last[i]) return;
  const int b = a.t_b[i], t = a.t_pos[i] + 1, x = a.draft_tok[b], V = a.V;
  const float* __restrict__ lq = a.dl + (size_t)b * V;
  const float* __restrict__ lp = a.tl + (size_t)i * V;
  const float it = a.inv_temperature;
  float mq = -INFINITY, mp = -INFINITY;
  for (int v = tid; v < V; v += 256) { mq = fmaxf(mq, lq[v] * it); mp = fmaxf(mp, lp[v] * it); }
  mq = block_max256(mq, s4);
  mp = block_max256(mp, s4);
  float sq = 0.f, sp = 0.f;
  for (int v = tid; v < V; v += 256) { sq += expf(lq[v] * it - mq); sp += expf(lp[v] * it - mp); }
  sq = block_sum256(sq, s4);
  sp = block_sum256(sp, s4);
  const float lse_q = mq + logf(sq), lse_p = mp + logf(sp);
  const float log_ratio = (lp[x] * it - lse_p) - (lq[x] * it - lse_q);
  const unsigned cw = philox_word(a.seed_lo, a.seed_hi, 2u, (unsigned)b, (unsigned)t, 0u);
  const float coin = ((float)(cw >> 9) + 0.5f) * 1.1920928955078125e-07f;
  const bool kept = coin <= fminf(1.0f, expf(log_ratio));       // uniform over the workgroup
  if (kept) {
    if (tid == 0) { a.committed[b] = x; atomicAdd(a.coin_kept, 1); }
    return;
  }
  u64 best = 0;
  for (int v = tid; v < V; v += 256) {
    const float r = expf(lp[v] * it - lse_p) - expf(lq[v] * it - lse_q);
    if (r > 0.f) {
      const float z = logf(r) + gumbel_from_word(philox_word(a.seed_lo, a.seed_hi, 1u, (unsigned)b, (unsigned)t, (unsigned)v));
      best = umax64(best, pack_key(z, (unsigned)v));
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) best = umax64(best, shfl_xor_u64(best, o));
  if (lane == 0) s_key[w] = best;
  __syncthreads();
  if (tid == 0) {
    best = umax64(umax64(s_key[0], s_key[1]), umax64(s_key[2], s_key[3]));
    a.committed[b] = best ? key_index(best) : x;      // (an empty residual cannot occur when the coin rejects)
  }
}
void launch_sd_correct(const SdArgs& a, int max_rows, hipStream_t s) {
  hipLaunchKernelGGL(k_sd_correct, dim3(max_rows), dim3(256), 0, s, a);
}

__global__ void k_set_i32(int* p, int v) { *p = v; }
void launch_set_i32(int* p, int v, hipStream_t s) { hipLaunchKernelGGL(k_set_i32, dim3(1), dim3(1), 0, s, p, v); }

__global__ void k_set_f32(float* p, float v) { *p = v; }
void launch_set_f32(float* p, float v, hipStream_t s) { hipLaunchKernelGGL(k_set_f32, dim3(1), dim3(1), 0, s, p, v); }

__global__ void k_reset_gen_idx(long long* counters) { counters[3] = 0; }
void launch_reset_gen_idx(long long* counters, hipStream_t s) {
  hipLaunchKernelGGL(k_reset_gen_idx, dim3(1), dim3(1), 0, s, counters);
}

__global__ __launch_bounds__(256) void k_copy_rows(const float* __restrict__ src, float* __restrict__ dst,
                                                   const int* __restrict__ n_rows, int row_len) {
  int r = blockIdx.x;
  if (r >= *n_rows) return;
  for (int k = threadIdx.x; k < row_len; k += 256) dst[(size_t)r * row_len + k] = src[(size_t)r * row_len + k];
}
void launch_copy_f32(const float* src, float* dst, const int* n_rows, int row_len, int max_rows, hipStream_t s) {
  hipLaunchKernelGGL(k_copy_rows, dim3(max_rows), dim3(256), 0, s, src, dst, n_rows, row_len);
}

}  // namespace sprinter
