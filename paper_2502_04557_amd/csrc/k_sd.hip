// HIP kernels of standard speculative decoding (Sec. 2 with Eq. (1)) for gfx950: work lists of the draft window
// and of the target's parallel pass, the p/q coin with the residual draw, and the commit of a round.
#include "dev.h"

namespace sprinter {

__global__ __launch_bounds__(1024) void k_sd_begin(SdBase a, int fresh) {
  const int b = threadIdx.x;
  if (b < a.B) {
    a.o_cnt[b] = 0;
    if (fresh) {
      const int lq = a.st.len_q[b];
      a.len_dc[b] = lq;
      a.d0_b[b] = b; a.d0_tok[b] = a.st.last_tok[b]; a.d0_pos[b] = lq; a.d0_last[b] = 1;
    }
  }
  if (b == 0 && fresh) *a.d0_n = a.B;
}
void launch_sd_begin(const SdBase& a, int fresh, hipStream_t s) {
  hipLaunchKernelGGL(k_sd_begin, dim3(1), dim3(1024), 0, s, a, fresh);
}

__global__ __launch_bounds__(1024) void k_sd_take_chunk(SdBase a, int start, int n, RowDescW out, int* is_last) {
  for (int i = threadIdx.x; i < n; i += 1024) {
    const int e = start + i;
    out.b[i] = a.d0_b[e]; out.tok[i] = a.d0_tok[e];
    out.pos[i] = a.d0_pos[e]; out.slot[i] = a.d0_pos[e];
    is_last[i] = a.d0_last[e];
  }
  if (threadIdx.x == 0) *out.n_rows = n;
}
void launch_sd_take_chunk(const SdBase& a, int start, int n, RowDescW out, int* is_last, hipStream_t s) {
  hipLaunchKernelGGL(k_sd_take_chunk, dim3(1), dim3(1024), 0, s, a, start, n, out, is_last);
}

// One wave per row of the pass.
__global__ __launch_bounds__(256) void k_sd_draft_next(SdBase a, int j, const u64* __restrict__ am_part, int n_lm_wg, int Mpad,
                                                       RowDesc in, const int* __restrict__ is_last, int logits_row_base,
                                                       RowDescW out) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + wave_index();
  if (blockIdx.x == 0 && threadIdx.x == 0) *out.n_rows = a.B;
  if (i >= *in.n_rows) return;
  if (is_last && !is_last[i]) return;
  const u64 k = merge_partials(am_part, n_lm_wg, Mpad, i, lane);
  if (lane == 0) {
    const int b = in.b[i], x = key_index(k), p = in.pos[i];
    a.win[b * a.gamma + j] = x;
    a.qrow[b * a.gamma + j] = logits_row_base + i;
    a.st.hist[(size_t)b * a.st.hist_stride + p + 1] = x;
    out.b[b] = b; out.tok[b] = x; out.pos[b] = p + 1; out.slot[b] = p + 1;
  }
}
void launch_sd_draft_next(const SdBase& a, int j, const unsigned long long* am_part, int n_lm_wg, int Mpad, RowDesc in,
                          const int* is_last, int logits_row_base, RowDescW out, int max_rows, hipStream_t s) {
  hipLaunchKernelGGL(k_sd_draft_next, dim3((max_rows + 3) / 4), dim3(256), 0, s, a, j, am_part, n_lm_wg, Mpad, in, is_last,
                     logits_row_base, out);
}

__global__ __launch_bounds__(1024) void k_sd_target_list(SdBase a, int start, int n, RowDescW out) {
  const int per = a.gamma + 1;
  for (int i = threadIdx.x; i < n; i += 1024) {
    const int e = start + i, b = e / per, j = e - b * per;
    const int pos = a.st.len_q[b] + j;
    out.b[i] = b; out.tok[i] = a.st.hist[(size_t)b * a.st.hist_stride + pos];
    out.pos[i] = pos; out.slot[i] = pos;                 // the target's cache has no gaps here: slot = position
  }
  if (threadIdx.x == 0) *out.n_rows = n;
}
void launch_sd_target_list(const SdBase& a, int start, int n, RowDescW out, hipStream_t s) {
  hipLaunchKernelGGL(k_sd_target_list, dim3(1), dim3(1024), 0, s, a, start, n, out);
}

// q = softmax(draft logits / T), p = softmax(target logits / T); sweeps over the vocabulary for the maxima, the
// sums of exponentials and - only where the coin fails - the Gumbel-max draw from max(0, p - q), taken on
// ln(p - q) + noise of the target stream.  float32 throughout.
__global__ __launch_bounds__(256) void k_sd_window_check(SdBase a, int start, const u64* __restrict__ am_part, int n_lm_wg,
                                                         int Mpad) {
  __shared__ float s4[4];
  __shared__ u64 s_key[4];
  const int i = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = wave_index();
  const int per = a.gamma + 1, e = start + i, b = e / per, j = e - b * per, V = a.V;
  if (j == a.gamma) {                                    // the extra token: the target's own sample of this entry
    if (w == 0) {
      const u64 k = merge_partials(am_part, n_lm_wg, Mpad, i, lane);
      if (lane == 0) a.alt[b * per + j] = key_index(k);
    }
    return;
  }
  const int t = a.st.len_q[b] + j + 1;                   // sequence position of the checked token
  const int x = a.win[b * a.gamma + j];
  const float* __restrict__ lq = a.dlw + (size_t)a.qrow[b * a.gamma + j] * V;
  const float* __restrict__ lp = a.tlw + (size_t)e * V;
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
  const bool kept = coin <= fminf(1.0f, expf(log_ratio));        // uniform over the workgroup
  if (tid == 0) a.kept[b * a.gamma + j] = kept ? 1 : 0;
  if (kept) return;
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
    a.alt[b * per + j] = best ? key_index(best) : x;     // (an empty residual cannot occur when the coin fails)
  }
}
void launch_sd_window_check(const SdBase& a, int start, int n, const unsigned long long* am_part, int n_lm_wg, int Mpad,
                            hipStream_t s) {
  hipLaunchKernelGGL(k_sd_window_check, dim3(n), dim3(256), 0, s, a, start, am_part, n_lm_wg, Mpad);
}

// Single workgroup, one thread per row: the first failed coin ends the window; commit, advance the state, and
// lay out the next round's first draft pass (a row whose window was kept whole still owes the draft model its
// last window token).
__global__ __launch_bounds__(1024) void k_sd_round_finish(SdBase a, SdFinishArgs f) {
  __shared__ int s_wave_cnt[16];
  __shared__ int s_cut, s_kept;
  const int b = threadIdx.x, lane = b & 63, w = b >> 6, G = a.gamma;
  if (b == 0) { s_cut = 0; s_kept = 0; }
  __syncthreads();
  int cnt = 0, ndc = 0, nlq = 0;
  if (b < a.B) {
    const int lq = a.st.len_q[b];
    int n_acc = G;
    for (int j = G - 1; j >= 0; --j) if (!a.kept[b * G + j]) n_acc = j;
    const int last = a.alt[b * (G + 1) + n_acc];
    int* hist = a.st.hist + (size_t)b * a.st.hist_stride;
    hist[lq + 1 + n_acc] = last;
    const int done = a.o_cnt[b];
    if (f.o_tok) {
      for (int k = 0; k < n_acc; ++k) f.o_tok[(size_t)b * f.tok_stride + done + k] = a.win[b * G + k];
      f.o_tok[(size_t)b * f.tok_stride + done + n_acc] = last;
    }
    a.o_cnt[b] = done + n_acc + 1;
    if (f.o_n_tok) f.o_n_tok[b] = done + n_acc + 1;
    if (f.o_n_acc) f.o_n_acc[(size_t)b * f.n_rounds + f.round] = n_acc;
    if (f.o_draft) for (int j = 0; j < G; ++j) f.o_draft[((size_t)b * f.n_rounds + f.round) * G + j] = a.win[b * G + j];
    nlq = lq + n_acc + 1;
    ndc = min(lq + G, nlq);                 // the draft cache holds the inputs of its G passes: positions < lq + G
    a.st.len_q[b] = nlq; a.st.len_p[b] = nlq; a.st.last_tok[b] = last; a.len_dc[b] = ndc;
    a.st.n_target_calls[b] += 1;
    cnt = nlq - ndc + 1;
    if (n_acc < G) atomicAdd(&s_cut, 1);
    atomicAdd(&s_kept, n_acc);
  }
  int inc = cnt;                                         // inclusive scan inside the wave
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) { const int up = __shfl_up(inc, o); if (lane >= o) inc += up; }
  if (lane == 63) s_wave_cnt[w] = inc;
  __syncthreads();
  int before = 0, all = 0;
  for (int q = 0; q < 16; ++q) { const int c = s_wave_cnt[q]; if (q < w) before += c; all += c; }
  if (b < a.B) {
    const int off = before + inc - cnt;
    const int* hist = a.st.hist + (size_t)b * a.st.hist_stride;
    for (int k = 0; k < cnt; ++k) {
      a.d0_b[off + k] = b; a.d0_pos[off + k] = ndc + k; a.d0_tok[off + k] = hist[ndc + k];
      a.d0_last[off + k] = (k == cnt - 1) ? 1 : 0;
    }
  }
  if (b == 0) {
    *a.d0_n = all;
    a.st.counters[0] += 1; a.st.counters[1] += 1; a.st.counters[2] += s_cut;
    *a.coin_kept += s_kept;
    if (f.host_word)
      __hip_atomic_store(f.host_word, ((unsigned long long)f.ticket << 32) | (unsigned)all, __ATOMIC_RELEASE,
                         __HIP_MEMORY_SCOPE_SYSTEM);
  }
}
void launch_sd_round_finish(const SdBase& a, const SdFinishArgs& f, hipStream_t s) {
  hipLaunchKernelGGL(k_sd_round_finish, dim3(1), dim3(1024), 0, s, a, f);
}

}  // namespace sprinter
