// Device-side pieces shared by the persistent decode kernels (mega.hip: any batch; mega16.hip: at most
// 16 rows): device-scope loads and stores, the flag-tree grid barrier, embedding, verifier partials,
// arg-max merge, the decision / compaction step and the scatter-back step.
#pragma once
#include "dev.h"

namespace sprinter {
namespace {

constexpr int NT = 512;
constexpr int NWV = 8;
constexpr int GS = 32;                       // workgroups per barrier group
constexpr long long SPIN_LIMIT = 8000000LL;  // polling iterations before a wait gives up (~ seconds)

// ---------------------------------------------------------------- coherent access
__device__ __forceinline__ void st_u32(void* p, unsigned v) {
  __hip_atomic_store((unsigned*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_i32(int* p, int v) { st_u32(p, (unsigned)v); }
__device__ __forceinline__ void st_f32(float* p, float v) { st_u32(p, __float_as_uint(v)); }
__device__ __forceinline__ void st_u64(void* p, u64 v) {
  __hip_atomic_store((u64*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_u16(void* p, unsigned v) {
  asm volatile("global_store_short %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void st_u8(void* p, unsigned v) {
  asm volatile("global_store_byte %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ unsigned ld_u32(const void* p) {
  return __hip_atomic_load((const unsigned*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld_i32(const int* p) { return (int)ld_u32(p); }
__device__ __forceinline__ u64 ld_u64(const void* p) {
  return __hip_atomic_load((const u64*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Bulk loads: uniform base pointer (scalar registers) + 32-bit per-lane index, explicitly in the
// global address space, so the compiler emits global_load with a scalar base instead of flat
// loads with a 64-bit address per lane.
template <class T> using gptr = const T __attribute__((address_space(1)))*;
template <class T>
__device__ __forceinline__ T ldg(const T* base, unsigned idx) {
  typedef unsigned u4v __attribute__((ext_vector_type(4)));
  typedef unsigned u2v __attribute__((ext_vector_type(2)));
  static_assert(sizeof(T) == 4 || sizeof(T) == 8 || sizeof(T) == 16, "ldg element size");
  if constexpr (sizeof(T) == 16) return __builtin_bit_cast(T, ((gptr<u4v>)base)[idx]);
  else if constexpr (sizeof(T) == 8) return __builtin_bit_cast(T, ((gptr<u2v>)base)[idx]);
  else return __builtin_bit_cast(T, ((gptr<unsigned>)base)[idx]);
}
__device__ __forceinline__ int wave_id() { return wave_index(); }

// two adjacent activations (k even, k + 1) as hi/lo bf16 pairs: two 4-byte write-through stores
__device__ __forceinline__ void act_store_pair(bf16_t* base, size_t plane, int m, int k, int K, float v0, float v1) {
  size_t i = act_idx<bf16_t>(m, k, K);
  bf16_t h0 = f2bf(v0), h1 = f2bf(v1);
  bf16_t l0 = f2bf(v0 - bf2f(h0)), l1 = f2bf(v1 - bf2f(h1));
  st_u32(base + i, (unsigned)h0 | ((unsigned)h1 << 16));
  st_u32(base + plane + i, (unsigned)l0 | ((unsigned)l1 << 16));
}

// ---------------------------------------------------------------- grid barrier
// sync words: arrive[g][r] at g*64 + r, top[g] at 4096 + g, release[g] at 8192 + g*64.
struct Bar {
  unsigned* s;
  int* err;
  unsigned epoch;
  int nwg;
};
__device__ __forceinline__ bool bar_wait(const unsigned* p, unsigned ep, int* err, long long& spins) {
  while ((int)(ld_u32(p) - ep) < 0) {
    if (++spins > SPIN_LIMIT) { st_i32(err, 1); return false; }
    if ((spins & 4095) == 0 && ld_i32(err)) return false;
  }
  return true;
}
// Returns false (to every thread of the workgroup) when a wait gave up or another workgroup
// reported a failure; the caller then leaves the kernel, so the grid always drains.
// `pre` runs after this wave's stores have been acknowledged and before the wait: the place to
// request data that does not depend on other workgroups (weights of the next phase).
template <class F, class G>
__device__ __forceinline__ bool grid_barrier(Bar& b, F&& pre, G&& post) {
  __shared__ int s_fail;
  const unsigned ep = ++b.epoch;
  pre();                           // requests that depend on no other workgroup (next phase's weights)
  __builtin_amdgcn_s_waitcnt(0);   // this wave's stores have been acknowledged (and the requests have landed)
  post();
  __syncthreads();
  if (threadIdx.x < 64) {
    const int wg = blockIdx.x, g = wg / GS, r = wg % GS, ng = (b.nwg + GS - 1) / GS;
    const int gsize = min(GS, b.nwg - g * GS);
    const int lane = threadIdx.x;
    long long spins = 0;
    bool ok = true;
    if (r != 0) {
      if (lane == 0) st_u32(b.s + g * 64 + r, ep);
      ok = bar_wait(b.s + 8192 + g * 64, ep, b.err, spins);
    } else {
      // group leader: wait for the members, publish, wait for all leaders, release the members
      if (lane > 0 && lane < gsize) ok = bar_wait(b.s + g * 64 + lane, ep, b.err, spins);
      if (__all(ok)) {
        if (lane == 0) st_u32(b.s + 4096 + g, ep);
        if (lane < ng) ok = bar_wait(b.s + 4096 + lane, ep, b.err, spins);
      }
      if (lane == 0) st_u32(b.s + 8192 + g * 64, ep);
    }
    ok = __all(ok);
    if (lane == 0) s_fail = ok ? 0 : 1;
  }
  __syncthreads();
  return s_fail == 0;
}

__device__ __forceinline__ bool grid_barrier(Bar& b) {
  return grid_barrier(b, [] {}, [] {});
}

// Optional per-phase timing of workgroup 0 (100 MHz wall clock ticks), for tuning.
enum { PH_EMBED = 0, PH_NORM, PH_QKV, PH_ATTN, PH_OPROJ, PH_FFN1, PH_FFN2, PH_LMHEAD, PH_VERIFIER, PH_DECIDE, PH_FINISH,
       PH_BARRIER, PH_FENCE, PH_COUNT };
struct Prof {
  unsigned long long* p;
  unsigned long long last;
  __device__ __forceinline__ void tick(int idx) {
    if (p && blockIdx.x == 0 && threadIdx.x == 0) {
      unsigned long long t = wall_clock64();
      p[idx] += t - last;
      p[64 + idx] += 1;
      last = t;
    }
  }
};

// block reductions over the 8 waves of a workgroup (result broadcast); red = 8 floats of LDS
__device__ __forceinline__ float block_sum8(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = red[0];
#pragma unroll
  for (int q = 1; q < NWV; ++q) s += red[q];
  return s;
}
__device__ __forceinline__ float block_max8(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = red[0];
#pragma unroll
  for (int q = 1; q < NWV; ++q) s = fmaxf(s, red[q]);
  return s;
}

// ---------------------------------------------------------------- verifier partials
__device__ __forceinline__ void phase_verifier(const MegaParams& P, int B, float* smem, int wg, int nwg) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int d = P.draft.md.d, H = P.ver_d_hidden;
  const float* hf = P.draft.hf;
  if (H == 0) {
    if (wg == 0)
      for (int m = w; m < B; m += NWV) {
        float acc = 0.f;
        for (int k = lane; k < d; k += 64) acc += P.v_w2[k] * hf[(size_t)m * d + k];
        acc = wave_sum(acc);
        if (lane == 0) st_f32(P.ver_part + m, acc);
      }
    return;
  }
  for (int c = wg; c < P.ver_chunks; c += nwg) {
    const int j = c * NWV + w;
    for (int m = 0; m < B; ++m) {
      float cv = 0.f;
      if (j < H) {
        float acc = 0.f;
        for (int k = lane; k < d; k += 64) acc += P.v_w1[(size_t)j * d + k] * hf[(size_t)m * d + k];
        acc = wave_sum(acc) + P.v_b1[j];
        cv = fmaxf(acc, 0.f) * P.v_w2[j];
      }
      if (lane == 0) smem[w * B + m] = cv;
    }
    __syncthreads();
    for (int m = threadIdx.x; m < B; m += NT) {
      float s = 0.f;
#pragma unroll
      for (int q = 0; q < NWV; ++q) s += smem[q * B + m];
      st_f32(P.ver_part + (size_t)c * B + m, s);
    }
    __syncthreads();
  }
}

__device__ __forceinline__ u64 merge_partials_c(const u64* part, int n_part, int Mpad, int m, int lane) {
  u64 k = 0;
  for (int i = lane; i < n_part; i += 64) k = umax64(k, ld_u64(part + (size_t)i * Mpad + m));
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) k = umax64(k, shfl_xor_u64(k, o));
  return k;
}

// ---------------------------------------------------------------- decide (workgroup 0)
// accept <=> sigmoid(logit) >= tau in float32; rejected rows listed in ascending order.
__device__ __forceinline__ void decide(const MegaParams& P, const MegaOut& out, int nwg, float* smem) {
  int* s_tok = reinterpret_cast<int*>(smem);          // [1024]
  int* s_rej = s_tok + 1024;                           // [1024]
  int* s_cnt = s_rej + 1024;                           // [8]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int B = out.B;
  const MegaModel& D = P.draft;
  const MegaModel& T = P.target;
  for (int m = w; m < B; m += NWV) {
    u64 k = merge_partials_c(D.am_part, nwg, P.rows_alloc, m, lane);
    if (lane == 0) s_tok[m] = key_index(k);
  }
  __syncthreads();
  const float tau = *P.tau;
  int base = 0;
  for (int b0 = 0; b0 < B; b0 += NT) {
    const int b = b0 + tid;
    const bool active = b < B;
    float score = 0.f;
    bool acc = true;
    if (active) {
      float z = P.v_b2[0];
      for (int c = 0; c < P.ver_chunks; ++c) z += P.ver_part[(size_t)c * B + b];
      score = 1.0f / (1.0f + expf(-z));
      acc = score >= tau;
    }
    const bool rej = active && !acc;
    const u64 mask = __ballot(rej);
    const int rank = __popcll(mask & ((1ull << lane) - 1ull));
    __syncthreads();
    if (lane == 0) s_cnt[w] = __popcll(mask);
    __syncthreads();
    int off = base, total = 0;
    for (int q = 0; q < NWV; ++q) {
      int c = s_cnt[q];
      if (q < w) off += c;
      total += c;
    }
    if (rej) s_rej[off + rank] = b;
    if (active) {
      int dt = s_tok[b];
      P.draft_tok[b] = dt;
      P.score[b] = score;
      P.accept[b] = acc ? 1 : 0;
      P.committed[b] = acc ? dt : -1;
      if (out.o_draft_tok) out.o_draft_tok[b] = dt;
      if (out.o_score) out.o_score[b] = score;
      if (out.o_accept) out.o_accept[b] = acc ? 1 : 0;
    }
    base += total;
  }
  __syncthreads();
  const int R = base;
  for (int i = tid; i < R; i += NT) {
    int b = s_rej[i];
    P.rej_idx[i] = b;
    if (out.o_rej_idx) out.o_rej_idx[i] = b;
    st_i32(T.rd_b + i, b);
    st_i32(T.rd_tok + i, P.st.last_tok[b]);
    st_i32(T.rd_pos + i, P.st.len_q[b]);
    st_i32(T.rd_slot + i, P.st.len_p[b]);
  }
  if (tid == 0) {
    st_i32(P.n_rej, R);
    st_i32(T.rd_n, R);
    if (out.o_n_rej) *out.o_n_rej = R;
  }
  __syncthreads();
}

// ---------------------------------------------------------------- finish (workgroup 0)
__device__ __forceinline__ void finish(const MegaParams& P, const MegaOut& out, int R, int nwg, float* smem) {
  int* s_commit = reinterpret_cast<int*>(smem);        // [1024]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int B = out.B;
  const MegaModel& D = P.draft;
  for (int b = tid; b < B; b += NT) s_commit[b] = P.committed[b];
  __syncthreads();
  for (int i = w; i < R; i += NWV) {
    u64 k = merge_partials_c(P.target.am_part, nwg, P.rows_alloc, i, lane);
    if (lane == 0) s_commit[P.rej_idx[i]] = key_index(k);
  }
  __syncthreads();
  const long long g = P.st.counters[3];
  for (int b = tid; b < B; b += NT) {
    int c = s_commit[b];
    bool acc = P.accept[b] != 0;
    P.committed[b] = c;
    P.st.last_tok[b] = c;
    int lq = P.st.len_q[b] + 1;
    P.st.len_q[b] = lq;
    if (!acc) {
      P.st.len_p[b] += 1;
      P.st.n_target_calls[b] += 1;
    }
    if (out.o_committed) out.o_committed[b] = c;
    if (out.n_tokens > 0 && g < out.n_tokens) {
      size_t o = (size_t)b * out.n_tokens + (size_t)g;
      if (out.g_tok) out.g_tok[o] = c;
      if (out.g_accept) out.g_accept[o] = acc ? 1 : 0;
      if (out.g_score) out.g_score[o] = P.score[b];
      if (out.g_draft_tok) out.g_draft_tok[o] = P.draft_tok[b];
    }
    st_i32(D.rd_b + b, b);
    st_i32(D.rd_tok + b, c);
    st_i32(D.rd_pos + b, lq);
    st_i32(D.rd_slot + b, lq);
  }
  if (tid == 0) {
    st_i32(D.rd_n, B);
    P.st.counters[0] += 1;
    P.st.counters[1] += (R > 0) ? 1 : 0;
    P.st.counters[2] += R;
    P.st.counters[3] = g + 1;
  }
  __syncthreads();
}

__device__ __forceinline__ void act_store_pair1(bf16_t* base, size_t plane, int m, int k, int K, float v0, float v1) {
  size_t i = act_idx<bf16_t>(m, k, K);
  unsigned hi, lo;
  split2(v0, v1, hi, lo);
  st_u32(base + i, hi);
  st_u32(base + plane + i, lo);
}

// embedding for at most 16 rows: one wave per 16-column tile
__device__ __forceinline__ void phase_embed1(const MegaModel& M, int n_rows, int wg, int nwg) {
  const int d = M.md.d, dh = M.md.dh, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const bf16_t* E = (const bf16_t*)M.tok_emb;
  const bf16_t* P = (const bf16_t*)M.pos_emb;
  const int n_tiles = (d + 15) / 16, m_l = lane & 15, grp = lane >> 4;
  int tok[4], pos[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int m = grp * 4 + v;
    tok[v] = m < n_rows ? min(max(ld_i32(M.rd_tok + m), 0), M.md.V - 1) : 0;
    pos[v] = m < n_rows ? min(max(ld_i32(M.rd_pos + m), 0), M.md.max_pos - 1) : 0;
  }
  for (int nt = wg * NWV + w; nt < n_tiles; nt += nwg * NWV) {
    const int n = nt * 16 + m_l;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int m = grp * 4 + v;
      const bool ok = m < n_rows && n < d;
      float val = 0.f;
      if (ok) {
        val = bf2f(E[(size_t)tok[v] * d + n]);
        if (P) val += bf2f(P[(size_t)pos[v] * d + n]);
        st_f32(M.h0 + (size_t)m * d + n, val);
      }
    }
  }
  if (M.md.arch == 1 && wg == nwg - 1) {
    for (int i = threadIdx.x; i < n_rows * (dh / 2); i += NT) {
      const int r = i / (dh / 2), j = i % (dh / 2);
      const int p = ld_i32(M.rd_pos + r);
      double inv = pow((double)M.md.theta, -2.0 * (double)j / (double)dh);
      double ang = (double)p * inv;
      st_f32(M.rope + (size_t)r * dh + 2 * j, (float)cos(ang));
      st_f32(M.rope + (size_t)r * dh + 2 * j + 1, (float)sin(ang));
    }
  }
}

// ---------------------------------------------------------------- embed
__device__ __forceinline__ void phase_embed(const MegaModel& M, int n_rows, int wg, int nwg) {
  const int d = M.md.d, dh = M.md.dh;
  const bf16_t* E = (const bf16_t*)M.tok_emb;
  const bf16_t* P = (const bf16_t*)M.pos_emb;
  for (int r = wg; r < n_rows; r += nwg) {
    int tok = ld_i32(M.rd_tok + r), pos = ld_i32(M.rd_pos + r);
    tok = min(max(tok, 0), M.md.V - 1);
    const int ppos = min(max(pos, 0), M.md.max_pos - 1);
    const bf16_t* e = E + (size_t)tok * d;
    const bf16_t* p = P ? P + (size_t)ppos * d : nullptr;
    for (int k = threadIdx.x; k < d; k += NT) {
      float v = bf2f(e[k]);
      if (p) v += bf2f(p[k]);
      st_f32(M.h0 + (size_t)r * d + k, v);
    }
    if (M.md.arch == 1 && (int)threadIdx.x < dh / 2) {
      double inv = pow((double)M.md.theta, -2.0 * (double)threadIdx.x / (double)dh);
      double ang = (double)pos * inv;
      st_f32(M.rope + (size_t)r * dh + 2 * threadIdx.x, (float)cos(ang));
      st_f32(M.rope + (size_t)r * dh + 2 * threadIdx.x + 1, (float)sin(ang));
    }
  }
}

// ---------------------------------------------------------------- norm
// One row per workgroup; two-pass statistics; output as hi/lo operand tiles (+ optional float32 copy).
__device__ __forceinline__ void phase_norm(int arch, const float* h, const float* g, const float* b, float eps, int d, int n_rows,
                           bf16_t* act, size_t plane, float* f32_out, float* smem, int wg, int nwg) {
  for (int r = wg; r < n_rows; r += nwg) {
    const float* x = h + (size_t)r * d;
    float v[8][2];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int k = 2 * threadIdx.x + i * 2 * NT;
      float2 t = k < d ? *reinterpret_cast<const float2*>(x + k) : make_float2(0.f, 0.f);
      v[i][0] = t.x; v[i][1] = t.y;
      sum += t.x + t.y;
    }
    float mean = 0.f;
    if (arch == 0) mean = block_sum8(sum, smem) / (float)d;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int k = 2 * threadIdx.x + i * 2 * NT;
      if (k < d) {
        float c0 = v[i][0] - mean, c1 = v[i][1] - mean;
        sq += c0 * c0 + c1 * c1;
      }
    }
    float var = block_sum8(sq, smem) / (float)d;
    float rstd = 1.0f / sqrtf(var + eps);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int k = 2 * threadIdx.x + i * 2 * NT;
      if (k < d) {
        float o0 = (v[i][0] - mean) * rstd * g[k], o1 = (v[i][1] - mean) * rstd * g[k + 1];
        if (arch == 0) { o0 += b[k]; o1 += b[k + 1]; }
        act_store_pair(act, plane, r, k, d, o0, o1);
        if (f32_out) { st_f32(f32_out + (size_t)r * d + k, o0); st_f32(f32_out + (size_t)r * d + k + 1, o1); }
      }
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------- attention
// One work item = (row, KV head): rotary on q and the new k, append k/v, scores over all cached
// keys, softmax, weighted values, for the G query heads sharing the KV head.
template <int DH, int G>
__device__ __forceinline__ void phase_attn(const MegaModel& M, int layer, int n_rows, int max_seq, int max_batch, float* smem, int wg,
                           int nwg) {
  const ModelDims& md = M.md;
  float* qs = smem;                    // [G][DH]
  float* knew = qs + G * DH;           // [DH]
  float* vnew = knew + DH;             // [DH]
  float* red = vnew + DH;              // [8][G][DH]
  float* s_inv = red + NWV * G * DH;   // [8]
  float* s8 = s_inv + 8;               // [8]
  float* sc = s8 + 8;                  // [G][max_seq]
  const int tid = threadIdx.x, lane = tid & 63, w = wave_id();
  const int S = max_seq, KVH = md.KVH, H = md.H;
  const bool use_rope = md.arch == 1;
  const float scale = 1.0f / sqrtf((float)DH);
  constexpr int HALF = DH / 2;
  constexpr int EPL = 8, LPK = DH / EPL, KPW = 64 / LPK;
  const int chunk = lane % LPK, kin = lane / LPK;
  const float* Y = M.y + M.y_stride * layer;
  bf16_t* AO = M.ao + M.ao_stride * layer;
  const int n_items = n_rows * KVH;
  for (int it = wg; it < n_items; it += nwg) {
    const int r = it / KVH, kvh = it % KVH;
    const int b = min(max(ld_i32(M.rd_b + r), 0), max_batch - 1);
    const int slot = min(max(ld_i32(M.rd_slot + r), 0), max_seq - 1), nk = slot + 1;
    const float* y = Y + (size_t)r * md.dqkv;
    const float* cs = M.rope + (size_t)r * DH;
    for (int idx = tid; idx < G * DH; idx += NT) {
      int g = idx / DH, i = idx % DH;
      const float* qh = y + (size_t)(kvh * G + g) * DH;
      float val = qh[i];
      if (use_rope) {
        int j = i < HALF ? i : i - HALF;
        float c = cs[2 * j], sn = cs[2 * j + 1];
        val = i < HALF ? qh[i] * c - qh[i + HALF] * sn : qh[i] * c + qh[i - HALF] * sn;
      }
      qs[idx] = val * scale;
    }
    bf16_t* Kc = (bf16_t*)M.kcache + M.layer_stride * layer + ((size_t)b * KVH + kvh) * (size_t)S * DH;
    bf16_t* Vc = (bf16_t*)M.vcache + M.layer_stride * layer + ((size_t)b * KVH + kvh) * (size_t)S * DH;
    for (int i = tid; i < DH; i += NT) {
      const float* kh = y + (size_t)(H + kvh) * DH;
      const float* vh = y + (size_t)(H + KVH + kvh) * DH;
      float kv = kh[i];
      if (use_rope) {
        int j = i < HALF ? i : i - HALF;
        float c = cs[2 * j], sn = cs[2 * j + 1];
        kv = i < HALF ? kh[i] * c - kh[i + HALF] * sn : kh[i] * c + kh[i - HALF] * sn;
      }
      bf16_t kt = f2bf(kv), vt = f2bf(vh[i]);
      st_u16(Kc + (size_t)slot * DH + i, kt);
      st_u16(Vc + (size_t)slot * DH + i, vt);
      knew[i] = bf2f(kt);
      vnew[i] = bf2f(vt);
    }
    __syncthreads();
    float qreg[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < EPL; ++e) qreg[g][e] = qs[g * DH + chunk * EPL + e];
    for (int key0 = w * KPW; key0 < nk; key0 += NWV * KPW) {
      int key = key0 + kin;
      float kv[EPL];
      if (key < slot) {
        uint4 raw = ldg(reinterpret_cast<const uint4*>(Kc), (unsigned)((key * DH + chunk * EPL) >> 3));
        const bf16_t* t = reinterpret_cast<const bf16_t*>(&raw);
#pragma unroll
        for (int e = 0; e < EPL; ++e) kv[e] = bf2f(t[e]);
      } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) kv[e] = (key == slot) ? knew[chunk * EPL + e] : 0.f;
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float p = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) p += qreg[g][e] * kv[e];
#pragma unroll
        for (int o = 1; o < LPK; o <<= 1) p += __shfl_xor(p, o);
        if (chunk == 0 && key < nk) sc[g * S + key] = p;
      }
    }
    __syncthreads();
    for (int g = 0; g < G; ++g) {
      float mx = -INFINITY;
      for (int k = tid; k < nk; k += NT) mx = fmaxf(mx, sc[g * S + k]);
      mx = block_max8(mx, s8);
      float sum = 0.f;
      for (int k = tid; k < nk; k += NT) {
        float e = expf(sc[g * S + k] - mx);
        sc[g * S + k] = e;
        sum += e;
      }
      sum = block_sum8(sum, s8);
      if (tid == 0) s_inv[g] = 1.0f / sum;
    }
    __syncthreads();
    float acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    for (int key0 = w * KPW; key0 < nk; key0 += NWV * KPW) {
      int key = key0 + kin;
      float vv[EPL];
      if (key < slot) {
        uint4 raw = ldg(reinterpret_cast<const uint4*>(Vc), (unsigned)((key * DH + chunk * EPL) >> 3));
        const bf16_t* t = reinterpret_cast<const bf16_t*>(&raw);
#pragma unroll
        for (int e = 0; e < EPL; ++e) vv[e] = bf2f(t[e]);
      } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) vv[e] = (key == slot) ? vnew[chunk * EPL + e] : 0.f;
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float p = key < nk ? sc[g * S + key] : 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] += p * vv[e];
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        float v = acc[g][e];
#pragma unroll
        for (int o = LPK; o < 64; o <<= 1) v += __shfl_xor(v, o);
        if (kin == 0) red[(w * G + g) * DH + chunk * EPL + e] = v;
      }
    __syncthreads();
    for (int i2 = tid; i2 < G * DH / 2; i2 += NT) {
      const int idx = 2 * i2, g = idx / DH;
      float o0 = red[idx], o1 = red[idx + 1];
#pragma unroll
      for (int q = 1; q < NWV; ++q) { o0 += red[q * G * DH + idx]; o1 += red[q * G * DH + idx + 1]; }
      o0 *= s_inv[g]; o1 *= s_inv[g];
      act_store_pair(AO, M.pl_a, r, kvh * G * DH + idx, H * DH, o0, o1);
    }
    __syncthreads();
  }
}

__device__ __forceinline__ void attn_dispatch(const MegaModel& M, int layer, int n_rows, int max_seq, int max_batch, float* smem, int wg,
                              int nwg) {
  const int G = M.md.H / M.md.KVH;
  if (M.md.dh == 64) {
    switch (G) {
      case 1: phase_attn<64, 1>(M, layer, n_rows, max_seq, max_batch, smem, wg, nwg); break;
      case 2: phase_attn<64, 2>(M, layer, n_rows, max_seq, max_batch, smem, wg, nwg); break;
      case 4: phase_attn<64, 4>(M, layer, n_rows, max_seq, max_batch, smem, wg, nwg); break;
      default: phase_attn<64, 8>(M, layer, n_rows, max_seq, max_batch, smem, wg, nwg); break;
    }
  } else {
    switch (G) {
      case 1: phase_attn<128, 1>(M, layer, n_rows, max_seq, max_batch, smem, wg, nwg); break;
      case 2: phase_attn<128, 2>(M, layer, n_rows, max_seq, max_batch, smem, wg, nwg); break;
      case 4: phase_attn<128, 4>(M, layer, n_rows, max_seq, max_batch, smem, wg, nwg); break;
      default: phase_attn<128, 8>(M, layer, n_rows, max_seq, max_batch, smem, wg, nwg); break;
    }
  }
}

// ---------------------------------------------------------------- LM head + sampling partials
template <int MT>
__device__ __forceinline__ void phase_lmhead(const MegaModel& M, int n_rows, const SamplerArgs& sa, int Mpad, float* logits_out,
                             float* smem, int wg, int nwg) {
  u64* sbest = reinterpret_cast<u64*>(smem);   // [8][MT*16]
  const int lane = threadIdx.x & 63, w = wave_id();
  const int V = M.md.V, Kt = (M.md.d + 31) / 32, n_tiles = (V + 15) / 16;
  const int tpw = (n_tiles + nwg - 1) / nwg;
  const int t0 = wg * tpw, t1 = min(t0 + tpw, n_tiles);
  const uint4* __restrict__ Wp = (const uint4*)M.lm_head;
  const uint4* __restrict__ Xp = (const uint4*)M.hfn;
  const uint4* __restrict__ Xl = Xp + M.pl_d / 8;
  for (int m0 = 0; m0 < n_rows; m0 += MT * 16) {
    const int mt_act = min(MT, (n_rows - m0 + 15) >> 4);
    const int mtile0 = m0 >> 4;
    u64 best[MT][4];
    int rb[MT][4], rt[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        best[mt][v] = 0;
        int m = m0 + mt * 16 + (lane >> 4) * 4 + v;
        rb[mt][v] = m < n_rows ? ld_i32(M.rd_b + m) : 0;
        rt[mt][v] = m < n_rows ? ld_i32(M.rd_pos + m) + 1 : 0;
      }
    for (int nt = t0 + w; nt < t1; nt += NWV) {
      f32x4 acc[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      constexpr int U = 4;
      for (int kt = 0; kt < Kt; kt += U) {
        uint4 wv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) wv[u] = ldg(Wp + (size_t)nt * Kt * 64, (unsigned)(min(kt + u, Kt - 1) * 64 + lane));
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (kt + u < Kt) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              if (mt < mt_act) {
                uint4 xv = ldg(Xp + (size_t)(mtile0 + mt) * Kt * 64, (unsigned)((kt + u) * 64 + lane));
                uint4 xl = ldg(Xl + (size_t)(mtile0 + mt) * Kt * 64, (unsigned)((kt + u) * 64 + lane));
                acc[mt] = mfma_bf16(xv, wv[u], acc[mt]);
                acc[mt] = mfma_bf16(xl, wv[u], acc[mt]);
              }
          }
      }
      const int n = nt * 16 + (lane & 15);
      if (n < V) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          if (mt < mt_act) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              int m = m0 + mt * 16 + (lane >> 4) * 4 + v;
              if (m < n_rows) {
                float logit = acc[mt][v];
                if (logits_out) logits_out[(size_t)m * V + n] = logit;
                best[mt][v] = umax64(best[mt][v], sample_key(logit, sa, rb[mt][v], rt[mt][v], n));
              }
            }
          }
      }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        u64 k = best[mt][v];
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) k = umax64(k, shfl_xor_u64(k, o));
        if ((lane & 15) == 0) sbest[w * MT * 16 + mt * 16 + (lane >> 4) * 4 + v] = k;
      }
    __syncthreads();
    for (int i = threadIdx.x; i < MT * 16; i += NT) {
      u64 k = sbest[i];
#pragma unroll
      for (int q = 1; q < NWV; ++q) k = umax64(k, sbest[q * MT * 16 + i]);
      if (m0 + i < Mpad) st_u64(M.am_part + (size_t)wg * Mpad + m0 + i, k);
    }
    __syncthreads();
  }
}

}  // namespace
}  // namespace sprinter
