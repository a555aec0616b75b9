// Persistent decode kernel (bf16 mode): n_steps whole SPRINTER decode steps in one
// cooperative launch, one workgroup of 512 threads per compute unit.
//
// Per step (Alg. 2 of the paper, B rows in lock step):
//   draft forward -> LM head + Gumbel-max partials + verifier partials | barrier |
//   workgroup 0: arg-max merge, sigmoid, threshold, ballot compaction of rejected rows | barrier |
//   if R > 0: target forward on the R rows -> LM head partials | barrier |
//   workgroup 0: merge, scatter back, advance state | barrier
// A model forward is a sequence of phases (embed, norm, QKV, attention, O-proj, norm, FFN-up,
// FFN-down per layer, final norm, LM head) with a grid barrier between dependent phases.
//
// Memory protocol between workgroups (the 8 XCDs have separate, mutually non-coherent L2s):
//   * everything another workgroup will read is stored write-through with device scope
//     (global_store ... sc1), control words are read with device-scope loads;
//   * bulk activations live in buffers that are written once per step and read, with ordinary
//     cached loads, only after the barrier that follows their producer phase; one device-scope
//     fence per step (cache write-back + invalidate) makes the addresses reusable by the next step;
//   * the barrier itself is a tree of flags (members -> group leader -> all leaders -> members)
//     built from device-scope stores and polling loads only: no read-modify-write atomics and
//     no cache flushes on the critical path.
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
__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

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
      p[16 + idx] += 1;
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

// ---------------------------------------------------------------- GEMM
struct GArgs {
  const uint4* W; const uint4* W2; const uint4* X; size_t x_plane16;   // plane distance in 16-byte units
  int N, Kt, n_tiles;
  const float* bias; const float* resid; float* out_f32; int ldo;
  bf16_t* out_act; int out_K; size_t out_plane;
};

// D[m][n] += X[m][k] W[n][k] on v_mfma_f32_16x16x32_bf16; accumulator lane l holds n = l%16, m = (l/16)*4 + v.
// 8 waves = (8/KW) column tiles x KW-way split of K, partial sums combined through LDS in fixed order.
template <int MT, int EPI>
__device__ __forceinline__ void phase_gemm(const GArgs& a, int n_rows, float* smem, int wg, int nwg) {
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int KW = MT <= 2 ? 8 : (MT == 4 ? 4 : 2);
  constexpr int NW = NWV / KW;
  constexpr int NI = MT * 4;
  constexpr int NI2 = NI * (DUAL ? 2 : 1);
  constexpr int U = 4;
  const int lane = threadIdx.x & 63, w = wave_id();
  const int kw = w % KW, ng = w / KW;
  const int Kt = a.Kt;
  const uint4* Xl = a.X + a.x_plane16;
  const int n_groups = (a.n_tiles + NW - 1) / NW;
  for (int vb = wg; vb < n_groups; vb += nwg) {
    const int nt_raw = vb * NW + ng;
    const int nt = min(nt_raw, a.n_tiles - 1);
    for (int m0 = 0; m0 < n_rows; m0 += MT * 16) {
      const int mt_act = min(MT, (n_rows - m0 + 15) >> 4);
      const int mtile0 = m0 >> 4;
      f32x4 acc[MT], acc2[DUAL ? MT : 1];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        acc[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
        if (DUAL) acc2[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      }
      for (int kt = kw; kt < Kt; kt += KW * U) {
        uint4 wv[U], wv2[DUAL ? U : 1];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          int kc = min(kt + u * KW, Kt - 1);
          wv[u] = ldg(a.W + (size_t)nt * Kt * 64, (unsigned)(kc * 64 + lane));
          if (DUAL) wv2[u] = ldg(a.W2 + (size_t)nt * Kt * 64, (unsigned)(kc * 64 + lane));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          int kc = kt + u * KW;
          if (kc < Kt) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
              if (mt < mt_act) {
                uint4 xv = ldg(a.X + (size_t)(mtile0 + mt) * Kt * 64, (unsigned)(kc * 64 + lane));
                uint4 xl = ldg(Xl + (size_t)(mtile0 + mt) * Kt * 64, (unsigned)(kc * 64 + lane));
                acc[mt] = mfma_bf16(xv, wv[u], acc[mt]);
                acc[mt] = mfma_bf16(xl, wv[u], acc[mt]);
                if (DUAL) {
                  acc2[mt] = mfma_bf16(xv, wv2[u], acc2[mt]);
                  acc2[mt] = mfma_bf16(xl, wv2[u], acc2[mt]);
                }
              }
            }
          }
        }
      }
      if (kw > 0) {
        float* dst = smem + (size_t)(ng * (KW - 1) + kw - 1) * NI2 * 64;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            dst[(mt * 4 + v) * 64 + lane] = acc[mt][v];
            if (DUAL) dst[(NI + mt * 4 + v) * 64 + lane] = acc2[mt][v];
          }
      }
      __syncthreads();
      if (kw == 0) {
#pragma unroll
        for (int q = 1; q < KW; ++q) {
          const float* src = smem + (size_t)(ng * (KW - 1) + q - 1) * NI2 * 64;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              acc[mt][v] += src[(mt * 4 + v) * 64 + lane];
              if (DUAL) acc2[mt][v] += src[(NI + mt * 4 + v) * 64 + lane];
            }
        }
        const int n = nt_raw * 16 + (lane & 15);
        const bool n_ok = nt_raw < a.n_tiles && n < a.N;
        const float bias = (a.bias && n_ok) ? a.bias[n] : 0.f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          if (mt < mt_act) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const int m = m0 + mt * 16 + (lane >> 4) * 4 + v;
              const bool ok = n_ok && m < n_rows;
              if (EPI == EPI_F32) {
                if (ok) st_f32(a.out_f32 + (size_t)m * a.ldo + n, acc[mt][v] + bias);
              } else if (EPI == EPI_RESID) {
                if (ok) st_f32(a.out_f32 + (size_t)m * a.ldo + n, a.resid[(size_t)m * a.ldo + n] + acc[mt][v] + bias);
              } else {
                float val = (EPI == EPI_GELU) ? gelu_tanh(acc[mt][v] + bias) : silu(acc[mt][v]) * acc2[mt][v];
                float nb = __shfl_xor(val, 1);           // the neighbouring column's value
                if (ok && !(lane & 1)) act_store_pair(a.out_act, a.out_plane, m, n, a.out_K, val, nb);
              }
            }
          }
        }
      }
      __syncthreads();
    }
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

// =====================================================================================
// M <= 16 path (one row tile): layer norms are folded into the consuming GEMM.
// Producers of the residual stream (embedding, O-proj, FFN-down) leave, per 16-column tile,
// the per-row sum and sum of squares; a consumer wave adds these up in a fixed order, then
// normalises exactly the activation fragments it needs while building its MFMA operands, so
// no separate norm phase (and no barrier for it) exists.  Weights for the first pass of a
// phase are requested before the barrier that precedes it (they depend on nothing).
// =====================================================================================
__device__ __forceinline__ void tick(int idx);
typedef float f2v __attribute__((ext_vector_type(2)));
typedef __bf16 b2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pk_bf16(float a, float b) {
  f2v v = {a, b};
  b2v h = __builtin_convertvector(v, b2v);   // v_cvt_pk_bf16_f32, round to nearest even
  return __builtin_bit_cast(unsigned, h);
}
__device__ __forceinline__ void split2(float a, float b, unsigned& hi, unsigned& lo) {
  hi = pk_bf16(a, b);
  lo = pk_bf16(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}
__device__ __forceinline__ void act_store_pair1(bf16_t* base, size_t plane, int m, int k, int K, float v0, float v1) {
  size_t i = act_idx<bf16_t>(m, k, K);
  unsigned hi, lo;
  split2(v0, v1, hi, lo);
  st_u32(base + i, hi);
  st_u32(base + plane + i, lo);
}

typedef PhaseDesc G1;

template <int EPI>
struct Pre1 {
  static constexpr int PF = (EPI == EPI_SWIGLU) ? 4 : 8;
  uint4 w[2][PF];
  uint4 w2[2][(EPI == EPI_SWIGLU) ? PF : 1];
};

// request the weight tiles of this workgroup's first pass (column tiles wg and wg + nwg)
template <int EPI>
__device__ __forceinline__ void gemm1_prefetch(const G1& a, int wg, int nwg, Pre1<EPI>& p) {
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int PF = Pre1<EPI>::PF;
  const int lane = threadIdx.x & 63, kw = wave_id();
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int nt = wg + j * nwg;
    if (nt < a.n_tiles) {
      const uint4* Wt = a.W + (size_t)nt * a.Kt * 64;
      const uint4* W2t = DUAL ? a.W2 + (size_t)nt * a.Kt * 64 : nullptr;
#pragma unroll
      for (int i = 0; i < PF; ++i) {
        const int kt = min(kw + NWV * i, a.Kt - 1);
        p.w[j][i] = ldg(Wt, (unsigned)(kt * 64 + lane));
        if (DUAL) p.w2[j][i] = ldg(W2t, (unsigned)(kt * 64 + lane));
      }
    }
  }
}

// One chunk of PF k-tiles for up to two column tiles: fetch the activation fragments, convert
// (and normalise) them tile by tile and multiply.  w0/w1 (v0/v1 for the second matrix of SwiGLU)
// are the weight tiles already requested by the caller.
template <int EPI, bool NORM, int PF>
__device__ __forceinline__ void gemm1_chunk(const G1& a, const uint4 (&w0)[PF], const uint4 (&w1)[PF],
                                            const uint4 (&v0)[PF], const uint4 (&v1)[PF], int c0, bool has1, float mean,
                                            float rstd, const float* gb, f32x4 (&acc)[2], f32x4 (&acc2)[2]) {
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  const int lane = threadIdx.x & 63, kw = wave_id();
  const int m_l = lane & 15, grp = lane >> 4;
  const int Kt = a.Kt;
  float4 ra[NORM ? PF : 1][2];
  uint4 xh[NORM ? 1 : PF], xl[NORM ? 1 : PF];
  if (NORM) {
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      const int kt = min(kw + NWV * (c0 + i), Kt - 1);
      const int k = min(kt * 32 + grp * 8, a.K - 8);
      const unsigned e4 = (unsigned)(m_l * a.K + k) >> 2;     // float4 index (K and k are multiples of 8)
      ra[i][0] = ldg(reinterpret_cast<const float4*>(a.h), e4);
      ra[i][1] = ldg(reinterpret_cast<const float4*>(a.h), e4 + 1);
    }
  } else {
    const uint4* Xl = a.X + a.x_plane16;
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      const int kt = min(kw + NWV * (c0 + i), Kt - 1);
      xh[i] = ldg(a.X, (unsigned)(kt * 64 + lane));
      xl[i] = ldg(Xl, (unsigned)(kt * 64 + lane));
    }
  }
#pragma unroll
  for (int i = 0; i < PF; ++i) {
    uint4 ah, al;
    if (NORM) {
      const int kt = min(kw + NWV * (c0 + i), Kt - 1);
      const int kreal = kt * 32 + grp * 8;
      const int k = min(kreal, a.K - 8);
      const float4 g0 = *reinterpret_cast<const float4*>(gb + k), g1 = *reinterpret_cast<const float4*>(gb + k + 4);
      const float4 b0 = *reinterpret_cast<const float4*>(gb + a.K + k), b1 = *reinterpret_cast<const float4*>(gb + a.K + k + 4);
      float x0 = (ra[i][0].x - mean) * rstd * g0.x + b0.x, x1 = (ra[i][0].y - mean) * rstd * g0.y + b0.y;
      float x2 = (ra[i][0].z - mean) * rstd * g0.z + b0.z, x3 = (ra[i][0].w - mean) * rstd * g0.w + b0.w;
      float x4 = (ra[i][1].x - mean) * rstd * g1.x + b1.x, x5 = (ra[i][1].y - mean) * rstd * g1.y + b1.y;
      float x6 = (ra[i][1].z - mean) * rstd * g1.z + b1.z, x7 = (ra[i][1].w - mean) * rstd * g1.w + b1.w;
      if (kreal + 8 > a.K) { x0 = x1 = x2 = x3 = x4 = x5 = x6 = x7 = 0.f; }   // K is a multiple of 8: all or nothing
      split2(x0, x1, ah.x, al.x);
      split2(x2, x3, ah.y, al.y);
      split2(x4, x5, ah.z, al.z);
      split2(x6, x7, ah.w, al.w);
    } else {
      ah = xh[i]; al = xl[i];
    }
    if (kw + NWV * (c0 + i) < Kt) {
      acc[0] = mfma_bf16(ah, w0[i], acc[0]);
      acc[0] = mfma_bf16(al, w0[i], acc[0]);
      if (DUAL) { acc2[0] = mfma_bf16(ah, v0[i], acc2[0]); acc2[0] = mfma_bf16(al, v0[i], acc2[0]); }
      if (has1) {
        acc[1] = mfma_bf16(ah, w1[i], acc[1]);
        acc[1] = mfma_bf16(al, w1[i], acc[1]);
        if (DUAL) { acc2[1] = mfma_bf16(ah, v1[i], acc2[1]); acc2[1] = mfma_bf16(al, v1[i], acc2[1]); }
      }
    }
  }
}

// Cross-wave sum of the partial accumulators (fixed order) and the fused epilogue; wave j
// finishes column tile j.
template <int EPI>
__device__ __forceinline__ void gemm1_finish(const G1& a, int n_rows, float* red, int nt0, int nt1, bool has1,
                                             const f32x4 (&acc)[2], const f32x4 (&acc2)[2]) {
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int NI2 = DUAL ? 8 : 4;
  const int lane = threadIdx.x & 63, kw = wave_id();
  const int m_l = lane & 15, grp = lane >> 4;
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      red[((kw * 2 + j) * NI2 + v) * 64 + lane] = acc[j][v];
      if (DUAL) red[((kw * 2 + j) * NI2 + 4 + v) * 64 + lane] = acc2[j][v];
    }
  __syncthreads();
  if (kw < 2 && (kw == 0 || has1)) {
    const int j = kw, nt = j == 0 ? nt0 : nt1;
    float r1[4], r2[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      float s = 0.f, t = 0.f;
#pragma unroll
      for (int q = 0; q < NWV; ++q) {
        s += red[((q * 2 + j) * NI2 + v) * 64 + lane];
        if (DUAL) t += red[((q * 2 + j) * NI2 + 4 + v) * 64 + lane];
      }
      r1[v] = s; r2[v] = t;
    }
    const int n = nt * 16 + m_l;
    const bool n_ok = n < a.N;
    const float bias = (a.bias && n_ok) ? ldg(a.bias, (unsigned)n) : 0.f;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int m = grp * 4 + v;
      const bool ok = n_ok && m < n_rows;
      if (EPI == EPI_F32) {
        if (ok) st_f32(a.out_f32 + (size_t)m * a.ldo + n, r1[v] + bias);
      } else if (EPI == EPI_RESID) {
        float val = ok ? ldg(a.resid, (unsigned)(m * a.ldo + n)) + r1[v] + bias : 0.f;
        if (ok) st_f32(a.out_f32 + (size_t)m * a.ldo + n, val);
        float s1 = val, s2 = val * val;
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) { s1 += __shfl_xor(s1, o); s2 += __shfl_xor(s2, o); }
        if (m_l == 0 && a.stats_out)
          st_u64(a.stats_out + ((size_t)nt * 16 + m) * 2, ((u64)__float_as_uint(s2) << 32) | __float_as_uint(s1));
      } else {
        float val = (EPI == EPI_GELU) ? gelu_tanh(r1[v] + bias) : silu(r1[v]) * r2[v];
        float nb = __shfl_xor(val, 1);
        if (ok && !(lane & 1)) act_store_pair1(a.out_act, a.out_plane, m, n, a.out_K, val, nb);
      }
    }
  }
  __syncthreads();
}

template <int EPI, bool NORM>
__device__ __forceinline__ void gemm1_run(const G1& a, int n_rows, float* smem, int wg, int nwg, Pre1<EPI>& p) {
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int PF = Pre1<EPI>::PF;
  const int lane = threadIdx.x & 63, kw = wave_id();
  const int m_l = lane & 15, grp = lane >> 4;
  const int Kt = a.Kt;
  const int nk_w = (Kt - kw + NWV - 1) / NWV;          // k tiles of this wave: kw, kw + 8, ...
  float* red = smem;                                   // [8 waves][2 tiles][8][64]
  float* gb = smem + NWV * 2 * 8 * 64;                 // [2][K] gain, offset
  float mean = 0.f, rstd = 1.f;
  if (NORM) {
    // row statistics: the producers' per-tile (sum, sum of squares) -> LDS in one batch of loads,
    // then every wave adds them up in tile order (gain / offset were parked in LDS before the barrier)
    float2* st_l = reinterpret_cast<float2*>(gb + 2 * a.K);
    const int n_ent = a.n_stat_tiles * 16;
    for (int e0 = 0; e0 < n_ent; e0 += 4 * NT) {
      float2 v[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int e = e0 + threadIdx.x + q * NT;
        v[q] = e < n_ent ? ldg(reinterpret_cast<const float2*>(a.stats_in), (unsigned)e) : make_float2(0.f, 0.f);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int e = e0 + threadIdx.x + q * NT;
        if (e < n_ent) st_l[e] = v[q];
      }
    }
    __syncthreads();
    float s1 = 0.f, s2 = 0.f;
    for (int t = grp; t < a.n_stat_tiles; t += 4) {
      float2 v = st_l[t * 16 + m_l];
      s1 += v.x; s2 += v.y;
    }
    s1 += __shfl_xor(s1, 16); s1 += __shfl_xor(s1, 32);
    s2 += __shfl_xor(s2, 16); s2 += __shfl_xor(s2, 32);
    const double invK = 1.0 / (double)a.K;
    double mu = a.arch == 0 ? (double)s1 * invK : 0.0;
    double var = (double)s2 * invK - mu * mu;
    if (var < 0.0) var = 0.0;
    mean = (float)mu;
    rstd = (float)(1.0 / sqrt(var + (double)a.eps));
  }
  tick(13);
  for (int base = wg; base < a.n_tiles; base += 2 * nwg) {
    const int nt0 = base, nt1 = base + nwg;
    const bool has1 = nt1 < a.n_tiles;
    f32x4 acc[2], acc2[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) { acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f}; acc2[j] = (f32x4){0.f, 0.f, 0.f, 0.f}; }
    int c_begin = 0;
    if (base == wg) {   // the first chunk of the first pass was requested before the barrier
      if constexpr (DUAL) gemm1_chunk<EPI, NORM, PF>(a, p.w[0], p.w[1], p.w2[0], p.w2[1], 0, has1, mean, rstd, gb, acc, acc2);
      else gemm1_chunk<EPI, NORM, PF>(a, p.w[0], p.w[1], p.w[0], p.w[1], 0, has1, mean, rstd, gb, acc, acc2);
      c_begin = PF;
    }
    for (int c0 = c_begin; c0 < nk_w; c0 += PF) {
      uint4 w0[PF], w1[PF], v0[DUAL ? PF : 1], v1[DUAL ? PF : 1];
#pragma unroll
      for (int i = 0; i < PF; ++i) {
        const int kt = min(kw + NWV * (c0 + i), Kt - 1);
        const unsigned o = (unsigned)(kt * 64 + lane);
        w0[i] = ldg(a.W + (size_t)nt0 * Kt * 64, o);
        if (DUAL) v0[i] = ldg(a.W2 + (size_t)nt0 * Kt * 64, o);
        if (has1) {
          w1[i] = ldg(a.W + (size_t)nt1 * Kt * 64, o);
          if (DUAL) v1[i] = ldg(a.W2 + (size_t)nt1 * Kt * 64, o);
        }
      }
      if constexpr (DUAL) gemm1_chunk<EPI, NORM, PF>(a, w0, w1, v0, v1, c0, has1, mean, rstd, gb, acc, acc2);
      else gemm1_chunk<EPI, NORM, PF>(a, w0, w1, w0, w1, c0, has1, mean, rstd, gb, acc, acc2);
    }
    tick(14);
    gemm1_finish<EPI>(a, n_rows, red, nt0, nt1, has1, acc, acc2);
  }
}

// embedding for the M <= 16 path: one wave per 16-column tile, leaves the tile's row statistics
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
      float s1 = val, s2 = val * val;
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) { s1 += __shfl_xor(s1, o); s2 += __shfl_xor(s2, o); }
      if (m_l == 0) st_u64(M.stats + ((size_t)nt * 16 + m) * 2, ((u64)__float_as_uint(s2) << 32) | __float_as_uint(s1));
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

// =====================================================================================
// Phase interpreter.  The host prepares, per model, the list of phases of one forward
// (PhaseDesc); the kernel walks it.  Every phase is its own non-inlined function, so each
// gets its own register allocation, and reads its descriptor with scalar loads.
// =====================================================================================
struct Shared {          // per-workgroup state kept in LDS across phase functions
  unsigned* sync;
  int* err;
  unsigned long long* prof;
  unsigned long long prof_last;
  unsigned epoch;
  int fail;
};
static __shared__ Shared sh;

__device__ __forceinline__ void tick(int idx) {
  if (sh.prof && blockIdx.x == 0 && threadIdx.x == 0) {
    unsigned long long t = wall_clock64();
    sh.prof[idx] += t - sh.prof_last;
    sh.prof[16 + idx] += 1;
    sh.prof_last = t;
  }
}

template <class F, class G>
__device__ __forceinline__ bool sbarrier(F&& pre, G&& post) {
  Bar b{sh.sync, sh.err, sh.epoch, (int)gridDim.x};
  const bool ok = grid_barrier(b, pre, [&] { tick(15); post(); });   // all threads read sh.epoch before its first __syncthreads
  if (threadIdx.x == 0) sh.epoch = b.epoch;
  tick(PH_BARRIER);
  return ok;
}
__device__ __forceinline__ bool sbarrier() { return sbarrier([] {}, [] {}); }

// uniform pointer -> scalar registers -> constant address space, so that descriptor fields are
// fetched with scalar loads (the tables are written by the host before the launch and never after)
template <class T>
__device__ __forceinline__ T load_desc(const T* p) {
  unsigned long long u = (unsigned long long)p;
  unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)u), hi = __builtin_amdgcn_readfirstlane((unsigned)(u >> 32));
  typedef const unsigned __attribute__((address_space(4)))* cptr;
  cptr c = (cptr)(((unsigned long long)hi << 32) | lo);
  static_assert(sizeof(T) % 4 == 0, "descriptor size");
  union { T t; unsigned w[sizeof(T) / 4]; } u2;
#pragma unroll
  for (unsigned i = 0; i < sizeof(T) / 4; ++i) u2.w[i] = c[i];
  return u2.t;
}
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

template <int EPI, bool NORM>
__device__ __forceinline__ bool ph_gemm1(const PhaseDesc* dp, int n_rows_, float* smem) {
  const G1 a = load_desc(dp);
  const int n_rows = uni(n_rows_), wg = blockIdx.x, nwg = gridDim.x;
  Pre1<EPI> p;
  // norm gain / offset: requested before the wait, parked in LDS after it (constants of the model)
  float4 gq[NORM ? 4 : 1], bq[NORM ? 4 : 1];
  const int n4 = a.K >> 2;
  if (!sbarrier(
          [&] {
            gemm1_prefetch<EPI>(a, wg, nwg, p);
            if (NORM) {
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const int i4 = threadIdx.x + q * NT;
                if (i4 < n4) {
                  gq[q] = ldg(reinterpret_cast<const float4*>(a.g), (unsigned)i4);
                  bq[q] = a.arch == 0 ? ldg(reinterpret_cast<const float4*>(a.b), (unsigned)i4) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
              }
            }
          },
          [&] {
            if (NORM) {
              float4* gb4 = reinterpret_cast<float4*>(smem + NWV * 2 * 8 * 64);
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const int i4 = threadIdx.x + q * NT;
                if (i4 < n4) { gb4[i4] = gq[q]; gb4[n4 + i4] = bq[q]; }
              }
            }
          }))
    return false;
  gemm1_run<EPI, NORM>(a, n_rows, smem, wg, nwg, p);
  return true;
}

template <int MT, int EPI>
__device__ __forceinline__ bool ph_gemm(const PhaseDesc* dp, int n_rows_, float* smem) {
  const PhaseDesc d = load_desc(dp);
  const int n_rows = uni(n_rows_);
  if (!sbarrier()) return false;
  GArgs a{d.W, d.W2, d.X, d.x_plane16, d.N, d.Kt, d.n_tiles, d.bias, d.resid, d.out_f32, d.ldo, d.out_act, d.out_K,
          d.out_plane};
  phase_gemm<MT, EPI>(a, n_rows, smem, blockIdx.x, gridDim.x);
  return true;
}

__device__ __forceinline__ bool ph_norm(const PhaseDesc* dp, int n_rows_, float* smem) {
  const PhaseDesc d = load_desc(dp);
  const int n_rows = uni(n_rows_);
  if (!sbarrier()) return false;
  phase_norm(d.arch, d.h, d.g, d.b, d.eps, d.K, n_rows, d.out_act, d.out_plane, d.f32_out2, smem, blockIdx.x, gridDim.x);
  return true;
}

template <int MT>
__device__ __forceinline__ void ph_embed(const MegaModel* Mp, int n_rows_) {
  const MegaModel& M = *Mp;
  const int n_rows = uni(n_rows_);
  if constexpr (MT == 1) phase_embed1(M, n_rows, blockIdx.x, gridDim.x);
  else phase_embed(M, n_rows, blockIdx.x, gridDim.x);
}

__device__ __forceinline__ bool ph_attn(const MegaModel* Mp, int layer_, int n_rows_, int max_seq, int max_batch, float* smem) {
  const MegaModel& M = *Mp;
  const int n_rows = uni(n_rows_), layer = uni(layer_);
  if (!sbarrier()) return false;
  attn_dispatch(M, layer, n_rows, uni(max_seq), uni(max_batch), smem, blockIdx.x, gridDim.x);
  return true;
}

template <int MT>
__device__ __forceinline__ bool ph_lmhead(const MegaParams* Pp, const MegaModel* Mp, int n_rows_, unsigned stream_id,
                                       float* logits_out, float* hidden_out, float* smem) {
  const MegaParams& P = *Pp;
  const MegaModel& M = *Mp;
  const int n_rows = uni(n_rows_), wg = blockIdx.x, nwg = gridDim.x;
  if (!sbarrier()) return false;
  SamplerArgs sa{P.seed_lo, P.seed_hi, stream_id, P.inv_temperature};
  phase_lmhead<MT>(M, n_rows, sa, P.rows_alloc, logits_out, smem, wg, nwg);
  if (hidden_out)
    for (size_t i = (size_t)wg * NT + threadIdx.x; i < (size_t)n_rows * M.md.d; i += (size_t)nwg * NT)
      hidden_out[i] = M.hf[i];
  return true;
}

__device__ __forceinline__ void ph_verifier(const MegaParams* Pp, int B, float* smem) {
  phase_verifier(*Pp, uni(B), smem, blockIdx.x, gridDim.x);
}
__device__ __forceinline__ void ph_decide(const MegaParams* Pp, const MegaOut* out, float* smem) {
  decide(*Pp, *out, gridDim.x, smem);
}
__device__ __forceinline__ void ph_finish(const MegaParams* Pp, const MegaOut* out, int R, float* smem) {
  finish(*Pp, *out, uni(R), gridDim.x, smem);
}

template <int MT>
__device__ __forceinline__ bool run_gemm(const PhaseDesc* dp, int epi, int fused, int n_rows, float* smem) {
  if constexpr (MT == 1) {
    switch (epi) {
      case EPI_F32: return fused ? ph_gemm1<EPI_F32, true>(dp, n_rows, smem) : ph_gemm1<EPI_F32, false>(dp, n_rows, smem);
      case EPI_RESID: return ph_gemm1<EPI_RESID, false>(dp, n_rows, smem);
      case EPI_GELU: return ph_gemm1<EPI_GELU, true>(dp, n_rows, smem);
      default: return ph_gemm1<EPI_SWIGLU, true>(dp, n_rows, smem);
    }
  } else {
    (void)fused;
    switch (epi) {
      case EPI_F32: return ph_gemm<MT, EPI_F32>(dp, n_rows, smem);
      case EPI_RESID: return ph_gemm<MT, EPI_RESID>(dp, n_rows, smem);
      case EPI_GELU: return ph_gemm<MT, EPI_GELU>(dp, n_rows, smem);
      default: return ph_gemm<MT, EPI_SWIGLU>(dp, n_rows, smem);
    }
  }
}

template <int MT>
__global__ __launch_bounds__(NT) void k_mega(const MegaParams* __restrict__ Pp, int n_steps, MegaOut out) {
  extern __shared__ float smem[];
  const MegaParams& P = *Pp;
  const int wg = blockIdx.x;
  if (threadIdx.x == 0) {
    sh.sync = P.sync; sh.err = P.err; sh.prof = P.prof; sh.prof_last = P.prof ? wall_clock64() : 0ull;
    sh.epoch = ld_u32(P.epoch); sh.fail = 0;
  }
  __syncthreads();
  const int B = out.B;
  for (int step = 0; step < n_steps; ++step) {
    // buffers written in the previous step are about to be rewritten and reread:
    // write back and invalidate this compute unit's view once per step
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "agent");
    tick(PH_FENCE);
    int R = 0;
    for (int which = 0; which < 2; ++which) {
      const MegaModel* M = which == 0 ? &Pp->draft : &Pp->target;
      const int n_rows = which == 0 ? B : R;
      if (which == 1 && R == 0) break;
      const PhaseDesc* ph = M->phases;
      const int n_ph = M->n_phases;
      for (int i = 0; i < n_ph; ++i) {
        const PhaseDesc* dp = ph + i;
        const int kind = dp->kind;
        bool ok = true;
        if (kind == PK_EMBED) {
          ph_embed<MT>(M, n_rows);
          tick(PH_EMBED);
        } else if (kind == PK_NORM) {
          ok = ph_norm(dp, n_rows, smem);
          tick(PH_NORM);
        } else if (kind == PK_GEMM) {
          const int epi = dp->epi, slot = dp->layer;
          ok = run_gemm<MT>(dp, epi, dp->fused_norm, n_rows, smem);
          tick(slot);
        } else if (kind == PK_ATTN) {
          ok = ph_attn(M, dp->layer, n_rows, P.max_seq, P.max_batch, smem);
          tick(PH_ATTN);
        } else {
          ok = ph_lmhead<MT>(Pp, M, n_rows, (unsigned)which, which == 0 ? out.o_draft_logits : out.o_target_logits,
                             which == 0 ? out.o_draft_hidden : out.o_target_hidden, smem);
          tick(PH_LMHEAD);
        }
        if (!ok) return;
      }
      if (which == 0) {
        ph_verifier(Pp, B, smem);
        tick(PH_VERIFIER);
        if (!sbarrier()) return;
        if (wg == 0) ph_decide(Pp, &out, smem);
        tick(PH_DECIDE);
        if (!sbarrier()) return;
        R = min(max(ld_i32(P.n_rej), 0), B);
      } else {
        if (!sbarrier()) return;
      }
    }
    if (wg == 0) ph_finish(Pp, &out, R, smem);
    tick(PH_FINISH);
    if (!sbarrier()) return;
  }
  if (wg == 0 && threadIdx.x == 0) st_u32(P.epoch, sh.epoch);
}

template <int MT>
hipError_t launch_t(const MegaParams* dp, int n_steps, const MegaOut& out, size_t smem, int grid, hipStream_t s) {
  MegaOut o = out;
  void* args[] = {(void*)&dp, (void*)&n_steps, (void*)&o};
  return hipLaunchCooperativeKernel((const void*)k_mega<MT>, dim3(grid), dim3(NT), args, (unsigned)smem, s);
}
template <int MT>
hipError_t prepare_t(size_t smem, int* max_grid) {
  hipError_t e = hipFuncSetAttribute((const void*)k_mega<MT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  int per_cu = 0;
  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)k_mega<MT>, NT, smem);
  if (e != hipSuccess) return e;
  int dev = 0, cus = 0;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
  *max_grid = per_cu > 0 ? cus : 0;
  return hipSuccess;
}

}  // namespace

size_t mega_smem_bytes(const MegaParams& hp, int MT) {
  size_t need = 0;
  auto upd = [&](size_t b) { if (b > need) need = b; };
  // GEMM partial sums
  {
    int KW = MT <= 2 ? 8 : (MT == 4 ? 4 : 2), NW = 8 / KW;
    upd((size_t)(KW - 1) * NW * MT * 4 * 2 * 64 * 4);
  }
  for (const MegaModel* m : {&hp.draft, &hp.target}) {
    int G = m->md.H / m->md.KVH, DH = m->md.dh;
    upd((size_t)(G * DH + 2 * DH + 8 * G * DH + 16 + G * hp.max_seq) * 4);
  }
  if (MT == 1) {
    int dmax = hp.draft.md.d > hp.target.md.d ? hp.draft.md.d : hp.target.md.d;
    upd((size_t)8 * 2 * 8 * 64 * 4 + (size_t)2 * dmax * 4 + (size_t)((dmax + 15) / 16) * 16 * 8);   // fused-norm GEMM: partial sums + gain/offset + row statistics
  }
  upd((size_t)8 * MT * 16 * 8);              // LM-head partial keys
  upd((size_t)8 * hp.max_batch * 4);         // verifier contributions
  upd((size_t)(2 * 1024 + 16) * 4);          // decide / finish
  return (need + 255) & ~(size_t)255;
}

hipError_t mega_prepare(int MT, size_t smem, int* max_grid) {
  switch (MT) {
    case 1: return prepare_t<1>(smem, max_grid);
    case 2: return prepare_t<2>(smem, max_grid);
    case 4: return prepare_t<4>(smem, max_grid);
    default: return prepare_t<8>(smem, max_grid);
  }
}

hipError_t launch_mega(const MegaParams* dev_params, int MT, int n_steps, const MegaOut& out, size_t smem, int grid,
                       hipStream_t s) {
  switch (MT) {
    case 1: return launch_t<1>(dev_params, n_steps, out, smem, grid, s);
    case 2: return launch_t<2>(dev_params, n_steps, out, smem, grid, s);
    case 4: return launch_t<4>(dev_params, n_steps, out, smem, grid, s);
    default: return launch_t<8>(dev_params, n_steps, out, smem, grid, s);
  }
}

}  // namespace sprinter
