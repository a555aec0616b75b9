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
#include "mega_dev.h"

namespace sprinter {

namespace {

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
    sh.prof[64 + idx] += 1;
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

__device__ __forceinline__ void ph_embed(const MegaModel* Mp, int n_rows_) {
  phase_embed(*Mp, uni(n_rows_), blockIdx.x, gridDim.x);
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
__device__ __forceinline__ bool run_gemm(const PhaseDesc* dp, int epi, int n_rows, float* smem) {
  switch (epi) {
    case EPI_F32: return ph_gemm<MT, EPI_F32>(dp, n_rows, smem);
    case EPI_RESID: return ph_gemm<MT, EPI_RESID>(dp, n_rows, smem);
    case EPI_GELU: return ph_gemm<MT, EPI_GELU>(dp, n_rows, smem);
    default: return ph_gemm<MT, EPI_SWIGLU>(dp, n_rows, smem);
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
          ph_embed(M, n_rows);
          tick(PH_EMBED);
        } else if (kind == PK_NORM) {
          ok = ph_norm(dp, n_rows, smem);
          tick(PH_NORM);
        } else if (kind == PK_GEMM) {
          const int epi = dp->epi, slot = dp->layer;
          ok = run_gemm<MT>(dp, epi, n_rows, smem);
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
  upd((size_t)8 * MT * 16 * 8);              // LM-head partial keys
  upd((size_t)8 * hp.max_batch * 4);         // verifier contributions
  upd((size_t)(2 * 1024 + 16) * 4);          // decide / finish
  return (need + 255) & ~(size_t)255;
}

hipError_t mega_prepare(int MT, size_t smem, int* max_grid) {
  switch (MT) {
    case 2: return prepare_t<2>(smem, max_grid);
    case 4: return prepare_t<4>(smem, max_grid);
    default: return prepare_t<8>(smem, max_grid);
  }
}

hipError_t launch_mega(const MegaParams* dev_params, int MT, int n_steps, const MegaOut& out, size_t smem, int grid,
                       hipStream_t s) {
  switch (MT) {
    case 2: return launch_t<2>(dev_params, n_steps, out, smem, grid, s);
    case 4: return launch_t<4>(dev_params, n_steps, out, smem, grid, s);
    default: return launch_t<8>(dev_params, n_steps, out, smem, grid, s);
  }
}

}  // namespace sprinter
