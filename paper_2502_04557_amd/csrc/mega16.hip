// Persistent decode kernel for at most 16 rows per model forward (one MFMA row tile), bf16 mode:
// n_steps whole SPRINTER decode steps (Alg. 2 of the paper, rows in lock step) in one cooperative
// launch, one workgroup of 8 waves per compute unit.
//
// Roles inside a workgroup: wave 0 runs the grid barrier and every GEMM epilogue (it is the only
// wave whose stores other workgroups wait for, so it is the only one that has to see its stores
// acknowledged before the barrier); waves 1..7 stream weights and feed the matrix cores.  While
// wave 0 waits at a barrier the compute waves already hold the requests for the next phase's
// weights (up to 32 operand tiles = 32 KiB per wave), so HBM latency overlaps the barrier and
// nothing but activation loads (L2) sits between a barrier and the MFMAs.
//
// A GEMM phase for one workgroup: column tiles nt = wg, wg + nwg, ...; K is split over the 7
// compute waves (k tile kt = kw + 7 i).  A wave's 32 register slots hold, per "round",
// PG tiles x KG k-groups of 8 k tiles (PG * KG = 4, or 2 when two matrices are streamed for SwiGLU).
// Partial sums go through LDS (double buffered) to wave 0, which adds them in a fixed order and
// applies bias / residual / activation.  Layer norms are folded into the consuming GEMM: the
// compute waves add up the row statistics of exactly the residual-stream fragments they load.
#include "mega_dev.h"

namespace sprinter {
namespace {

constexpr int NCW = 7;     // compute waves
constexpr int WS = 16;     // weight operand tiles held in registers per compute wave
constexpr int SUB1 = WS / 8;   // sub-blocks of 8 k tiles per round when one matrix is streamed
constexpr int PART_FLOATS = SUB1 * 4 * 64;   // partial sums of one wave and round (one matrix: SUB1 x 4, two: SUB1 / 2 x 8 registers)

struct W32 { uint4 s[WS]; };

struct Sh16 {
  unsigned long long* prof;
  unsigned long long prof_last;    // wave 0's last time stamp
  unsigned long long c_last;       // compute wave 1's last time stamp
  int fail;
};
static __shared__ Sh16 sh16;

enum { T_EMBED = 0, T_NORM, T_QKV, T_ATTN, T_OPROJ, T_FFN1, T_FFN2, T_LMHEAD, T_VERIFIER, T_DECIDE, T_FINISH, T_BARRIER,
       T_FENCE, T_GA, T_GB, T_GC };
__device__ __forceinline__ void tick16(int idx) {
  if (sh16.prof && blockIdx.x == 0 && threadIdx.x == 0) {
    unsigned long long t = wall_clock64();
    sh16.prof[idx] += t - sh16.prof_last;
    sh16.prof[64 + idx] += 1;
    sh16.prof_last = t;
  }
}

// time line of compute wave 1 of workgroup 0: slot 16 + 8 * kind + j (kind: QKV, O-proj, FFN-up, FFN-down)
__device__ __forceinline__ void tickc(int kind, int j) {
  if (sh16.prof && blockIdx.x == 0 && threadIdx.x == 64) {
    unsigned long long t = wall_clock64();
    const int idx = 16 + 8 * kind + j;
    sh16.prof[idx] += t - sh16.c_last;
    sh16.prof[64 + idx] += 1;
    sh16.c_last = t;
  }
}
enum { C_BARRIER = 0, C_STATS, C_OPERANDS, C_MFMA, C_PREFETCH, C_SYNC };

__device__ __forceinline__ int ufl(int v) { return __builtin_amdgcn_readfirstlane(v); }

// A phase record from the LDS copy of the phase table, field by field into scalar registers.
__device__ __forceinline__ PhaseDesc lds_desc(const PhaseDesc* p) {
  static_assert(sizeof(PhaseDesc) % 4 == 0, "descriptor size");
  union { PhaseDesc d; unsigned w[sizeof(PhaseDesc) / 4]; } u;
  const unsigned* src = reinterpret_cast<const unsigned*>(p);
#pragma unroll
  for (unsigned i = 0; i < sizeof(PhaseDesc) / 4; ++i) u.w[i] = (unsigned)ufl((int)src[i]);
  return u.d;
}

// The inter-workgroup part of the grid barrier, run by wave 0 only.
__device__ __forceinline__ bool w0_protocol(unsigned* s, int* err, unsigned ep, int nwg) {
  const int wg = blockIdx.x, g = wg / GS, r = wg % GS, ng = (nwg + GS - 1) / GS;
  const int gsize = min(GS, nwg - g * GS);
  const int lane = threadIdx.x;
  long long spins = 0;
  bool ok = true;
  if (r != 0) {
    if (lane == 0) st_u32(s + g * 64 + r, ep);
    ok = bar_wait(s + 8192 + g * 64, ep, err, spins);
  } else {
    if (lane > 0 && lane < gsize) ok = bar_wait(s + g * 64 + lane, ep, err, spins);
    if (__all(ok)) {
      if (lane == 0) st_u32(s + 4096 + g, ep);
      if (lane < ng) ok = bar_wait(s + 4096 + lane, ep, err, spins);
    }
    if (lane == 0) st_u32(s + 8192 + g * 64, ep);
  }
  return __all(ok);
}

__device__ __forceinline__ int kg_per_round(int n_kg, int sub) { return n_kg == 1 ? 1 : sub; }
__device__ __forceinline__ int gemm_nkg(int Kt) { return ((Kt + NCW - 1) / NCW + 7) / 8; }

// Requests the weight tiles of round (tile group tg, k round kr).  Slot q * 8 + ii (one matrix) or
// q * 16 + 2 ii + {0,1} (two matrices) holds tile pl = q / KG of the group, k group kr * KG + q % KG.
template <int MATS>
__device__ __forceinline__ void prefetch_round(const uint4* W, const uint4* W2, int Kt, int n_tiles, int lgKG, int tg, int kr,
                                               int kw, int wg, int nwg, W32& w) {
  constexpr int SUB = SUB1 / MATS;
  const int lane = threadIdx.x & 63;
  const int nkw = max(0, (Kt - kw + NCW - 1) / NCW), n_kg = gemm_nkg(Kt);
  const int KG = 1 << lgKG, PG = SUB >> lgKG;
  const int kt_safe = kw < Kt ? kw : 0;             // a k tile that exists, for the slots beyond the wave's share
#pragma unroll
  for (int q = 0; q < SUB; ++q) {
    const int pl = q >> lgKG, kg = kr * KG + (q & (KG - 1));
    const int nt = wg + (tg * PG + pl) * nwg;
    if (nt < n_tiles && kg < n_kg) {                 // uniform: one branch per sub-block, none per load
      const uint4* b1 = W + (size_t)nt * Kt * 64;
      const uint4* b2 = MATS == 2 ? W2 + (size_t)nt * Kt * 64 : nullptr;
#pragma unroll
      for (int ii = 0; ii < 8; ++ii) {
        const int i = kg * 8 + ii;
        const int kt = i < nkw ? kw + NCW * i : kt_safe;
        const unsigned off = (unsigned)(kt * 64 + lane);
        if (MATS == 1) {
          w.s[q * 8 + ii] = ldg(b1, off);
        } else {
          w.s[q * 16 + ii * 2] = ldg(b1, off);
          w.s[q * 16 + ii * 2 + 1] = ldg(b2, off);
        }
      }
    } else {                                         // zero weights: the MFMAs run unconditionally and add nothing
#pragma unroll
      for (int j = 0; j < 8 * MATS; ++j) w.s[q * 8 * MATS + j] = make_uint4(0u, 0u, 0u, 0u);
    }
  }
}

// Round 0 of the next phase, if it is a GEMM: issued as soon as the slots are free.
__device__ __forceinline__ bool prefetch_next(const PhaseDesc* nx, W32& w, int wg, int nwg) {
  if (!nx) return false;
  if (ufl(nx->kind) != PK_GEMM) return false;
  const PhaseDesc d = lds_desc(nx);
  const int kw = wave_id() - 1;
  const bool dual = d.epi == EPI_SWIGLU;
  const int n_kg = gemm_nkg(d.Kt);
  const int KG = kg_per_round(n_kg, dual ? SUB1 / 2 : SUB1);
  const int lg = KG == 4 ? 2 : (KG == 2 ? 1 : 0);
  if (dual) prefetch_round<2>(d.W, d.W2, d.Kt, d.n_tiles, lg, 0, 0, kw, wg, nwg, w);
  else prefetch_round<1>(d.W, d.W2, d.Kt, d.n_tiles, lg, 0, 0, kw, wg, nwg, w);
  return true;
}

// Norm gain / offset of a fused-norm phase: requested by the compute waves before the barrier wait
// (they are constants of the model), parked in LDS after it.
constexpr int NGB = 4;                    // float4 per compute thread: covers K <= 7168 without a second trip
struct GB { float4 g[NGB], b[NGB]; };
__device__ __forceinline__ void gb_request(const PhaseDesc& a, GB& r) {
  const int t = (int)threadIdx.x - 64, n4 = a.K >> 2;
  if (t < 0) return;
#pragma unroll
  for (int q = 0; q < NGB; ++q) {
    const int i4 = t + q * (NCW * 64);
    if (i4 < n4) {
      r.g[q] = ldg(reinterpret_cast<const float4*>(a.g), (unsigned)i4);
      r.b[q] = a.arch == 0 ? ldg(reinterpret_cast<const float4*>(a.b), (unsigned)i4) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
}
__device__ __forceinline__ void gb_park(const PhaseDesc& a, const GB& r, float* gbl) {
  const int t = (int)threadIdx.x - 64, n4 = a.K >> 2;
  if (t < 0) return;
  float4* g4 = reinterpret_cast<float4*>(gbl);
  float4* b4 = g4 + n4;
#pragma unroll
  for (int q = 0; q < NGB; ++q) {
    const int i4 = t + q * (NCW * 64);
    if (i4 < n4) { g4[i4] = r.g[q]; b4[i4] = r.b[q]; }
  }
  for (int i4 = t + NGB * (NCW * 64); i4 < n4; i4 += NCW * 64) {     // very wide models: the rest, after the barrier
    g4[i4] = ldg(reinterpret_cast<const float4*>(a.g), (unsigned)i4);
    b4[i4] = a.arch == 0 ? ldg(reinterpret_cast<const float4*>(a.b), (unsigned)i4) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
}

// ------------------------------------------------------------------ compute waves (1..7)
// PF_IN: the slots may already hold round 0 (pf_valid says so); PF_OUT: leave round 0 of the next phase in them.
template <int EPI, bool NORM, int KG, bool PF_IN, bool PF_OUT>
__device__ __forceinline__ void gemm16_compute(const PhaseDesc& a, const PhaseDesc* nx, W32& w, bool& pf_valid, float* part,
                                               float* stl, const float* gbl, int wg, int nwg) {
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int MATS = DUAL ? 2 : 1, SUB = SUB1 / MATS, PG = SUB / KG, NI = DUAL ? 8 : 4;
  constexpr int LG = KG == 4 ? 2 : (KG == 2 ? 1 : 0);
  const int lane = threadIdx.x & 63, kw = wave_id() - 1;
  const int m_l = lane & 15, grp = lane >> 4;
  const int Kt = a.Kt, K = a.K;
  const int nkw = max(0, (Kt - kw + NCW - 1) / NCW);
  const int n_kg = gemm_nkg(Kt);
  const int n_kr = (n_kg + KG - 1) / KG;
  const int n_t = wg < a.n_tiles ? (a.n_tiles - wg + nwg - 1) / nwg : 0;
  const int n_tg = (n_t + PG - 1) / PG;
  const bool keep = n_kg == 1;           // all of the wave's activation fragments stay in registers
  const uint4* Xl = NORM ? nullptr : a.X + a.x_plane16;
  const int kt_safe = kw < Kt ? kw : 0;            // an existing k tile for the units beyond the wave's share
  uint4 xa[8][2];
  auto load_group = [&](int kg) {                   // no branches: clamped addresses, the extra units are zeroed at use
#pragma unroll
    for (int ii = 0; ii < 8; ++ii) {
      const int i = kg * 8 + ii;
      const int kt = i < nkw ? kw + NCW * i : kt_safe;
      if (NORM) {
        const int k = min(kt * 32 + grp * 8, K - 8);
        const unsigned e4 = (unsigned)(m_l * K + k) >> 2;      // K and k are multiples of 8
        xa[ii][0] = ldg(reinterpret_cast<const uint4*>(a.h), e4);
        xa[ii][1] = ldg(reinterpret_cast<const uint4*>(a.h), e4 + 1);
      } else {
        xa[ii][0] = ldg(a.X, (unsigned)(kt * 64 + lane));
        xa[ii][1] = ldg(Xl, (unsigned)(kt * 64 + lane));
      }
    }
  };
  float mean = 0.f, rstd = 1.f;
  const int pk = a.layer == 2 ? 0 : a.layer == 4 ? 1 : a.layer == 5 ? 2 : 3;
  tickc(pk, C_BARRIER);
  if (NORM) {
    // row statistics of the residual stream: every k tile belongs to exactly one compute wave
    float s1 = 0.f, s2 = 0.f;
    for (int kg = 0; kg < n_kg; ++kg) {
      load_group(kg);
#pragma unroll
      for (int ii = 0; ii < 8; ++ii) {
        const int i = kg * 8 + ii, kt = kw + NCW * i;
        const bool ok = i < nkw && kt * 32 + grp * 8 + 8 <= K;
        const float* f = reinterpret_cast<const float*>(&xa[ii][0]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float v = ok ? f[e] : 0.f;
          s1 += v; s2 += v * v;
        }
      }
    }
    s1 += __shfl_xor(s1, 16); s1 += __shfl_xor(s1, 32);
    s2 += __shfl_xor(s2, 16); s2 += __shfl_xor(s2, 32);
    if (grp == 0) { stl[(kw * 16 + m_l) * 2] = s1; stl[(kw * 16 + m_l) * 2 + 1] = s2; }
    __syncthreads();
    float S1 = 0.f, S2 = 0.f;
#pragma unroll
    for (int q = 0; q < NCW; ++q) { S1 += stl[(q * 16 + m_l) * 2]; S2 += stl[(q * 16 + m_l) * 2 + 1]; }
    const double invK = 1.0 / (double)K;
    const double mu = a.arch == 0 ? (double)S1 * invK : 0.0;
    double var = (double)S2 * invK - mu * mu;
    if (var < 0.0) var = 0.0;
    mean = (float)mu;
    rstd = (float)(1.0 / sqrt(var + (double)a.eps));
  } else if (keep) {
    load_group(0);
  }
  tickc(pk, C_STATS);
  for (int tg = 0; tg < n_tg; ++tg) {
    for (int kr = 0; kr < n_kr; ++kr) {
      const int round = tg * n_kr + kr;
      if (!(PF_IN && round == 0 && pf_valid)) prefetch_round<MATS>(a.W, a.W2, Kt, a.n_tiles, LG, tg, kr, kw, wg, nwg, w);
      f32x4 acc[SUB], acc2[DUAL ? SUB : 1];
#pragma unroll
      for (int q = 0; q < SUB; ++q) {
        acc[q] = (f32x4){0.f, 0.f, 0.f, 0.f};
        if (DUAL) acc2[q] = (f32x4){0.f, 0.f, 0.f, 0.f};
      }
      if (sh16.prof) {                 // diagnosis only: separates waiting for the weights from the arithmetic
        __builtin_amdgcn_s_waitcnt(0);
        tickc(pk, C_OPERANDS);
      }
#pragma unroll
      for (int g = 0; g < KG; ++g) {                  // straight-line code: no branch between the loads and the MFMAs
        const int kg = kr * KG + g;
        if (!keep) load_group(kg < n_kg ? kg : 0);
#pragma unroll
        for (int ii = 0; ii < 8; ++ii) {
          const int i = kg * 8 + ii, kt = kw + NCW * i;
          uint4 ah, al;
          if (NORM) {
            const int kreal = kt * 32 + grp * 8;
            const int k = min(max(kreal, 0), K - 8);
            const bool ok = kg < n_kg && i < nkw && kreal + 8 <= K;     // K is a multiple of 8: all or nothing
            const float* f = reinterpret_cast<const float*>(&xa[ii][0]);
            const float4 g0 = *reinterpret_cast<const float4*>(gbl + k), g1 = *reinterpret_cast<const float4*>(gbl + k + 4);
            const float4 b0 = *reinterpret_cast<const float4*>(gbl + K + k), b1 = *reinterpret_cast<const float4*>(gbl + K + k + 4);
            float x[8];
            x[0] = (f[0] - mean) * rstd * g0.x + b0.x; x[1] = (f[1] - mean) * rstd * g0.y + b0.y;
            x[2] = (f[2] - mean) * rstd * g0.z + b0.z; x[3] = (f[3] - mean) * rstd * g0.w + b0.w;
            x[4] = (f[4] - mean) * rstd * g1.x + b1.x; x[5] = (f[5] - mean) * rstd * g1.y + b1.y;
            x[6] = (f[6] - mean) * rstd * g1.z + b1.z; x[7] = (f[7] - mean) * rstd * g1.w + b1.w;
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = ok ? x[e] : 0.f;
            split2(x[0], x[1], ah.x, al.x);
            split2(x[2], x[3], ah.y, al.y);
            split2(x[4], x[5], ah.z, al.z);
            split2(x[6], x[7], ah.w, al.w);
          } else {
            const bool ok = kg < n_kg && i < nkw;
            ah = ok ? xa[ii][0] : make_uint4(0u, 0u, 0u, 0u);
            al = ok ? xa[ii][1] : make_uint4(0u, 0u, 0u, 0u);
          }
#pragma unroll
          for (int pl = 0; pl < PG; ++pl) {
            const int q = pl * KG + g;
            if (!DUAL) {
              acc[q] = mfma_bf16(ah, w.s[q * 8 + ii], acc[q]);
              acc[q] = mfma_bf16(al, w.s[q * 8 + ii], acc[q]);
            } else {
              acc[q] = mfma_bf16(ah, w.s[q * 16 + ii * 2], acc[q]);
              acc[q] = mfma_bf16(al, w.s[q * 16 + ii * 2], acc[q]);
              acc2[q] = mfma_bf16(ah, w.s[q * 16 + ii * 2 + 1], acc2[q]);
              acc2[q] = mfma_bf16(al, w.s[q * 16 + ii * 2 + 1], acc2[q]);
            }
          }
        }
      }
      float* dst = part + (size_t)((round & 1) * NCW + kw) * PART_FLOATS;
#pragma unroll
      for (int q = 0; q < SUB; ++q)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          dst[(q * NI + v) * 64 + lane] = acc[q][v];
          if (DUAL) dst[(q * NI + 4 + v) * 64 + lane] = acc2[q][v];
        }
      tickc(pk, C_MFMA);
      __syncthreads();
      tickc(pk, C_SYNC);
      // after the hand-over: requests that find the memory pipeline full must not hold up wave 0's epilogue
      if (PF_OUT && tg == n_tg - 1 && kr == n_kr - 1) pf_valid = prefetch_next(nx, w, wg, nwg);
      tickc(pk, C_PREFETCH);
    }
  }
  if (PF_OUT && n_tg == 0) pf_valid = prefetch_next(nx, w, wg, nwg);
  if (!PF_OUT) pf_valid = false;
}

// ------------------------------------------------------------------ wave 0: sums and epilogues
template <int EPI, bool NORM, int KG>
__device__ __forceinline__ void gemm16_epilogue(const PhaseDesc& a, int n_rows, const float* part, int wg, int nwg) {
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int MATS = DUAL ? 2 : 1, SUB = SUB1 / MATS, PG = SUB / KG, NI = DUAL ? 8 : 4;
  const int lane = threadIdx.x & 63;
  const int m_l = lane & 15, grp = lane >> 4;
  const int n_kg = gemm_nkg(a.Kt);
  const int n_kr = (n_kg + KG - 1) / KG;
  const int n_t = wg < a.n_tiles ? (a.n_tiles - wg + nwg - 1) / nwg : 0;
  const int n_tg = (n_t + PG - 1) / PG;
  if (NORM) __syncthreads();           // the compute waves' statistics exchange
  for (int tg = 0; tg < n_tg; ++tg) {
    f32x4 t1[PG], t2[DUAL ? PG : 1];
    float bias[PG], res[PG][4];
#pragma unroll
    for (int pl = 0; pl < PG; ++pl) {
      t1[pl] = (f32x4){0.f, 0.f, 0.f, 0.f};
      if (DUAL) t2[pl] = (f32x4){0.f, 0.f, 0.f, 0.f};
      const int nt = wg + (tg * PG + pl) * nwg, n = nt * 16 + m_l;
      const bool n_ok = tg * PG + pl < n_t && n < a.N;
      bias[pl] = (a.bias && n_ok) ? ldg(a.bias, (unsigned)n) : 0.f;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int m = grp * 4 + v;
        res[pl][v] = (EPI == EPI_RESID && n_ok && m < n_rows) ? ldg(a.resid, (unsigned)(m * a.ldo + n)) : 0.f;
      }
    }
    for (int kr = 0; kr < n_kr; ++kr) {
      const int round = tg * n_kr + kr;
      __syncthreads();
      tick16(13);
      const float* src = part + (size_t)((round & 1) * NCW) * PART_FLOATS;
#pragma unroll
      for (int pl = 0; pl < PG; ++pl)
#pragma unroll
        for (int g = 0; g < KG; ++g) {
          const int q = pl * KG + g;
#pragma unroll
          for (int kw = 0; kw < NCW; ++kw)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              t1[pl][v] += src[(size_t)kw * PART_FLOATS + (q * NI + v) * 64 + lane];
              if (DUAL) t2[pl][v] += src[(size_t)kw * PART_FLOATS + (q * NI + 4 + v) * 64 + lane];
            }
        }
    }
#pragma unroll
    for (int pl = 0; pl < PG; ++pl) {
      const int nt = wg + (tg * PG + pl) * nwg, n = nt * 16 + m_l;
      const bool n_ok = tg * PG + pl < n_t && n < a.N;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int m = grp * 4 + v;
        const bool ok = n_ok && m < n_rows;
        if (EPI == EPI_F32) {
          if (ok) st_f32(a.out_f32 + (size_t)m * a.ldo + n, t1[pl][v] + bias[pl]);
        } else if (EPI == EPI_RESID) {
          if (ok) st_f32(a.out_f32 + (size_t)m * a.ldo + n, res[pl][v] + t1[pl][v] + bias[pl]);
        } else {
          float val = (EPI == EPI_GELU) ? gelu_tanh(t1[pl][v] + bias[pl]) : silu(t1[pl][v]) * t2[pl][v];
          float nb = __shfl_xor(val, 1);
          if (ok && !(lane & 1)) act_store_pair1(a.out_act, a.out_plane, m, n, a.out_K, val, nb);
        }
      }
    }
  }
}

template <int EPI, bool NORM, int KG, bool PF_IN, bool PF_OUT>
__device__ __forceinline__ void gemm16(const PhaseDesc& a, const PhaseDesc* nx, int n_rows, W32& w, bool& pf_valid,
                                       float* part, float* stl, const float* gbl) {
  const int wg = blockIdx.x, nwg = gridDim.x;
  if (wave_id() == 0) gemm16_epilogue<EPI, NORM, KG>(a, n_rows, part, wg, nwg);
  else gemm16_compute<EPI, NORM, KG, PF_IN, PF_OUT>(a, nx, w, pf_valid, part, stl, gbl, wg, nwg);
}

// k groups per round: 1 when a wave's share of K fits 8 k tiles, else all sub-blocks (one tile per round)
template <int EPI, bool NORM, bool PF_IN, bool PF_OUT>
__device__ __forceinline__ void gemm16_kg(const PhaseDesc& a, const PhaseDesc* nx, int n_rows, W32& w, bool& pf_valid,
                                          float* part, float* stl, const float* gbl) {
  constexpr int SUB = EPI == EPI_SWIGLU ? SUB1 / 2 : SUB1;
  if (gemm_nkg(a.Kt) == 1) gemm16<EPI, NORM, 1, PF_IN, PF_OUT>(a, nx, n_rows, w, pf_valid, part, stl, gbl);
  else gemm16<EPI, NORM, SUB, PF_IN, PF_OUT>(a, nx, n_rows, w, pf_valid, part, stl, gbl);
}

// ------------------------------------------------------------------ phases that keep the older structure
// (all 8 waves compute and store); separate functions so that each gets its own register allocation
__device__ __noinline__ void ph16_embed(const MegaModel* M, int n_rows) {
  phase_embed1(*M, ufl(n_rows), blockIdx.x, gridDim.x);
}
__device__ __noinline__ void ph16_norm(const PhaseDesc* dp, int n_rows, float* scratch) {
  const PhaseDesc d = lds_desc(dp);
  phase_norm(d.arch, d.h, d.g, d.b, d.eps, d.K, ufl(n_rows), d.out_act, d.out_plane, d.f32_out2, scratch, blockIdx.x, gridDim.x);
}
__device__ __noinline__ void ph16_attn(const MegaModel* M, int layer, int n_rows, int max_seq, int max_batch, float* scratch) {
  attn_dispatch(*M, ufl(layer), ufl(n_rows), ufl(max_seq), ufl(max_batch), scratch, blockIdx.x, gridDim.x);
}
__device__ __noinline__ void ph16_lmhead(const MegaParams* Pp, const MegaModel* M, int n_rows, unsigned stream_id, float* logits_out,
                                         float* hidden_out, float* scratch) {
  const MegaParams& P = *Pp;
  SamplerArgs sa{P.seed_lo, P.seed_hi, stream_id, P.inv_temperature};
  phase_lmhead<1>(*M, ufl(n_rows), sa, P.rows_alloc, logits_out, scratch, blockIdx.x, gridDim.x);
  if (hidden_out)
    for (size_t j = (size_t)blockIdx.x * NT + threadIdx.x; j < (size_t)n_rows * M->md.d; j += (size_t)gridDim.x * NT)
      hidden_out[j] = M->hf[j];
}
__device__ __noinline__ void ph16_verifier(const MegaParams* Pp, int B, float* scratch) {
  phase_verifier(*Pp, ufl(B), scratch, blockIdx.x, gridDim.x);
}
__device__ __noinline__ void ph16_decide(const MegaParams* Pp, const MegaOut* out, float* scratch) {
  decide(*Pp, *out, gridDim.x, scratch);
}
__device__ __noinline__ void ph16_finish(const MegaParams* Pp, const MegaOut* out, int R, float* scratch) {
  finish(*Pp, *out, ufl(R), gridDim.x, scratch);
}

// ------------------------------------------------------------------ the kernel
// Phase table of one model: embed, then per layer QKV, attention, O-proj, FFN-up, FFN-down, then the
// final norm and the LM head.
__global__ __launch_bounds__(NT) void k_mega16(const MegaParams* __restrict__ Pp, int n_steps, MegaOut out, int tab_bytes) {
  extern __shared__ float smem[];
  const MegaParams& P = *Pp;
  const int wg = blockIdx.x, nwg = gridDim.x, wv = wave_id();
  PhaseDesc* tab = reinterpret_cast<PhaseDesc*>(smem);
  const int nq = P.draft.n_phases, np = P.target.n_phases;
  {   // phase tables of both models into LDS
    const unsigned* s1 = reinterpret_cast<const unsigned*>(P.draft.phases);
    const unsigned* s2 = reinterpret_cast<const unsigned*>(P.target.phases);
    unsigned* d = reinterpret_cast<unsigned*>(smem);
    const int n1 = nq * (int)(sizeof(PhaseDesc) / 4), n2 = np * (int)(sizeof(PhaseDesc) / 4);
    for (int i = threadIdx.x; i < n1; i += NT) d[i] = s1[i];
    for (int i = threadIdx.x; i < n2; i += NT) d[n1 + i] = s2[i];
  }
  float* scratch = smem + tab_bytes / 4;
  float* part = scratch;                                  // [2][7][PART_FLOATS] partial sums
  float* stl = scratch + 2 * NCW * PART_FLOATS;           // [7][16][2] row statistics
  float* gbl = stl + NCW * 16 * 2;                        // [2][K] norm gain, offset of the running fused-norm phase
  if (threadIdx.x == 0) {
    sh16.prof = P.prof; sh16.prof_last = P.prof ? wall_clock64() : 0ull; sh16.c_last = sh16.prof_last; sh16.fail = 0;
  }
  unsigned epoch = ld_u32(P.epoch);
  __syncthreads();

  // all == true: stores of every wave have to be acknowledged before the workgroup arrives
  auto BAR = [&](bool all) -> bool {
    if (all) {
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
    }
    if (wv == 0) {
      __builtin_amdgcn_s_waitcnt(0);
      const bool ok = w0_protocol(P.sync, P.err, ++epoch, nwg);
      if (!ok && threadIdx.x == 0) sh16.fail = 1;
    }
    __syncthreads();
    tick16(T_BARRIER);
    return sh16.fail == 0;
  };

  const int B = out.B;
  for (int step = 0; step < n_steps; ++step) {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "agent");     // buffers of the previous step are rewritten below
    tick16(T_FENCE);
    int R = 0;
    for (int which = 0; which < 2; ++which) {
      const MegaModel* M = which == 0 ? &Pp->draft : &Pp->target;
      const int n_rows = ufl(which == 0 ? B : R);
      if (which == 1 && R == 0) break;
      const PhaseDesc* ph = tab + (which == 0 ? 0 : nq);
      const int n_layer = ((which == 0 ? nq : np) - 3) / 5;
      ph16_embed(M, n_rows);
      tick16(T_EMBED);
      {
        W32 w;
#pragma unroll
        for (int i = 0; i < WS; ++i) w.s[i] = make_uint4(0u, 0u, 0u, 0u);
        bool pf_valid = false;
        for (int l = 0; l < n_layer; ++l) {
          const PhaseDesc* lp = ph + 1 + 5 * l;
          {   // QKV projection (layer norm folded in); the attention phase takes no prefetch
            const PhaseDesc d = lds_desc(lp);
            GB gb;
            gb_request(d, gb);
            if (!BAR(l == 0)) return;
            gb_park(d, gb, gbl);
            gemm16_kg<EPI_F32, true, true, false>(d, nullptr, n_rows, w, pf_valid, part, stl, gbl);
            tick16(T_QKV);
          }
          if (!BAR(false)) return;
          ph16_attn(M, l, n_rows, P.max_seq, P.max_batch, scratch);
          tick16(T_ATTN);
          {   // O-proj + residual
            const PhaseDesc d = lds_desc(lp + 2);
            if (!BAR(true)) return;
            gemm16_kg<EPI_RESID, false, false, true>(d, lp + 3, n_rows, w, pf_valid, part, stl, gbl);
            tick16(T_OPROJ);
          }
          {   // FFN-up (layer norm folded in) + activation
            const PhaseDesc d = lds_desc(lp + 3);
            GB gb;
            gb_request(d, gb);
            if (!BAR(false)) return;
            gb_park(d, gb, gbl);
            if (d.epi == EPI_GELU) gemm16_kg<EPI_GELU, true, true, true>(d, lp + 4, n_rows, w, pf_valid, part, stl, gbl);
            else gemm16_kg<EPI_SWIGLU, true, true, true>(d, lp + 4, n_rows, w, pf_valid, part, stl, gbl);
            tick16(T_FFN1);
          }
          {   // FFN-down + residual; leaves the next layer's QKV weights requested
            const PhaseDesc d = lds_desc(lp + 4);
            if (!BAR(false)) return;
            gemm16_kg<EPI_RESID, false, true, true>(d, l + 1 < n_layer ? lp + 5 : nullptr, n_rows, w, pf_valid, part, stl, gbl);
            tick16(T_FFN2);
          }
        }
      }
      if (!BAR(false)) return;
      ph16_norm(ph + 1 + 5 * n_layer, n_rows, scratch);
      tick16(T_NORM);
      if (!BAR(true)) return;
      ph16_lmhead(Pp, M, n_rows, (unsigned)which, which == 0 ? out.o_draft_logits : out.o_target_logits,
                  which == 0 ? out.o_draft_hidden : out.o_target_hidden, scratch);
      tick16(T_LMHEAD);
      if (which == 0) {
        ph16_verifier(Pp, B, scratch);
        tick16(T_VERIFIER);
        if (!BAR(true)) return;
        if (wg == 0) ph16_decide(Pp, &out, scratch);
        tick16(T_DECIDE);
        if (!BAR(true)) return;
        R = min(max(ld_i32(P.n_rej), 0), B);
      } else {
        if (!BAR(true)) return;
      }
    }
    if (wg == 0) ph16_finish(Pp, &out, R, scratch);
    tick16(T_FINISH);
    if (!BAR(true)) return;
  }
  if (wg == 0 && threadIdx.x == 0) st_u32(P.epoch, epoch);
}

}  // namespace

size_t mega16_smem_bytes(const MegaParams& hp, int* tab_bytes) {
  size_t tab = (size_t)(hp.draft.n_phases + hp.target.n_phases) * sizeof(PhaseDesc);
  tab = (tab + 255) & ~(size_t)255;
  int dmax = hp.draft.md.d > hp.target.md.d ? hp.draft.md.d : hp.target.md.d;
  size_t need = (size_t)2 * NCW * PART_FLOATS * 4 + (size_t)NCW * 16 * 2 * 4 + (size_t)2 * dmax * 4;   // partial sums + row statistics
  auto upd = [&](size_t b) { if (b > need) need = b; };
  for (const MegaModel* m : {&hp.draft, &hp.target}) {
    int G = m->md.H / m->md.KVH, DH = m->md.dh;
    upd((size_t)(G * DH + 2 * DH + 8 * G * DH + 16 + G * hp.max_seq) * 4);      // attention
  }
  upd((size_t)8 * 16 * 8);                   // LM-head partial keys
  upd((size_t)8 * hp.max_batch * 4);         // verifier contributions
  upd((size_t)(2 * 1024 + 16) * 4);          // decide / finish
  *tab_bytes = (int)tab;
  return tab + ((need + 255) & ~(size_t)255);
}

hipError_t mega16_prepare(size_t smem, int* max_grid) {
  hipError_t e = hipFuncSetAttribute((const void*)k_mega16, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  int per_cu = 0;
  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)k_mega16, NT, smem);
  if (e != hipSuccess) return e;
  int dev = 0, cus = 0;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
  *max_grid = per_cu > 0 ? cus : 0;
  return hipSuccess;
}

hipError_t launch_mega16(const MegaParams* dev_params, int n_steps, const MegaOut& out, size_t smem, int tab_bytes, int grid,
                         hipStream_t s) {
  MegaOut o = out;
  void* args[] = {(void*)&dev_params, (void*)&n_steps, (void*)&o, (void*)&tab_bytes};
  return hipLaunchCooperativeKernel((const void*)k_mega16, dim3(grid), dim3(NT), args, (unsigned)smem, s);
}

}  // namespace sprinter
