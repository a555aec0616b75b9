// HIP kernels of the batched SPRINTER decode step for gfx950 (wave64, MFMA).
//
// One decode step (Alg. 2 of the paper, run for B rows in lock step):
//   draft forward -> LM head + Gumbel-max sample -> verifier + threshold ->
//   compaction of rejected rows -> target forward on those rows -> sample ->
//   scatter back.  Every kernel reads the number of active rows from device
//   memory; the launch shapes are upper bounds the host chooses.
#include "dev.h"
#include <algorithm>
#include <cstring>

namespace sprinter {

// ================================================================ packing
// [N, K] row-major bf16 -> operand tiles (zero padded to 16 rows x 32 k).
__global__ __launch_bounds__(256) void k_pack_bf16(const bf16_t* __restrict__ w, uint4* __restrict__ out, int N, int K,
                                                   int Kt, size_t total) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  int lane = (int)(i & 63);
  size_t tile = i >> 6;
  int kt = (int)(tile % Kt);
  int nt = (int)(tile / Kt);
  int n = nt * 16 + (lane & 15);
  int k0 = kt * 32 + (lane >> 4) * 8;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (n < N) {
    if (k0 + 8 <= K) {
      v = *reinterpret_cast<const uint4*>(w + (size_t)n * K + k0);   // K % 8 == 0 keeps this aligned
    } else if (k0 < K) {
      bf16_t t[8];
      for (int e = 0; e < 8; ++e) t[e] = (k0 + e < K) ? w[(size_t)n * K + k0 + e] : (bf16_t)0;
      v = *reinterpret_cast<uint4*>(t);
    }
  }
  out[i] = v;
}
void launch_pack_bf16(const void* w, void* out, int N, int K, hipStream_t s) {
  int Kt = (K + 31) / 32, Nt = (N + 15) / 16;
  size_t total = (size_t)Nt * Kt * 64;
  hipLaunchKernelGGL(k_pack_bf16, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t*)w,
                     (uint4*)out, N, K, Kt, total);
}

__global__ __launch_bounds__(256) void k_fill_zero(uint4* p, size_t n16) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  size_t stride = (size_t)gridDim.x * 256;
  for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}
void launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  size_t n16 = bytes / 16;
  if (!n16) return;
  unsigned grid = (unsigned)((n16 + 255) / 256);
  if (grid > 4096) grid = 4096;
  hipLaunchKernelGGL(k_fill_zero, dim3(grid), dim3(256), 0, s, (uint4*)p, n16);
}

// ================================================================== embed
template <typename T>
__global__ __launch_bounds__(256) void k_embed(const T* __restrict__ E, const T* __restrict__ P, RowDesc rd,
                                               float* __restrict__ h, float* __restrict__ rope, int d, int dh,
                                               float theta, int use_rope, int V, int max_pos) {
  int r = blockIdx.x;
  if (r >= *rd.n_rows) return;
  int tok = rd.tok[r], pos = rd.pos[r];
  tok = min(max(tok, 0), V - 1);            // an out-of-vocabulary id must not become a wild read
  if (P) pos = min(max(pos, 0), max_pos - 1);
  const T* e = E + (size_t)tok * d;
  const T* p = P ? P + (size_t)pos * d : nullptr;
  for (int k = threadIdx.x; k < d; k += 256) {
    float v = to_f<T>(e[k]);
    if (p) v += to_f<T>(p[k]);
    h[(size_t)r * d + k] = v;
  }
  if (use_rope && (int)threadIdx.x < dh / 2) {
    // angle = pos * theta^(-2i/dh), evaluated in double so that large positions stay accurate
    double inv = pow((double)theta, -2.0 * (double)threadIdx.x / (double)dh);
    double ang = (double)pos * inv;
    rope[(size_t)r * dh + 2 * threadIdx.x] = (float)cos(ang);
    rope[(size_t)r * dh + 2 * threadIdx.x + 1] = (float)sin(ang);
  }
}
void launch_embed(int dtype, const ModelDims& md, const void* tok_emb, const void* pos_emb, const RowDesc& rd,
                  float* h, float* rope, int max_rows, hipStream_t s) {
  int use_rope = md.arch == 1;
  if (dtype == 0)
    hipLaunchKernelGGL(k_embed<float>, dim3(max_rows), dim3(256), 0, s, (const float*)tok_emb,
                       (const float*)pos_emb, rd, h, rope, md.d, md.dh, md.theta, use_rope, md.V, md.max_pos);
  else
    hipLaunchKernelGGL(k_embed<bf16_t>, dim3(max_rows), dim3(256), 0, s, (const bf16_t*)tok_emb,
                       (const bf16_t*)pos_emb, rd, h, rope, md.d, md.dh, md.theta, use_rope, md.V, md.max_pos);
}

// =================================================================== norm
// LayerNorm (arch 0) / RMSNorm (arch 1) of one row per workgroup; two-pass statistics.
template <typename AT, int ARCH>
__global__ __launch_bounds__(256) void k_norm(const float* __restrict__ h, const float* __restrict__ g,
                                              const float* __restrict__ b, float eps, int d,
                                              const int* __restrict__ n_rows, AT* __restrict__ act_out,
                                              size_t plane, float* __restrict__ f32_out) {
  __shared__ float s4[4];
  int r = blockIdx.x;
  if (r >= *n_rows) return;
  const float* x = h + (size_t)r * d;
  float v[32];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    int k = threadIdx.x + i * 256;
    v[i] = k < d ? x[k] : 0.f;
    sum += v[i];
  }
  float mean = 0.f;
  if (ARCH == 0) mean = block_sum256(sum, s4) / (float)d;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    int k = threadIdx.x + i * 256;
    float c = k < d ? v[i] - mean : 0.f;
    sq += c * c;
  }
  float var = block_sum256(sq, s4) / (float)d;
  float rstd = 1.0f / sqrtf(var + eps);
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    int k = threadIdx.x + i * 256;
    if (k < d) {
      float o = (v[i] - mean) * rstd * g[k];
      if (ARCH == 0) o += b[k];
      act_store<AT>(act_out, plane, r, k, d, o);
      if (f32_out) f32_out[(size_t)r * d + k] = o;
    }
  }
}
// bf16 output: one row per workgroup, one thread per 8 consecutive columns (= one 16-byte slot of an
// operand tile per plane), so the row, gain and offset are requested with six 16-byte loads per thread
// before anything is waited for and the result leaves as two 16-byte stores.  d <= 8192.
// NI = 2048-column blocks per row (1, 2 or 4); SH = 0, or the most partial products a pending update of the
// residual stream may consist of (4 or 8): the row is then h + bias + share 0 + share 1 + ..., added in that
// order, written back and normalised.  The partial loads are issued with the others, before the row count
// is known, with clamped share indices and the surplus selected away - no branch, no second memory round.
template <int ARCH, int NI, int SH>
__global__ __launch_bounds__(256) void k_norm_bf16(const float* __restrict__ h, const float* __restrict__ g,
                                                   const float* __restrict__ b, float eps, int d,
                                                   const int* __restrict__ n_rows, bf16_t* __restrict__ act_out, size_t plane,
                                                   float* __restrict__ f32_out, NormPending pend) {
  __shared__ float s4[4];
  const int r = blockIdx.x, tid = threadIdx.x;
  const float4* __restrict__ x4 = reinterpret_cast<const float4*>(h + (size_t)r * d);
  const float4* __restrict__ g4 = reinterpret_cast<const float4*>(g);
  const float4* __restrict__ b4 = reinterpret_cast<const float4*>(b);
  const int n_chunks = d >> 3;                       // d is a multiple of 8
  float x[NI][8], gg[NI][8], bb[NI][8];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int c = min(tid + i * 256, n_chunks - 1);  // clamped: no branch around the loads
    *reinterpret_cast<float4*>(&x[i][0]) = x4[2 * c]; *reinterpret_cast<float4*>(&x[i][4]) = x4[2 * c + 1];
    *reinterpret_cast<float4*>(&gg[i][0]) = g4[2 * c]; *reinterpret_cast<float4*>(&gg[i][4]) = g4[2 * c + 1];
    if (ARCH == 0) { *reinterpret_cast<float4*>(&bb[i][0]) = b4[2 * c]; *reinterpret_cast<float4*>(&bb[i][4]) = b4[2 * c + 1]; }
  }
  if (SH > 0) {
    const float4* __restrict__ pb4 = reinterpret_cast<const float4*>(pend.bias ? pend.bias : g);
    const bool has_bias = pend.bias != nullptr;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = min(tid + i * 256, n_chunks - 1);
      float4 p0[SH + 1], p1[SH + 1];
      p0[0] = pb4[2 * c]; p1[0] = pb4[2 * c + 1];
#pragma unroll
      for (int q = 0; q < SH; ++q) {
        const float4* p4 = reinterpret_cast<const float4*>(pend.part + (size_t)min(q, pend.shares - 1) * pend.stride + (size_t)r * d);
        p0[q + 1] = p4[2 * c]; p1[q + 1] = p4[2 * c + 1];
      }
#pragma unroll
      for (int q = 0; q <= SH; ++q) {                // fixed order: bias, share 0, share 1, ...
        const bool on = q == 0 ? has_bias : q - 1 < pend.shares;
        x[i][0] += on ? p0[q].x : 0.f; x[i][1] += on ? p0[q].y : 0.f; x[i][2] += on ? p0[q].z : 0.f; x[i][3] += on ? p0[q].w : 0.f;
        x[i][4] += on ? p1[q].x : 0.f; x[i][5] += on ? p1[q].y : 0.f; x[i][6] += on ? p1[q].z : 0.f; x[i][7] += on ? p1[q].w : 0.f;
      }
    }
  }
  if (r >= *n_rows) return;
  if (SH > 0) {
    float* hrow = const_cast<float*>(h) + (size_t)r * d;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = tid + i * 256;
      if (c < n_chunks) {
        *reinterpret_cast<float4*>(hrow + c * 8) = make_float4(x[i][0], x[i][1], x[i][2], x[i][3]);
        *reinterpret_cast<float4*>(hrow + c * 8 + 4) = make_float4(x[i][4], x[i][5], x[i][6], x[i][7]);
      }
    }
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const bool ok = tid + i * 256 < n_chunks;
#pragma unroll
    for (int e = 0; e < 8; ++e) { x[i][e] = ok ? x[i][e] : 0.f; sum += x[i][e]; }
  }
  float mean = 0.f;
  if (ARCH == 0) mean = block_sum256(sum, s4) / (float)d;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const bool ok = tid + i * 256 < n_chunks;
#pragma unroll
    for (int e = 0; e < 8; ++e) { const float c = ok ? x[i][e] - mean : 0.f; sq += c * c; }
  }
  const float var = block_sum256(sq, s4) / (float)d;
  const float rstd = 1.0f / sqrtf(var + eps);
  const int Kt = (d + 31) >> 5;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int c = tid + i * 256;
    if (c < n_chunks) {
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        o[e] = (x[i][e] - mean) * rstd * gg[i][e];
        if (ARCH == 0) o[e] += bb[i][e];
      }
      uint4 hi, lo;
      split2(o[0], o[1], hi.x, lo.x);
      split2(o[2], o[3], hi.y, lo.y);
      split2(o[4], o[5], hi.z, lo.z);
      split2(o[6], o[7], hi.w, lo.w);
      const int k = c * 8;
      const size_t slot = ((size_t)(r >> 4) * Kt + (k >> 5)) * 512 + ((((k & 31) >> 3) << 4) + (r & 15)) * 8;
      *reinterpret_cast<uint4*>(act_out + slot) = hi;
      *reinterpret_cast<uint4*>(act_out + plane + slot) = lo;
      if (f32_out) {
        *reinterpret_cast<float4*>(f32_out + (size_t)r * d + k) = make_float4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<float4*>(f32_out + (size_t)r * d + k + 4) = make_float4(o[4], o[5], o[6], o[7]);
      }
    }
  }
}

template <int ARCH, int NI>
static void launch_norm_bf16(const float* h, const float* g, const float* b, float eps, int d, const int* n_rows,
                             bf16_t* act_out, size_t plane, float* f32_out, int max_rows, hipStream_t s, const NormPending& np) {
#define SPRINTER_NORM(SH) hipLaunchKernelGGL((k_norm_bf16<ARCH, NI, SH>), dim3(max_rows), dim3(256), 0, s, h, g, b, eps, d, n_rows, act_out, plane, f32_out, np)
  if (np.shares <= 0) SPRINTER_NORM(0);
  else if (np.shares <= 4) SPRINTER_NORM(4);
  else SPRINTER_NORM(8);
#undef SPRINTER_NORM
}

void launch_norm(int dtype, int arch, const float* h, const float* g, const float* b, float eps, int d,
                 const int* n_rows, void* act_out, size_t plane, float* f32_out, int max_rows, hipStream_t s,
                 const NormPending* pend) {
  NormPending np;
  memset(&np, 0, sizeof np);
  if (pend) np = *pend;
#define NORM_CASE(AT, ARCH) \
  hipLaunchKernelGGL((k_norm<AT, ARCH>), dim3(max_rows), dim3(256), 0, s, h, g, b, eps, d, n_rows, (AT*)act_out, plane, f32_out)
  if (dtype == 0) { if (arch == 0) NORM_CASE(float, 0); else NORM_CASE(float, 1); }
  else if (d % 8 == 0 && d <= 8192) {
    bf16_t* out = (bf16_t*)act_out;
    if (arch == 0) {
      if (d <= 2048) launch_norm_bf16<0, 1>(h, g, b, eps, d, n_rows, out, plane, f32_out, max_rows, s, np);
      else if (d <= 4096) launch_norm_bf16<0, 2>(h, g, b, eps, d, n_rows, out, plane, f32_out, max_rows, s, np);
      else launch_norm_bf16<0, 4>(h, g, b, eps, d, n_rows, out, plane, f32_out, max_rows, s, np);
    } else {
      if (d <= 2048) launch_norm_bf16<1, 1>(h, g, b, eps, d, n_rows, out, plane, f32_out, max_rows, s, np);
      else if (d <= 4096) launch_norm_bf16<1, 2>(h, g, b, eps, d, n_rows, out, plane, f32_out, max_rows, s, np);
      else launch_norm_bf16<1, 4>(h, g, b, eps, d, n_rows, out, plane, f32_out, max_rows, s, np);
    }
  }
  else            { if (arch == 0) NORM_CASE(bf16_t, 0); else NORM_CASE(bf16_t, 1); }
#undef NORM_CASE
}

// =================================================================== GEMM
struct GemmArgs {
  const void* W; const void* W2; const void* X; const int* n_rows;
  int N, K, Kt, n_tiles;
  const float* bias; float* out_f32; int ldo; void* out_act; int out_K;
  size_t x_plane;     // elements between the hi and lo planes of X (bf16 mode)
  size_t out_plane;   // same for out_act
  int SK; float* part; size_t part_stride;   // k_gemm16_part: K shares, partial outputs [SK][rows][N], floats per share
};

// bias: the column's bias (0 if none); res: the current value of the output element (residual epilogue only)
template <int EPI, typename AT>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& a, int n_rows, int m, int n, float v, float v2, float bias, float res) {
  if (m >= n_rows || n >= a.N) return;
  if (EPI == EPI_F32) a.out_f32[(size_t)m * a.ldo + n] = v + bias;
  else if (EPI == EPI_RESID) a.out_f32[(size_t)m * a.ldo + n] = res + (v + bias);
  else if (EPI == EPI_GELU) act_store<AT>((AT*)a.out_act, a.out_plane, m, n, a.out_K, gelu_tanh(v + bias));
  else act_store<AT>((AT*)a.out_act, a.out_plane, m, n, a.out_K, silu(v) * v2);
}


// bf16 GEMM on MFMA for at most 16 rows.  512 threads = 8 waves that split K; each wave owns NTW column tiles
// (16 columns each): D[m][n] += X[m][k] W[n][k].
// All 8 waves leave their partial sums in LDS and every thread then finishes ONE output element: it adds the 8
// partials in fixed order, applies bias / residual / GELU / SwiGLU and stores.  With the element order chosen per
// output layout the 256 x NTW stores of the workgroup are contiguous: one 32-column operand tile (two planes) for
// the activation outputs, 64-128 byte runs for float32 rows.  (When wave 0 alone ran the epilogue - 8 tanh and 16
// scattered 2-byte stores per lane for FFN-up - it took 2.2 of the kernel's 7.1 us.)
// Accumulator layout of v_mfma_f32_16x16x32: lane l, register v hold n = l % 16, m = (l / 16) * 4 + v.
template <int NTW, int EPI>
__global__ __launch_bounds__(512) void k_gemm16(GemmArgs a) {
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr bool ACT_OUT = (EPI == EPI_GELU || EPI == EPI_SWIGLU);
  constexpr int U = 4;      // k tiles per chunk and wave (8 and 16 measured slower)
  constexpr int NI = NTW * 4, NI2 = NI * (DUAL ? 2 : 1), NOUT = NTW * 256;
  __shared__ float red[8 * NI2 * 64];
  const int tid = threadIdx.x, lane = tid & 63, kw = wave_index();
  const int nt0 = blockIdx.x * NTW;
  const uint4* __restrict__ Wp = (const uint4*)a.W;
  const uint4* __restrict__ W2p = (const uint4*)a.W2;
  const uint4* __restrict__ Xp = (const uint4*)a.X;
  const uint4* __restrict__ Xl = Xp + a.x_plane / 8;
  const int Kt = a.Kt;
  // Requests that depend on nothing are issued before the row count is even read: this wave's first weight
  // tiles and this thread's bias and (residual epilogue) current output value.
  uint4 wv[U][NTW], wv2[U][DUAL ? NTW : 1];
  auto load_weights = [&](int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int kc = min(kt + u * 8, Kt - 1);                     // clamped: always a valid tile
#pragma unroll
      for (int j = 0; j < NTW; ++j) {
        int nt = min(nt0 + j, a.n_tiles - 1);
        wv[u][j] = Wp[((size_t)nt * Kt + kc) * 64 + lane];
        if (DUAL) wv2[u][j] = W2p[((size_t)nt * Kt + kc) * 64 + lane];
      }
    }
  };
  uint4 xv[U], xl[U];
  auto load_x = [&](int kt) {                               // row tile 0 always exists: no dependence on the row count
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kc = min(kt + u * 8, Kt - 1);
      xv[u] = Xp[(size_t)kc * 64 + lane];
      xl[u] = Xl[(size_t)kc * 64 + lane];
    }
  };
  load_weights(min(kw, Kt - 1));
  load_x(min(kw, Kt - 1));
  // this thread's output element: (row m, column c of the workgroup's 16 NTW columns)
  int m, c;
  if (ACT_OUT) { m = (tid >> 3) & 15; c = (tid >> 7) * 8 + (tid & 7); }      // operand-tile order: 8 columns, 16 rows, next 8 columns
  else { m = tid / (16 * NTW); c = tid % (16 * NTW); }                      // row-major
  const int n = nt0 * 16 + c;
  const bool n_ok = tid < NOUT && n < a.N;
  const float pbias = (n_ok && a.bias) ? a.bias[n] : 0.f;
  const float pres = (EPI == EPI_RESID && n_ok) ? a.out_f32[(size_t)m * a.ldo + n] : 0.f;
  // (The row count is only needed by the epilogue: launches are sized by the host for rows that exist, so the loop
  // does not wait for it.)
  const int n_rows = *a.n_rows;
  f32x4 acc[NTW], acc2[DUAL ? NTW : 1];
#pragma unroll
  for (int j = 0; j < NTW; ++j) {
    acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f};
    if (DUAL) acc2[j] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }
  for (int kt = kw; kt < Kt; kt += 8 * U) {
    // Straight-line code: all loads of a chunk are issued together, k tiles beyond K are clamped on load and
    // zeroed as operands.  (A branch per k tile keeps the scheduler from hoisting the loads and serialises one
    // L2 latency per tile.)
    if (kt != kw) { load_weights(kt); load_x(kt); }         // (the first chunk is already on its way)
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in_k = kt + u * 8 < Kt;
      const uint4 ah = in_k ? xv[u] : make_uint4(0u, 0u, 0u, 0u), al = in_k ? xl[u] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
      for (int j = 0; j < NTW; ++j) {
        acc[j] = mfma_bf16(ah, wv[u][j], acc[j]);
        acc[j] = mfma_bf16(al, wv[u][j], acc[j]);
        if (DUAL) {
          acc2[j] = mfma_bf16(ah, wv2[u][j], acc2[j]);
          acc2[j] = mfma_bf16(al, wv2[u][j], acc2[j]);
        }
      }
    }
  }
  {
    float* dst = red + (size_t)kw * NI2 * 64;
#pragma unroll
    for (int j = 0; j < NTW; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        dst[(j * 4 + v) * 64 + lane] = acc[j][v];
        if (DUAL) dst[(NI + j * 4 + v) * 64 + lane] = acc2[j][v];
      }
  }
  __syncthreads();
  if (tid >= NOUT) return;
  const int it = (c >> 4) * 4 + (m & 3), sl = (m >> 2) * 16 + (c & 15);
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int q = 0; q < 8; ++q) {                             // fixed order: wave 0, 1, ..
    s1 += red[((size_t)q * NI2 + it) * 64 + sl];
    if (DUAL) s2 += red[((size_t)q * NI2 + NI + it) * 64 + sl];
  }
  gemm_epilogue<EPI, bf16_t>(a, n_rows, m, n, s1, s2, pbias, pres);
}

// bf16 GEMM for 17 .. 64 rows per pass (MT row tiles of 16), one column tile per workgroup, K split over
// the 8 waves.  At these row counts a workgroup pulls the whole activation matrix (MT x 2 KiB per k tile,
// from L2) for 1 KiB of weights per k tile, so the kernel lives on memory-level parallelism: two register
// buffers, the loads of chunk c + 1 (weights and all MT row tiles, both planes) are in flight while the
// MFMAs of chunk c run, and there is no branch inside the loop.  Row tiles beyond the row count are
// computed on whatever the buffers hold and dropped by the epilogue; k tiles beyond K are clamped on load
// and their weight operand zeroed.  blockIdx.y = pass over 16 * MT rows.
template <int MT, int NTW, int EPI>
__global__ __launch_bounds__(512) void k_gemm_rows(GemmArgs a) {
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int NWT = NTW * (DUAL ? 2 : 1);          // weight tiles per k tile and wave
  constexpr int U = (MT * NWT >= 8) ? 1 : 2, STEP = 8 * U;   // k tiles per buffer
  constexpr int NI = MT * NWT * 4;
  __shared__ float red[4 * NI * 64];
  const int lane = threadIdx.x & 63, kw = wave_index();
  const int nt0 = blockIdx.x * NTW, mtile0 = blockIdx.y * MT, Kt = a.Kt;
  // EPI_PART: blockIdx.z = K share, the partial product goes to part[share] (summed by the consumer)
  const int sk = (EPI == EPI_PART) ? blockIdx.z : 0, SK = (EPI == EPI_PART) ? gridDim.z : 1;
  const int k0 = (int)((long long)Kt * sk / SK), k1 = (int)((long long)Kt * (sk + 1) / SK);
  const uint4* __restrict__ Wp = (const uint4*)a.W + lane;
  const uint4* __restrict__ W2p = DUAL ? (const uint4*)a.W2 + lane : nullptr;
  const uint4* __restrict__ Xp = (const uint4*)a.X + (size_t)mtile0 * Kt * 64 + lane;
  const uint4* __restrict__ Xl = Xp + a.x_plane / 8;
  size_t wrow[NTW];
#pragma unroll
  for (int j = 0; j < NTW; ++j) wrow[j] = (size_t)min(nt0 + j, a.n_tiles - 1) * Kt * 64;
  struct Buf { uint4 w[U][NWT], xh[U][MT], xl[U][MT]; };
  auto load = [&](Buf& b, int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kc = min(kt + u * 8, k1 - 1);
#pragma unroll
      for (int j = 0; j < NTW; ++j) {
        b.w[u][j] = Wp[wrow[j] + (size_t)kc * 64];
        if (DUAL) b.w[u][NTW + j] = W2p[wrow[j] + (size_t)kc * 64];
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        b.xh[u][mt] = Xp[((size_t)mt * Kt + kc) * 64];
        b.xl[u][mt] = Xl[((size_t)mt * Kt + kc) * 64];
      }
    }
  };
  f32x4 acc[NWT][MT];
#pragma unroll
  for (int j = 0; j < NWT; ++j)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[j][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
  auto compute = [&](const Buf& b, int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in_k = kt + u * 8 < k1;
#pragma unroll
      for (int j = 0; j < NWT; ++j) {
        const uint4 w1 = in_k ? b.w[u][j] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          acc[j][mt] = mfma_bf16(b.xh[u][mt], w1, acc[j][mt]);
          acc[j][mt] = mfma_bf16(b.xl[u][mt], w1, acc[j][mt]);
        }
      }
    }
  };
  Buf A, B;
  load(A, min(k0 + kw, k1 - 1));
  const int n_rows = *a.n_rows;                               // only the epilogue needs it (passes are sized by the host)
  // (the scheduling barriers keep the compiler from sinking a buffer's loads down to their first use)
  for (int kt = k0 + kw; kt < k1; kt += 2 * STEP) {
    load(B, kt + STEP);
    __builtin_amdgcn_sched_barrier(0);
    compute(A, kt);
    __builtin_amdgcn_sched_barrier(0);
    load(A, kt + 2 * STEP);
    __builtin_amdgcn_sched_barrier(0);
    compute(B, kt + STEP);
    __builtin_amdgcn_sched_barrier(0);
  }
  // the 8 partial accumulators are summed pairwise through LDS: (0+4, 1+5, 2+6, 3+7), (0+2, 1+3), (0+1)
#pragma unroll
  for (int half = 4; half >= 1; half >>= 1) {
    if (kw >= half && kw < 2 * half) {
      float* dst = red + (size_t)(kw - half) * NI * 64;
#pragma unroll
      for (int j = 0; j < NWT; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int v = 0; v < 4; ++v) dst[((j * MT + mt) * 4 + v) * 64 + lane] = acc[j][mt][v];
    }
    __syncthreads();
    if (kw < half) {
      const float* src = red + (size_t)kw * NI * 64;
#pragma unroll
      for (int j = 0; j < NWT; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int v = 0; v < 4; ++v) acc[j][mt][v] += src[((j * MT + mt) * 4 + v) * 64 + lane];
    }
    __syncthreads();
  }
  // Wave 0 now holds the totals; it hands them to the whole workgroup through LDS and every thread finishes
  // MT * NTW / 2 (rounded up) output elements, in an order that makes the workgroup's stores contiguous per output layout
  // (one wave running the epilogue for up to 64 values per lane was a serial tail of several microseconds).
  if (kw == 0) {
#pragma unroll
    for (int j = 0; j < NWT; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[((j * MT + mt) * 4 + v) * 64 + lane] = acc[j][mt][v];
  }
  __syncthreads();
  constexpr bool ACT_OUT = (EPI == EPI_GELU || EPI == EPI_SWIGLU);
  float* part = (EPI == EPI_PART) ? a.part + (size_t)sk * a.part_stride : nullptr;
#pragma unroll
  for (int i = 0; i < (MT * NTW + 1) / 2; ++i) {
    const int o = i * 512 + (int)threadIdx.x;        // element index among the MT*16 x NTW*16 outputs
    if (o >= 256 * MT * NTW) break;
    int mt, m16, c;
    if (ACT_OUT) {                                   // operand-tile order: 8 columns, 16 rows, next 8 columns, next row tile
      const int rest = o >> 7;
      m16 = (o >> 3) & 15; c = (rest % (2 * NTW)) * 8 + (o & 7); mt = rest / (2 * NTW);
    } else {                                         // row-major
      const int m_all = o / (16 * NTW);
      c = o % (16 * NTW); mt = m_all >> 4; m16 = m_all & 15;
    }
    const int j = c >> 4, n = nt0 * 16 + c, m = (mtile0 + mt) * 16 + m16;
    const int sl = (m16 >> 2) * 16 + (c & 15), v = m16 & 3;
    const float s1 = red[((j * MT + mt) * 4 + v) * 64 + sl];
    const float s2 = DUAL ? red[(((NTW + j) * MT + mt) * 4 + v) * 64 + sl] : 0.f;
    if (m >= n_rows || n >= a.N) continue;
    if constexpr (EPI == EPI_PART) {
      part[(size_t)m * a.ldo + n] = s1;
    } else {
      const float bias = a.bias ? a.bias[n] : 0.f;
      const float res = (EPI == EPI_RESID) ? a.out_f32[(size_t)m * a.ldo + n] : 0.f;
      gemm_epilogue<EPI, bf16_t>(a, n_rows, m, n, s1, s2, bias, res);
    }
  }
}

// bf16 GEMM for at most 16 rows whose output only has to exist as a sum: O-proj and FFN-down add into the
// residual stream, and the layer norm that follows reads the whole row anyway.  K is split into SK shares
// over workgroups (workgroup = NTW column tiles x one share), each share leaves its partial product in
// part[s] and the norm kernel adds residual + bias + the shares in fixed order.  No reduction step, no
// fences, and every workgroup reads only its share of the activations - which at 16 rows cost as much as
// the weights: a workgroup needs 64 B of activations (L2) per k for 32 B of weights per k and tile.
template <int NTW>
__global__ __launch_bounds__(512) void k_gemm16_part(GemmArgs a) {
  constexpr int U = 4;
  __shared__ float red[8 * NTW * 4 * 64];
  const int lane = threadIdx.x & 63, kw = wave_index();
  const int n_groups = (a.n_tiles + NTW - 1) / NTW;
  const int g = blockIdx.x % n_groups, sk = blockIdx.x / n_groups;
  const int nt0 = g * NTW, Kt = a.Kt;
  const int k0 = (int)((long long)Kt * sk / a.SK), k1 = (int)((long long)Kt * (sk + 1) / a.SK);
  const uint4* __restrict__ Wp = (const uint4*)a.W;
  const uint4* __restrict__ Xp = (const uint4*)a.X;
  const uint4* __restrict__ Xl = Xp + a.x_plane / 8;
  uint4 wv[U][NTW];
  auto load_weights = [&](int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kc = min(kt + u * 8, k1 - 1);                // clamped: always a tile of this share
#pragma unroll
      for (int j = 0; j < NTW; ++j) wv[u][j] = Wp[((size_t)min(nt0 + j, a.n_tiles - 1) * Kt + kc) * 64 + lane];
    }
  };
  uint4 xv[U], xl[U];
  auto load_x = [&](int kt) {                                 // row tile 0 always exists
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kc = min(kt + u * 8, k1 - 1);
      xv[u] = Xp[(size_t)kc * 64 + lane];
      xl[u] = Xl[(size_t)kc * 64 + lane];
    }
  };
  load_weights(min(k0 + kw, k1 - 1));
  load_x(min(k0 + kw, k1 - 1));
  const int n_rows = *a.n_rows;                               // only the stores need it
  f32x4 acc[NTW];
#pragma unroll
  for (int j = 0; j < NTW; ++j) acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f};
  for (int kt = k0 + kw; kt < k1; kt += 8 * U) {
    if (kt != k0 + kw) { load_weights(kt); load_x(kt); }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in_k = kt + u * 8 < k1;
      const uint4 ah = in_k ? xv[u] : make_uint4(0u, 0u, 0u, 0u), al = in_k ? xl[u] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
      for (int j = 0; j < NTW; ++j) {
        acc[j] = mfma_bf16(ah, wv[u][j], acc[j]);
        acc[j] = mfma_bf16(al, wv[u][j], acc[j]);
      }
    }
  }
  {
    float* dst = red + (size_t)kw * NTW * 4 * 64;
#pragma unroll
    for (int j = 0; j < NTW; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) dst[(j * 4 + v) * 64 + lane] = acc[j][v];
  }
  __syncthreads();
  // one output element per thread, row-major: the 8 partial sums in fixed order, stores in 64-128 byte runs
  const int tid = threadIdx.x;
  if (tid >= NTW * 256) return;
  const int m = tid / (16 * NTW), c = tid % (16 * NTW), n = nt0 * 16 + c;
  const int it = (c >> 4) * 4 + (m & 3), sl = (m >> 2) * 16 + (c & 15);
  float sum = 0.f;
#pragma unroll
  for (int q = 0; q < 8; ++q) sum += red[((size_t)q * NTW * 4 + it) * 64 + sl];
  if (n < a.N && m < n_rows) (a.part + (size_t)sk * a.part_stride)[(size_t)m * a.ldo + n] = sum;
}

// float32 GEMM on the vector ALU: one wave per output column, 8 rows at a time.
template <int EPI>
__global__ __launch_bounds__(256) void k_gemm_f32(GemmArgs a) {
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  const int n_rows = *a.n_rows;
  const int lane = threadIdx.x & 63, w = wave_index();
  const int n = blockIdx.x * 4 + w;
  if (n >= a.N || n_rows <= 0) return;
  const int K = a.K;
  const float* __restrict__ wr = (const float*)a.W + (size_t)n * K;
  const float* __restrict__ wr2 = DUAL ? (const float*)a.W2 + (size_t)n * K : nullptr;
  const float* __restrict__ X = (const float*)a.X;
  for (int m0 = 0; m0 < n_rows; m0 += 8) {
    float acc[8], acc2[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = acc2[i] = 0.f;
    for (int k = lane * 4; k < K; k += 256) {
      float4 wv = *reinterpret_cast<const float4*>(wr + k);
      float4 wv2 = DUAL ? *reinterpret_cast<const float4*>(wr2 + k) : make_float4(0, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (m0 + i < n_rows) {
          float4 xv = *reinterpret_cast<const float4*>(X + (size_t)(m0 + i) * K + k);
          acc[i] += xv.x * wv.x + xv.y * wv.y + xv.z * wv.z + xv.w * wv.w;
          if (DUAL) acc2[i] += xv.x * wv2.x + xv.y * wv2.y + xv.z * wv2.z + xv.w * wv2.w;
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float s1 = wave_sum(acc[i]);
      float s2 = DUAL ? wave_sum(acc2[i]) : 0.f;
      if (lane == i && m0 + i < n_rows)
        gemm_epilogue<EPI, float>(a, n_rows, m0 + i, n, s1, s2, a.bias ? a.bias[n] : 0.f,
                                  EPI == EPI_RESID ? a.out_f32[(size_t)(m0 + i) * a.ldo + n] : 0.f);
    }
  }
}

template <int EPI>
static void launch_gemm_bf16(const GemmArgs& a, int max_rows, hipStream_t s) {
  // Up to 16 rows: one 16-column tile per workgroup (two per wave for wide outputs), K split over its 8 waves.
  // (Measured and dropped for that case: folding the layer norm into this kernel - every workgroup
  // then normalises the whole activation matrix again, 13.6 us against 5.3 + 5.0 us for norm + GEMM at
  // d = 1600 - and splitting K over workgroups with a last-arriver reduction - its two device-scope fences
  // cost more than the 4 us they save; and a variant that requests all of a wave's weight and activation
  // tiles up front (K <= 2048) - no faster.)
  // 17 .. 64 rows: 2, 3 or 4 row tiles per pass with double-buffered loads; more rows take further passes.
  // wide outputs with a short K: two column tiles per wave share the activation fragments (at K = 4096 one tile per
  // workgroup is faster: QKV 12288x4096 26 against 32 us, FFN-up 2x11008x4096 40 against 48 us)
  if (max_rows <= 16 && a.n_tiles >= 256 && a.Kt < 100)
    hipLaunchKernelGGL((k_gemm16<2, EPI>), dim3((a.n_tiles + 1) / 2), dim3(512), 0, s, a);
  else if (max_rows <= 16) hipLaunchKernelGGL((k_gemm16<1, EPI>), dim3(a.n_tiles), dim3(512), 0, s, a);
  else {
    // column tiles per wave that share the activation fragments: as many as leave about 192 workgroups
    const int passes = (max_rows + 63) / 64;
    const int mt = max_rows <= 32 ? 2 : max_rows <= 48 ? 3 : 4;
    constexpr bool DUAL = EPI == EPI_SWIGLU;
    const int ntw = (!DUAL && mt > 2 && a.n_tiles / 4 >= 192) ? 4 : (a.n_tiles / 2 >= (DUAL ? 256 : 128)) ? 2 : 1;
    const dim3 grid((a.n_tiles + ntw - 1) / ntw, passes, 1);
#define SPRINTER_ROWS(MT_, NTW_) hipLaunchKernelGGL((k_gemm_rows<MT_, NTW_, EPI>), grid, dim3(512), 0, s, a)
    if (ntw == 4) { if (mt == 3) SPRINTER_ROWS(3, 4); else SPRINTER_ROWS(4, 4); }
    else if (ntw == 2) { if (mt == 2) SPRINTER_ROWS(2, 2); else if (mt == 3) SPRINTER_ROWS(3, 2); else SPRINTER_ROWS(4, 2); }
    else { if (mt == 2) SPRINTER_ROWS(2, 1); else if (mt == 3) SPRINTER_ROWS(3, 1); else SPRINTER_ROWS(4, 1); }
#undef SPRINTER_ROWS
  }
}

void launch_gemm(int dtype, int epi, const void* W, const void* W2, const void* X, size_t x_plane, const int* n_rows,
                 int N, int K, const float* bias, float* out_f32, int ldo, void* out_act, int out_K, size_t out_plane,
                 int max_rows, hipStream_t s) {
  GemmArgs a;
  memset(&a, 0, sizeof a);
  a.x_plane = x_plane; a.out_plane = out_plane;
  a.W = W; a.W2 = W2; a.X = X; a.n_rows = n_rows; a.N = N; a.K = K;
  a.Kt = (K + 31) / 32; a.n_tiles = (N + 15) / 16;
  a.bias = bias; a.out_f32 = out_f32; a.ldo = ldo; a.out_act = out_act; a.out_K = out_K;
  if (dtype == 0) {
    dim3 grid((N + 3) / 4), block(256);
    switch (epi) {
      case EPI_F32: hipLaunchKernelGGL(k_gemm_f32<EPI_F32>, grid, block, 0, s, a); break;
      case EPI_RESID: hipLaunchKernelGGL(k_gemm_f32<EPI_RESID>, grid, block, 0, s, a); break;
      case EPI_GELU: hipLaunchKernelGGL(k_gemm_f32<EPI_GELU>, grid, block, 0, s, a); break;
      default: hipLaunchKernelGGL(k_gemm_f32<EPI_SWIGLU>, grid, block, 0, s, a); break;
    }
  } else {
    switch (epi) {
      case EPI_F32: launch_gemm_bf16<EPI_F32>(a, max_rows, s); break;
      case EPI_RESID: launch_gemm_bf16<EPI_RESID>(a, max_rows, s); break;
      case EPI_GELU: launch_gemm_bf16<EPI_GELU>(a, max_rows, s); break;
      default: launch_gemm_bf16<EPI_SWIGLU>(a, max_rows, s); break;
    }
  }
}

int launch_gemm_part(const void* W, const void* X, size_t x_plane, const int* n_rows, int N, int K, float* part,
                     size_t part_stride, int max_shares, int max_rows, hipStream_t s) {
  GemmArgs a;
  memset(&a, 0, sizeof a);
  a.W = W; a.X = X; a.x_plane = x_plane; a.n_rows = n_rows; a.N = N; a.K = K;
  a.Kt = (K + 31) / 32; a.n_tiles = (N + 15) / 16; a.ldo = N;
  a.part = part; a.part_stride = part_stride;
  if (max_rows <= 16) {
    // shares: fill the 256 compute units, at least 12 k tiles per share; long K takes two column tiles per wave
    const bool two = a.Kt >= 192 && a.n_tiles >= 64;   // (4096x4096: 8.2 us with one tile, 10.5 with two; 4096x11008: 24.1 / 19.8)
    const int groups = two ? (a.n_tiles + 1) / 2 : a.n_tiles;
    int sk = std::min(4, 256 / groups);              // (4: the norm kernel's smaller partial-sum variant)
    if (sk > max_shares) sk = max_shares;
    while (sk > 1 && a.Kt / sk < 12) --sk;
    if (sk < 1) sk = 1;
    a.SK = sk;
    if (two) hipLaunchKernelGGL((k_gemm16_part<2>), dim3(groups * sk), dim3(512), 0, s, a);
    else hipLaunchKernelGGL((k_gemm16_part<1>), dim3(groups * sk), dim3(512), 0, s, a);
    return sk;
  }
  // 17+ rows: the workgroup's activation traffic (2 KiB per k tile and 16 rows) is what costs, so a wave takes
  // four column tiles (two if that leaves too few workgroups) and K is split until about 256 workgroups exist,
  // with at least two k tiles per wave and share
  const int passes = (max_rows + 63) / 64;
  const int mt = max_rows <= 32 ? 2 : max_rows <= 48 ? 3 : 4;
  const int s_max = std::max(1, std::min(max_shares, a.Kt / 16));
  int ntw = 4, groups = (a.n_tiles + 3) / 4, sk = std::min(s_max, std::max(1, 256 / groups));
  if (groups * sk < 192) { ntw = 2; groups = (a.n_tiles + 1) / 2; sk = std::min(s_max, std::max(1, 256 / groups)); }
  a.SK = sk;
  const dim3 grid(groups, passes, sk);
#define SPRINTER_PART(MT_, NTW_) hipLaunchKernelGGL((k_gemm_rows<MT_, NTW_, EPI_PART>), grid, dim3(512), 0, s, a)
  if (ntw == 4) { if (mt == 2) SPRINTER_PART(2, 4); else if (mt == 3) SPRINTER_PART(3, 4); else SPRINTER_PART(4, 4); }
  else { if (mt == 2) SPRINTER_PART(2, 2); else if (mt == 3) SPRINTER_PART(3, 2); else SPRINTER_PART(4, 2); }
#undef SPRINTER_PART
  return sk;
}

// ============================================================== attention
// One workgroup per (row, KV head): rotary on q and the new k, append k/v to the
// cache, scores against all cached keys, softmax, weighted sum of values.
// The G query heads that share the KV head are processed together.
struct AttnArgs {
  const float* y; const float* rope; RowDesc rd;
  void* kcache; void* vcache; size_t layer_off;
  int H, KVH, dqkv, max_seq, use_rope; float scale;
  void* ao; int ao_K; size_t ao_plane;
  int phase;   // 0 append + attend, 1 append only, 2 attend only
};

template <typename T, int DH, int G>
__global__ __launch_bounds__(256) void k_attn(AttnArgs a) {
  extern __shared__ float smem[];
  __shared__ float s4[4];
  __shared__ float s_inv[G];
  float* qs = smem;                    // [G][DH]
  float* knew = qs + G * DH;           // [DH]
  float* vnew = knew + DH;             // [DH]
  float* red = vnew + DH;              // [4][G][DH]
  float* sc = red + 4 * G * DH;        // [G][max_seq]
  const int r = blockIdx.y;
  if (r >= *a.rd.n_rows) return;
  const int kvh = blockIdx.x, tid = threadIdx.x;
  const int b = a.rd.b[r], slot = a.rd.slot[r], nk = slot + 1, S = a.max_seq;
  const float* __restrict__ y = a.y + (size_t)r * a.dqkv;
  const float* __restrict__ cs = a.rope + (size_t)r * DH;
  constexpr int HALF = DH / 2;
  for (int idx = tid; idx < G * DH; idx += 256) {
    int g = idx / DH, i = idx % DH;
    const float* qh = y + (size_t)(kvh * G + g) * DH;
    float val = qh[i];
    if (a.use_rope) {
      int j = i < HALF ? i : i - HALF;
      float c = cs[2 * j], sn = cs[2 * j + 1];
      val = i < HALF ? qh[i] * c - qh[i + HALF] * sn : qh[i] * c + qh[i - HALF] * sn;
    }
    qs[idx] = val * a.scale;
  }
  T* __restrict__ Kc = (T*)a.kcache + a.layer_off + ((size_t)b * a.KVH + kvh) * (size_t)S * DH;
  T* __restrict__ Vc = (T*)a.vcache + a.layer_off + ((size_t)b * a.KVH + kvh) * (size_t)S * DH;
  for (int i = tid; i < DH; i += 256) {
    const float* kh = y + (size_t)(a.H + kvh) * DH;
    const float* vh = y + (size_t)(a.H + a.KVH + kvh) * DH;
    float kv = kh[i];
    if (a.use_rope) {
      int j = i < HALF ? i : i - HALF;
      float c = cs[2 * j], sn = cs[2 * j + 1];
      kv = i < HALF ? kh[i] * c - kh[i + HALF] * sn : kh[i] * c + kh[i - HALF] * sn;
    }
    T kt = from_f<T>(kv), vt = from_f<T>(vh[i]);
    if (a.phase != 2) {
      Kc[(size_t)slot * DH + i] = kt;
      Vc[(size_t)slot * DH + i] = vt;
    }
    knew[i] = to_f<T>(kt);             // the entry as later steps will read it back
    vnew[i] = to_f<T>(vt);
  }
  if (a.phase == 1) return;
  __syncthreads();

  constexpr int EPL = 16 / sizeof(T);  // elements per 16-byte lane load
  constexpr int LPK = DH / EPL;        // lanes per key
  constexpr int KPW = 64 / LPK;        // keys per wave per iteration
  const int lane = tid & 63, w = tid >> 6;
  const int chunk = lane % LPK, kin = lane / LPK;
  float qreg[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPL; ++e) qreg[g][e] = qs[g * DH + chunk * EPL + e];

  // pass 1: scores
  for (int key0 = w * KPW; key0 < nk; key0 += 4 * KPW) {
    int key = key0 + kin;
    float kv[EPL];
    if (key < slot) {
      uint4 raw = *reinterpret_cast<const uint4*>(Kc + (size_t)key * DH + chunk * EPL);
      const T* t = reinterpret_cast<const T*>(&raw);
#pragma unroll
      for (int e = 0; e < EPL; ++e) kv[e] = to_f<T>(t[e]);
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
  // softmax over the nk keys of every head
  for (int g = 0; g < G; ++g) {
    float mx = -INFINITY;
    for (int k = tid; k < nk; k += 256) mx = fmaxf(mx, sc[g * S + k]);
    mx = block_max256(mx, s4);
    float sum = 0.f;
    for (int k = tid; k < nk; k += 256) {
      float e = expf(sc[g * S + k] - mx);
      sc[g * S + k] = e;
      sum += e;
    }
    sum = block_sum256(sum, s4);
    if (tid == 0) s_inv[g] = 1.0f / sum;
  }
  __syncthreads();
  // pass 2: weighted values
  float acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  for (int key0 = w * KPW; key0 < nk; key0 += 4 * KPW) {
    int key = key0 + kin;
    float vv[EPL];
    if (key < slot) {
      uint4 raw = *reinterpret_cast<const uint4*>(Vc + (size_t)key * DH + chunk * EPL);
      const T* t = reinterpret_cast<const T*>(&raw);
#pragma unroll
      for (int e = 0; e < EPL; ++e) vv[e] = to_f<T>(t[e]);
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
  T* __restrict__ ao = (T*)a.ao;
  for (int idx = tid; idx < G * DH; idx += 256) {
    int g = idx / DH;
    float o = ((red[idx] + red[G * DH + idx]) + red[2 * G * DH + idx]) + red[3 * G * DH + idx];
    o *= s_inv[g];
    act_store<T>(ao, a.ao_plane, r, kvh * G * DH + idx, a.ao_K, o);
  }
}

// bf16 single-query attention with a short dependency chain: one workgroup (4 waves) per (row, KV head).
// Once the row's cache slot is known, every wave requests its share of the cached keys AND values
// at once (they do not depend on the new query), then the query / new key / new value; each lane
// group runs an online softmax over its own keys, the groups are merged by shuffles, the 4 waves
// and the new key by one pass through LDS: a single block-wide synchronisation.
//   lane = kin * LPK + chunk: LPK = DH / 8 lanes share one key (8 elements each), a wave-wide
//   16-byte load covers KPW = 64 / LPK consecutive keys; wave w takes key blocks w, w + 4, ...
template <int DH, int G, int NW>
__global__ __launch_bounds__(NW * 64) void k_attn_bf16(AttnArgs a) {
  constexpr int LPK = DH / 8, KPW = 64 / LPK, HALF = DH / 2;
  constexpr int NB = (G <= 4 && DH == 64) ? 8 : 4;       // key blocks held in registers per round and wave
  constexpr float NEG = -1e30f;
  __shared__ float s_m[NW][G], s_l[NW][G], s_o[NW][G][DH], s_vnew[DH], s_snew[G];
  const int r = blockIdx.y;
  if (r >= *a.rd.n_rows) return;
  const int kvh = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = wave_index();
  const int chunk = lane % LPK, kin = lane / LPK;
  const int b = a.rd.b[r], slot = a.rd.slot[r], S = a.max_seq;
  bf16_t* __restrict__ Kc = (bf16_t*)a.kcache + a.layer_off + ((size_t)b * a.KVH + kvh) * (size_t)S * DH;
  bf16_t* __restrict__ Vc = (bf16_t*)a.vcache + a.layer_off + ((size_t)b * a.KVH + kvh) * (size_t)S * DH;
  const int n_blocks = (slot + KPW - 1) / KPW;                 // blocks of cached keys
  const int n_rounds = (n_blocks + NW * NB - 1) / (NW * NB);
  // Two register buffers where the registers are there (head dimension 128, at most 2 query heads per KV head): the
  // keys and values of round rd + 1 are in flight while round rd is consumed (c4's step 15.5 -> 14.5 ms).  With more
  // query heads or 64-wide heads the second buffer costs occupancy and measured slower (c5's draft 38.6 -> 45.5 us).
  constexpr bool TWO_BUFFERS = DH == 128 && G <= 2;
  uint4 kA[NB], vA[NB], kB[TWO_BUFFERS ? NB : 1], vB[TWO_BUFFERS ? NB : 1];
  auto request = [&](uint4* kb, uint4* vb, int rd) {           // clamped addresses, no branches
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int key = min(((rd * NB + j) * NW + w) * KPW + kin, max(slot - 1, 0));
      kb[j] = *reinterpret_cast<const uint4*>(Kc + (size_t)key * DH + chunk * 8);
      vb[j] = *reinterpret_cast<const uint4*>(Vc + (size_t)key * DH + chunk * 8);
    }
  };
  request(kA, vA, 0);
  // Query heads, new key and new value: this lane's 8 elements and their rotary partners.  Everything is requested
  // up front as unconditional 16-byte loads (2 G + 3 pairs from the projection row, 4 from the cos / sin row) and only
  // then used: with a branch on the rotary flag between the loads each head paid its own memory round trip (12 us
  // before the first key at 4 query heads per KV head).  Without rotary the partner values are multiplied by 0.
  const float* __restrict__ y = a.y + (size_t)r * a.dqkv;
  const bool upper = chunk >= LPK / 2;
  const int pchunk = chunk ^ (LPK / 2);
  auto load8 = [&](const float* src, float* out) {            // 32-byte aligned: all offsets are multiples of 8 floats
    const float4 lo = reinterpret_cast<const float4*>(src)[0], hi = reinterpret_cast<const float4*>(src)[1];
    out[0] = lo.x; out[1] = lo.y; out[2] = lo.z; out[3] = lo.w; out[4] = hi.x; out[5] = hi.y; out[6] = hi.z; out[7] = hi.w;
  };
  float qx[G][8], qp[G][8], kx[8], kp[8], vnew[8], csr[16];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    load8(y + (size_t)(kvh * G + g) * DH + chunk * 8, qx[g]);
    load8(y + (size_t)(kvh * G + g) * DH + pchunk * 8, qp[g]);
  }
  load8(y + (size_t)(a.H + kvh) * DH + chunk * 8, kx);
  load8(y + (size_t)(a.H + kvh) * DH + pchunk * 8, kp);
  load8(y + (size_t)(a.H + a.KVH + kvh) * DH + chunk * 8, vnew);
  {
    const float* __restrict__ cs = a.rope + (size_t)r * DH + 2 * (chunk % (LPK / 2)) * 8;   // (cos, sin) pairs of this lane's 8 angles
    load8(cs, csr);
    load8(cs + 8, csr + 8);
  }
  float cr[8], sr[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { cr[e] = a.use_rope ? csr[2 * e] : 1.f; sr[e] = a.use_rope ? csr[2 * e + 1] : 0.f; }
  float q[G][8], knew[8];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e)
      q[g][e] = (upper ? qx[g][e] * cr[e] + qp[g][e] * sr[e] : qx[g][e] * cr[e] - qp[g][e] * sr[e]) * a.scale;
#pragma unroll
  for (int e = 0; e < 8; ++e) knew[e] = upper ? kx[e] * cr[e] + kp[e] * sr[e] : kx[e] * cr[e] - kp[e] * sr[e];
  unsigned kpk[4], vpk[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float v0 = vnew[2 * e], v1 = vnew[2 * e + 1];
    const bf16_t k0 = f2bf(knew[2 * e]), k1 = f2bf(knew[2 * e + 1]), w0 = f2bf(v0), w1 = f2bf(v1);
    kpk[e] = (unsigned)k0 | ((unsigned)k1 << 16);
    vpk[e] = (unsigned)w0 | ((unsigned)w1 << 16);
    knew[2 * e] = bf2f(k0); knew[2 * e + 1] = bf2f(k1);         // the entry as later steps will read it back
    vnew[2 * e] = bf2f(w0); vnew[2 * e + 1] = bf2f(w1);
  }
  if (w == 0 && kin == 0) {                                     // append to the cache
    if (a.phase != 2) {
      *reinterpret_cast<uint4*>(Kc + (size_t)slot * DH + chunk * 8) = make_uint4(kpk[0], kpk[1], kpk[2], kpk[3]);
      *reinterpret_cast<uint4*>(Vc + (size_t)slot * DH + chunk * 8) = make_uint4(vpk[0], vpk[1], vpk[2], vpk[3]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) s_vnew[chunk * 8 + e] = vnew[e];
  }
  if (a.phase == 1) return;
  float snew[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float p = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) p += q[g][e] * knew[e];
    snew[g] = group_sum<LPK>(p);
  }
  if (w == 0 && lane == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) s_snew[g] = snew[g];
  }
  // online softmax over this lane group's keys
  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = NEG; l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
  }
  // One softmax rescale per round instead of one per key block: the round's scores first, then their maximum, one
  // correction of the running sums, then the weighted values.
  auto consume = [&](const uint4* kb, const uint4* vb, int rd) {
    float sc[NB][G];
    bool valid[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int key = ((rd * NB + j) * NW + w) * KPW + kin;
      valid[j] = key < slot;
      const bf16_t* kt = reinterpret_cast<const bf16_t*>(&kb[j]);
      float kf[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) kf[e] = bf2f(kt[e]);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) d += q[g][e] * kf[e];
        sc[j][g] = group_sum<LPK>(d);
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mn = m[g];
#pragma unroll
      for (int j = 0; j < NB; ++j) mn = valid[j] ? fmaxf(mn, sc[j][g]) : mn;
      const float corr = __expf(m[g] - mn);
      m[g] = mn;
      l[g] *= corr;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[g][e] *= corr;
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const bf16_t* vt = reinterpret_cast<const bf16_t*>(&vb[j]);
      float vf[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) vf[e] = valid[j] ? bf2f(vt[e]) : 0.f;   // (an empty cache holds no finite data yet)
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float p = valid[j] ? __expf(sc[j][g] - m[g]) : 0.f;
        l[g] += p;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] += p * vf[e];
      }
    }
  };
  if constexpr (TWO_BUFFERS) {
    for (int rd = 0; rd < n_rounds; rd += 2) {    // (a round beyond the last one consumes nothing: all its keys are masked)
      request(kB, vB, rd + 1);
      __builtin_amdgcn_sched_barrier(0);
      consume(kA, vA, rd);
      __builtin_amdgcn_sched_barrier(0);
      request(kA, vA, rd + 2);
      __builtin_amdgcn_sched_barrier(0);
      consume(kB, vB, rd + 1);
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
    for (int rd = 0; rd < n_rounds; ++rd) {
      if (rd > 0) request(kA, vA, rd);
      consume(kA, vA, rd);
    }
  }
  // merge the KPW lane groups of the wave
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int o = LPK; o < 64; o <<= 1) {
      const float mo = __shfl_xor(m[g], o), lo = __shfl_xor(l[g], o);
      const float mn = fmaxf(m[g], mo);
      const float c1 = __expf(m[g] - mn), c2 = __expf(mo - mn);
      l[g] = l[g] * c1 + lo * c2;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[g][e] = acc[g][e] * c1 + __shfl_xor(acc[g][e], o) * c2;
      m[g] = mn;
    }
    if (kin == 0) {
      if (chunk == 0) { s_m[w][g] = m[g]; s_l[w][g] = l[g]; }
#pragma unroll
      for (int e = 0; e < 8; ++e) s_o[w][g][chunk * 8 + e] = acc[g][e];
    }
  }
  __syncthreads();
  // merge the NW waves and the new key; one output element per thread and pass
  bf16_t* __restrict__ ao = (bf16_t*)a.ao;
  for (int idx = tid; idx < G * DH; idx += NW * 64) {
    const int g = idx / DH, i = idx % DH;
    const float sn = s_snew[g];
    float mn = sn;
#pragma unroll
    for (int q4 = 0; q4 < NW; ++q4) mn = fmaxf(mn, s_m[q4][g]);
    float den = __expf(sn - mn), num = den * s_vnew[i];
#pragma unroll
    for (int q4 = 0; q4 < NW; ++q4) {
      const float c = __expf(s_m[q4][g] - mn);
      den += c * s_l[q4][g];
      num += c * s_o[q4][g][i];
    }
    act_store<bf16_t>(ao, a.ao_plane, r, kvh * G * DH + idx, a.ao_K, num / den);
  }
}

static size_t attn_smem_bytes(int DH, int G, int max_seq) {
  return (size_t)(G * DH + 2 * DH + 4 * G * DH + G * max_seq) * sizeof(float);
}

template <int DH>
static void launch_attn_bf16(const AttnArgs& a, int G, int max_rows, int ctx_bound, hipStream_t s) {
  // NW = waves per workgroup that share one (row, KV head)'s keys: 8 when the launch has no more workgroups than
  // the chip has compute units and the contexts are long (c5's target pass: 20 rows x 8 KV heads x 1000+ keys),
  // else 4 (at c2's 130-400 keys the 8-wave variant takes 9.5 us against 7.8)
  dim3 grid(a.KVH, max_rows);
  const bool wide = (long long)a.KVH * max_rows <= 256 && ctx_bound >= 512;
#define SPRINTER_ATTN(G_) do { if (wide) hipLaunchKernelGGL((k_attn_bf16<DH, G_, 8>), grid, dim3(512), 0, s, a); \
                               else hipLaunchKernelGGL((k_attn_bf16<DH, G_, 4>), grid, dim3(256), 0, s, a); } while (0)
  switch (G) {
    case 1: SPRINTER_ATTN(1); break;
    case 2: SPRINTER_ATTN(2); break;
    case 4: SPRINTER_ATTN(4); break;
    default: hipLaunchKernelGGL((k_attn_bf16<DH, 8, 4>), grid, dim3(256), 0, s, a); break;   // (8 waves would spill)
  }
#undef SPRINTER_ATTN
}

template <typename T, int DH>
static void launch_attn_g(const AttnArgs& a, int G, int max_rows, hipStream_t s) {
  dim3 grid(a.KVH, max_rows), block(256);
  size_t sm = attn_smem_bytes(DH, G, a.max_seq);
  switch (G) {
    case 1: hipLaunchKernelGGL((k_attn<T, DH, 1>), grid, block, sm, s, a); break;
    case 2: hipLaunchKernelGGL((k_attn<T, DH, 2>), grid, block, sm, s, a); break;
    case 4: hipLaunchKernelGGL((k_attn<T, DH, 4>), grid, block, sm, s, a); break;
    default: hipLaunchKernelGGL((k_attn<T, DH, 8>), grid, block, sm, s, a); break;
  }
}

void launch_attention(int dtype, const ModelDims& md, const float* y, const float* rope, const RowDesc& rd,
                      void* kcache, void* vcache, size_t layer_off, int ctx_bound, int max_seq, void* ao,
                      size_t ao_plane, int max_rows, hipStream_t s, int phase) {
  AttnArgs a;
  a.phase = phase;
  a.y = y; a.rope = rope; a.rd = rd; a.kcache = kcache; a.vcache = vcache; a.layer_off = layer_off;
  a.H = md.H; a.KVH = md.KVH; a.dqkv = md.dqkv; a.max_seq = max_seq; a.use_rope = md.arch == 1;
  a.scale = 1.0f / sqrtf((float)md.dh);
  a.ao = ao; a.ao_K = md.H * md.dh; a.ao_plane = ao_plane;
  int G = md.H / md.KVH;
  if (dtype == 0) {
    if (md.dh == 64) launch_attn_g<float, 64>(a, G, max_rows, s); else launch_attn_g<float, 128>(a, G, max_rows, s);
  } else {
    if (md.dh == 64) launch_attn_bf16<64>(a, G, max_rows, ctx_bound, s); else launch_attn_bf16<128>(a, G, max_rows, ctx_bound, s);
  }
}

// ======================================================= LM head + sample
struct LmArgs {
  const void* W; const void* X; RowDesc rd; int V, K, Kt, n_tiles;
  SamplerArgs sa; u64* part; int Mpad; float* logits_out; size_t x_plane;
};

// bf16: each workgroup owns a contiguous range of column tiles; its 8 waves take pairs of adjacent tiles
// round-robin (the two tiles share the activation fragments: at 16+ rows the activations, 2 KiB per k tile and
// row tile from L2, outweigh the 1 KiB of weights), keep a running (value, index) maximum per row, and the
// workgroup writes one partial per row.  The k loop has no branches: two register buffers, tiles and k tiles
// beyond the end are clamped on load; columns beyond the vocabulary and rows beyond the row count are dropped
// when the logits are sampled.  More than 16 MT rows take further passes over the workgroup's tiles.
template <int MT>
__global__ __launch_bounds__(512) void k_lmhead_bf16(LmArgs a) {
  __shared__ u64 sbest[8][MT * 16];
  __shared__ int s_rb[MT * 16], s_rt[MT * 16];
  const int lane = threadIdx.x & 63, w = wave_index();
  const int tpw = (a.n_tiles + gridDim.x - 1) / gridDim.x;
  const int t0 = blockIdx.x * tpw, t1 = min(t0 + tpw, a.n_tiles);
  const uint4* __restrict__ Wp = (const uint4*)a.W + lane;
  const uint4* __restrict__ Xp = (const uint4*)a.X + lane;
  const uint4* __restrict__ Xl = Xp + a.x_plane / 8;
  const int Kt = a.Kt;
  const int n_rows = *a.rd.n_rows;
  struct Buf { uint4 w[2], xh[MT], xl[MT]; };
  for (int m0 = 0; m0 < n_rows; m0 += MT * 16) {
    const int mtile0 = m0 >> 4;
    u64 best[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int v = 0; v < 4; ++v) best[mt][v] = 0;
    for (int i = threadIdx.x; i < MT * 16; i += 512) {     // the rows' random streams: batch row, position being generated
      s_rb[i] = m0 + i < n_rows ? a.rd.b[m0 + i] : 0;
      s_rt[i] = m0 + i < n_rows ? a.rd.pos[m0 + i] + 1 : 0;
    }
    __syncthreads();
    for (int nt = t0 + 2 * w; nt < t1; nt += 16) {
      const size_t wrow0 = (size_t)nt * Kt * 64, wrow1 = (size_t)min(nt + 1, t1 - 1) * Kt * 64;
      auto load = [&](Buf& b, int kt) {
        const int kc = min(kt, Kt - 1);
        b.w[0] = Wp[wrow0 + (size_t)kc * 64];
        b.w[1] = Wp[wrow1 + (size_t)kc * 64];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {                 // (row tiles beyond the rows hold old data: dropped below)
          b.xh[mt] = Xp[((size_t)(mtile0 + mt) * Kt + kc) * 64];
          b.xl[mt] = Xl[((size_t)(mtile0 + mt) * Kt + kc) * 64];
        }
      };
      f32x4 acc[2][MT];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[j][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      auto compute = [&](const Buf& b, int kt) {
        const bool in_k = kt < Kt;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const uint4 wj = in_k ? b.w[j] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            acc[j][mt] = mfma_bf16(b.xh[mt], wj, acc[j][mt]);
            acc[j][mt] = mfma_bf16(b.xl[mt], wj, acc[j][mt]);
          }
        }
      };
      Buf A, B;
      load(A, 0);
      for (int kt = 0; kt < Kt; kt += 2) {
        load(B, kt + 1);
        __builtin_amdgcn_sched_barrier(0);
        compute(A, kt);
        __builtin_amdgcn_sched_barrier(0);
        load(A, kt + 2);
        __builtin_amdgcn_sched_barrier(0);
        compute(B, kt + 1);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = (nt + j) * 16 + (lane & 15);
        if (nt + j < t1 && n < a.V) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              int m = m0 + mt * 16 + (lane >> 4) * 4 + v;
              if (m < n_rows) {
                float logit = acc[j][mt][v];
                if (a.logits_out) a.logits_out[(size_t)m * a.V + n] = logit;
                const int mi = mt * 16 + (lane >> 4) * 4 + v;
                best[mt][v] = umax64(best[mt][v], sample_key(logit, a.sa, s_rb[mi], s_rt[mi], n));
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
        if ((lane & 15) == 0) sbest[w][mt * 16 + (lane >> 4) * 4 + v] = k;
      }
    __syncthreads();
    for (int i = threadIdx.x; i < MT * 16; i += 512) {
      u64 k = sbest[0][i];
#pragma unroll
      for (int q = 1; q < 8; ++q) k = umax64(k, sbest[q][i]);
      if (m0 + i < a.Mpad) a.part[(size_t)blockIdx.x * a.Mpad + m0 + i] = k;
    }
    __syncthreads();
  }
}

// float32: one wave per vocabulary column, 8 rows at a time.
__global__ __launch_bounds__(256) void k_lmhead_f32(LmArgs a) {
  __shared__ u64 sbest[4][8];
  const int n_rows = *a.rd.n_rows;
  if (n_rows <= 0) return;
  const int lane = threadIdx.x & 63, w = wave_index();
  const int cpw = (a.V + gridDim.x - 1) / gridDim.x;
  const int c0 = blockIdx.x * cpw, c1 = min(c0 + cpw, a.V);
  const int K = a.K;
  const float* __restrict__ W = (const float*)a.W;
  const float* __restrict__ X = (const float*)a.X;
  for (int m0 = 0; m0 < n_rows; m0 += 8) {
    u64 best = 0;
    const int my_m = m0 + lane;
    const int my_b = (lane < 8 && my_m < n_rows) ? a.rd.b[my_m] : 0;
    const int my_t = (lane < 8 && my_m < n_rows) ? a.rd.pos[my_m] + 1 : 0;
    for (int n = c0 + w; n < c1; n += 4) {
      const float* wr = W + (size_t)n * K;
      float acc[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = 0.f;
      for (int k = lane * 4; k < K; k += 256) {
        float4 wv = *reinterpret_cast<const float4*>(wr + k);
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (m0 + i < n_rows) {
            float4 xv = *reinterpret_cast<const float4*>(X + (size_t)(m0 + i) * K + k);
            acc[i] += xv.x * wv.x + xv.y * wv.y + xv.z * wv.z + xv.w * wv.w;
          }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float sacc = wave_sum(acc[i]);
        if (lane == i && m0 + i < n_rows) {
          if (a.logits_out) a.logits_out[(size_t)(m0 + i) * a.V + n] = sacc;
          best = umax64(best, sample_key(sacc, a.sa, my_b, my_t, n));
        }
      }
    }
    if (lane < 8) sbest[w][lane] = best;
    __syncthreads();
    if (threadIdx.x < 8 && m0 + (int)threadIdx.x < a.Mpad) {
      u64 k = umax64(umax64(sbest[0][threadIdx.x], sbest[1][threadIdx.x]),
                     umax64(sbest[2][threadIdx.x], sbest[3][threadIdx.x]));
      a.part[(size_t)blockIdx.x * a.Mpad + m0 + threadIdx.x] = k;
    }
    __syncthreads();
  }
}

int lmhead_num_wg(int dtype, int V) {
  int n = (dtype == 0) ? (V + 7) / 8 : ((V + 15) / 16 + 7) / 8;
  return n < 512 ? n : 512;
}

void launch_lmhead(int dtype, const void* W, const void* X, size_t x_plane, const RowDesc& rd, int V, int K,
                   const SamplerArgs& sa, unsigned long long* part, int n_wg, int Mpad, float* logits_out, int max_rows,
                   hipStream_t s) {
  LmArgs a;
  a.x_plane = x_plane;
  a.W = W; a.X = X; a.rd = rd; a.V = V; a.K = K; a.Kt = (K + 31) / 32; a.n_tiles = (V + 15) / 16;
  a.sa = sa; a.part = part; a.Mpad = Mpad; a.logits_out = logits_out;
  if (dtype == 0) {
    hipLaunchKernelGGL(k_lmhead_f32, dim3(n_wg), dim3(256), 0, s, a);
  } else if (max_rows <= 16) {
    hipLaunchKernelGGL(k_lmhead_bf16<1>, dim3(n_wg), dim3(512), 0, s, a);
  } else if (max_rows <= 32) {
    hipLaunchKernelGGL(k_lmhead_bf16<2>, dim3(n_wg), dim3(512), 0, s, a);
  } else if (max_rows <= 48) {
    hipLaunchKernelGGL(k_lmhead_bf16<3>, dim3(n_wg), dim3(512), 0, s, a);
  } else {                                   // 4 row tiles per pass; more rows take further passes inside the kernel
    hipLaunchKernelGGL(k_lmhead_bf16<4>, dim3(n_wg), dim3(512), 0, s, a);
  }
}

// =============================================================== verifier
// Hidden layer of the verifier MLP, spread over workgroups of 8 waves (one hidden
// unit per wave); each workgroup leaves its share of the output logit per row.
// d_hidden == 0: the logit is w2 . hf (a single chunk).
__global__ __launch_bounds__(512) void k_verifier_part(const float* __restrict__ hf, int d, int d_hidden,
                                                       const float* __restrict__ w1, const float* __restrict__ b1,
                                                       const float* __restrict__ w2, const int* __restrict__ n_rows_p,
                                                       float* __restrict__ part, int max_rows) {
  extern __shared__ float contrib[];   // [8][max_rows]
  const int n_rows = *n_rows_p;
  const int lane = threadIdx.x & 63, w = wave_index();
  if (d_hidden == 0) {
    for (int m = w; m < n_rows; m += 8) {
      float acc = 0.f;
      for (int k = lane; k < d; k += 64) acc += w2[k] * hf[(size_t)m * d + k];
      acc = wave_sum(acc);
      if (lane == 0) part[m] = acc;
    }
    return;
  }
  // one hidden unit per wave: its weight row stays in registers (2048 columns at a time), the rows of the
  // batch go four at a time so that their loads and reductions overlap
  const int j = blockIdx.x * 8 + w;
  const bool unit = j < d_hidden;
  const float bj = unit ? b1[j] : 0.f, w2j = unit ? w2[j] : 0.f;
  for (int m0 = 0; m0 < n_rows; m0 += 4) {
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int kc = 0; kc < d; kc += 2048) {
      float wreg[32];
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        const int k = kc + lane + 64 * i;
        wreg[i] = (unit && k < d) ? w1[(size_t)j * d + k] : 0.f;
      }
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        const int k = min(kc + lane + 64 * i, d - 1);
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[r] += wreg[i] * hf[(size_t)min(m0 + r, n_rows - 1) * d + k];
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float t = wave_sum(acc[r]) + bj;
      if (lane == 0 && m0 + r < n_rows) contrib[w * max_rows + m0 + r] = unit ? fmaxf(t, 0.f) * w2j : 0.f;
    }
  }
  __syncthreads();
  for (int m = threadIdx.x; m < n_rows; m += 512) {
    float sacc = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) sacc += contrib[q * max_rows + m];
    part[(size_t)blockIdx.x * max_rows + m] = sacc;
  }
}
int verifier_num_chunks(int d_hidden) { return d_hidden > 0 ? (d_hidden + 7) / 8 : 1; }
void launch_verifier_part(const float* hf, int d, int d_hidden, const float* w1, const float* b1, const float* w2,
                          const int* n_rows, float* part, int max_rows, hipStream_t s) {
  int chunks = verifier_num_chunks(d_hidden);
  hipLaunchKernelGGL(k_verifier_part, dim3(chunks), dim3(512), (size_t)8 * max_rows * sizeof(float), s, hf, d,
                     d_hidden, w1, b1, w2, n_rows, part, max_rows);
}

// ====================================== decide: arg-max merge, threshold, compaction
__device__ __forceinline__ u64 merge_partials(const u64* part, int n_wg, int Mpad, int m, int lane) {
  u64 k = 0;
  for (int i = lane; i < n_wg; i += 64) k = umax64(k, part[(size_t)i * Mpad + m]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) k = umax64(k, shfl_xor_u64(k, o));
  return k;
}

// Single workgroup of 1024 threads (B <= 1024).  accept <=> sigmoid(logit) >= tau in float32.
// Rejected rows are listed in ascending order: ballot + popcount inside each wave,
// wave totals prefix-summed through LDS.
__global__ __launch_bounds__(1024) void k_draft_decide(DecideArgs a) {
  __shared__ int s_tok[1024];
  __shared__ int s_wave_cnt[16];
  __shared__ int s_rej[1024];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int B = a.B;
  for (int m = w; m < B; m += 16) {
    u64 k = merge_partials(a.am_part, a.n_lm_wg, a.Mpad, m, lane);
    if (lane == 0) s_tok[m] = key_index(k);
  }
  __syncthreads();
  bool active = tid < B;
  float score = 0.f;
  bool acc = true;
  if (active) {
    float z = a.b2[0];
    for (int c = 0; c < a.n_chunks; ++c) z += a.ver_part[(size_t)c * B + tid];
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
// Rows whose prompt still has a token at index j (other than its last one).
__global__ __launch_bounds__(1024) void k_prefill_prep(const int* __restrict__ prompt, int max_prompt, int j, int B,
                                                       const int* __restrict__ prompt_len, int* n_rows, int* rb,
                                                       int* rtok, int* rpos, int* rslot) {
  __shared__ int s_wave_cnt[16];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const bool on = tid < B && j < prompt_len[tid] - 1;
  const u64 mask = __ballot(on);
  const int rank = __popcll(mask & ((1ull << lane) - 1ull));
  if (lane == 0) s_wave_cnt[w] = __popcll(mask);
  __syncthreads();
  int off = 0, total = 0;
  for (int q = 0; q < 16; ++q) {
    int c = s_wave_cnt[q];
    if (q < w) off += c;
    total += c;
  }
  if (on) {
    int i = off + rank;
    rb[i] = tid;
    rtok[i] = prompt[(size_t)tid * max_prompt + j];
    rpos[i] = j;
    rslot[i] = j;
  }
  if (tid == 0) *n_rows = total;
}
void launch_prefill_prep(const int* prompt, int max_prompt, int j, int B, const int* prompt_len, int* n_rows, int* rb,
                         int* rtok, int* rpos, int* rslot, hipStream_t s) {
  hipLaunchKernelGGL(k_prefill_prep, dim3(1), dim3(1024), 0, s, prompt, max_prompt, j, B, prompt_len, n_rows, rb,
                     rtok, rpos, rslot);
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
