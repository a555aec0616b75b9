// HIP kernels of the batched SPRINTER decode step for gfx950 (wave64, MFMA): weight packing, embedding
// and the layer norms.  One decode step (Alg. 2 of the paper, run for B rows in lock step):
//   draft forward -> LM head + Gumbel-max sample -> verifier + threshold ->
//   compaction of rejected rows -> target forward on those rows -> sample -> scatter back.
// Every kernel reads the number of active rows from device memory; the launch shapes are upper
// bounds the host chooses.
#include "dev.h"
#include <algorithm>
#include <cstring>

namespace sprinter {

// ================================================================ packing
// [N, K] row-major bf16 -> operand tiles of float16 (zero padded to 16 rows x 32 k).  A bf16 value has 8 significant
// bits and converts exactly above 2^-14; smaller ones round to the float16 subnormal grid (2^-24 apart).
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
  const unsigned wd[4] = {v.x, v.y, v.z, v.w};
  unsigned o[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = pk_f16(__uint_as_float(wd[e] << 16), __uint_as_float(wd[e] & 0xffff0000u));
  out[i] = make_uint4(o[0], o[1], o[2], o[3]);
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
                                              float* __restrict__ f32_out) {
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
      act_store<AT>(act_out, r, k, d, o);
      if (f32_out) f32_out[(size_t)r * d + k] = o;
    }
  }
}
// bf16 output: one row per workgroup, one thread per 8 consecutive columns (= one 16-byte slot of an
// operand tile), so the row, gain and offset are requested with six 16-byte loads per thread
// before anything is waited for and the result leaves as one 16-byte store of float16.  d <= 8192.
// NI = 2048-column blocks per row (1, 2 or 4); SH = 0, or the most partial products a pending update of the
// residual stream may consist of (4 or 8): the row is then h + bias + share 0 + share 1 + ..., added in that
// order, written back and normalised.  The partial loads are issued with the others, before the row count
// is known, with clamped share indices and the surplus selected away - no branch, no second memory round.
template <int ARCH, int NI, int SH>
__global__ __launch_bounds__(256) void k_norm_bf16(const float* __restrict__ h, const float* __restrict__ g,
                                                   const float* __restrict__ b, float eps, int d,
                                                   const int* __restrict__ n_rows, bf16_t* __restrict__ act_out,
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
      const uint4 ov = make_uint4(pk_f16(o[0], o[1]), pk_f16(o[2], o[3]), pk_f16(o[4], o[5]), pk_f16(o[6], o[7]));
      const int k = c * 8;
      const size_t slot = ((size_t)(r >> 4) * Kt + (k >> 5)) * 512 + ((((k & 31) >> 3) << 4) + (r & 15)) * 8;
      *reinterpret_cast<uint4*>(act_out + slot) = ov;
      if (f32_out) {
        *reinterpret_cast<float4*>(f32_out + (size_t)r * d + k) = make_float4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<float4*>(f32_out + (size_t)r * d + k + 4) = make_float4(o[4], o[5], o[6], o[7]);
      }
    }
  }
}

template <int ARCH, int NI>
static void launch_norm_bf16(const float* h, const float* g, const float* b, float eps, int d, const int* n_rows,
                             bf16_t* act_out, float* f32_out, int max_rows, hipStream_t s, const NormPending& np) {
#define SPRINTER_NORM(SH) hipLaunchKernelGGL((k_norm_bf16<ARCH, NI, SH>), dim3(max_rows), dim3(256), 0, s, h, g, b, eps, d, n_rows, act_out, f32_out, np)
  if (np.shares <= 0) SPRINTER_NORM(0);
  else if (np.shares <= 4) SPRINTER_NORM(4);
  else SPRINTER_NORM(8);
#undef SPRINTER_NORM
}

void launch_norm(int dtype, int arch, const float* h, const float* g, const float* b, float eps, int d,
                 const int* n_rows, void* act_out, float* f32_out, int max_rows, hipStream_t s,
                 const NormPending* pend) {
  NormPending np;
  memset(&np, 0, sizeof np);
  if (pend) np = *pend;
#define NORM_CASE(AT, ARCH) \
  hipLaunchKernelGGL((k_norm<AT, ARCH>), dim3(max_rows), dim3(256), 0, s, h, g, b, eps, d, n_rows, (AT*)act_out, f32_out)
  if (dtype == 0) { if (arch == 0) NORM_CASE(float, 0); else NORM_CASE(float, 1); }
  else if (d % 8 == 0 && d <= 8192) {
    bf16_t* out = (bf16_t*)act_out;
    if (arch == 0) {
      if (d <= 2048) launch_norm_bf16<0, 1>(h, g, b, eps, d, n_rows, out, f32_out, max_rows, s, np);
      else if (d <= 4096) launch_norm_bf16<0, 2>(h, g, b, eps, d, n_rows, out, f32_out, max_rows, s, np);
      else launch_norm_bf16<0, 4>(h, g, b, eps, d, n_rows, out, f32_out, max_rows, s, np);
    } else {
      if (d <= 2048) launch_norm_bf16<1, 1>(h, g, b, eps, d, n_rows, out, f32_out, max_rows, s, np);
      else if (d <= 4096) launch_norm_bf16<1, 2>(h, g, b, eps, d, n_rows, out, f32_out, max_rows, s, np);
      else launch_norm_bf16<1, 4>(h, g, b, eps, d, n_rows, out, f32_out, max_rows, s, np);
    }
  }
  else            { if (arch == 0) NORM_CASE(bf16_t, 0); else NORM_CASE(bf16_t, 1); }
#undef NORM_CASE
}

}  // namespace sprinter
