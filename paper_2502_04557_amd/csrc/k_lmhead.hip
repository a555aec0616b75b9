// HIP kernels of the batched SPRINTER decode step for gfx950: LM head fused with sampling (Alg. 2: x ~ q_r,
// and the target's draw), and the verifier's hidden layer (Sec. 3.2).
#include "dev.h"
#include <algorithm>
#include <cstring>

namespace sprinter {

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
// Hidden layer of the verifier MLP, spread over workgroups of 8 waves (VU hidden
// units per wave); each workgroup leaves its share of the output logit per row.
// d_hidden == 0: the logit is w2 . hf (a single chunk).
constexpr int VU = 4;
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
  // VU hidden units per wave: their weight rows stay in registers (2048 columns at a time), the rows of the batch
  // go four at a time so that their loads and reductions overlap.  Every wave reads the whole hidden-state matrix
  // (from L2), so the units per wave set that traffic: with one unit per wave 512 waves re-read 0.5 MB each at
  // d = 2048 and 64 rows (81 us); with four it is a quarter of that.
  const int j0 = (blockIdx.x * 8 + w) * VU;
  float bj[VU], w2j[VU];
#pragma unroll
  for (int u = 0; u < VU; ++u) {
    const bool unit = j0 + u < d_hidden;
    bj[u] = unit ? b1[j0 + u] : 0.f;
    w2j[u] = unit ? w2[j0 + u] : 0.f;              // (a unit beyond the layer contributes relu(0) * 0)
  }
  for (int m0 = 0; m0 < n_rows; m0 += 4) {
    float acc[VU][4];
#pragma unroll
    for (int u = 0; u < VU; ++u)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[u][r] = 0.f;
    for (int kc = 0; kc < d; kc += 2048) {
      float wreg[VU][32];
#pragma unroll
      for (int u = 0; u < VU; ++u)
#pragma unroll
        for (int i = 0; i < 32; ++i) {
          const int k = kc + lane + 64 * i;
          wreg[u][i] = (j0 + u < d_hidden && k < d) ? w1[(size_t)(j0 + u) * d + k] : 0.f;
        }
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        const int k = min(kc + lane + 64 * i, d - 1);
        float h[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) h[r] = hf[(size_t)min(m0 + r, n_rows - 1) * d + k];
#pragma unroll
        for (int u = 0; u < VU; ++u)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[u][r] += wreg[u][i] * h[r];
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float t = 0.f;
#pragma unroll
      for (int u = 0; u < VU; ++u) t += fmaxf(wave_sum(acc[u][r]) + bj[u], 0.f) * w2j[u];
      if (lane == 0 && m0 + r < n_rows) contrib[w * max_rows + m0 + r] = t;
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
int verifier_num_chunks(int d_hidden) { return d_hidden > 0 ? (d_hidden + 8 * VU - 1) / (8 * VU) : 1; }
void launch_verifier_part(const float* hf, int d, int d_hidden, const float* w1, const float* b1, const float* w2,
                          const int* n_rows, float* part, int max_rows, hipStream_t s) {
  int chunks = verifier_num_chunks(d_hidden);
  hipLaunchKernelGGL(k_verifier_part, dim3(chunks), dim3(512), (size_t)8 * max_rows * sizeof(float), s, hf, d,
                     d_hidden, w1, b1, w2, n_rows, part, max_rows);
}

}  // namespace sprinter
