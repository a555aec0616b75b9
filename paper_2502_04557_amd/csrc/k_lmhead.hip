// HIP kernels of the batched SPRINTER decode step for gfx950: LM head fused with sampling (Alg. 2: x ~ q_r,
// and the target's draw), and the verifier's hidden layer (Sec. 3.2).
#include "dev.h"
#include <algorithm>
#include <cstring>

namespace sprinter {

// ======================================================= LM head + sample
struct LmArgs {
  const void* W; const void* X; RowDesc rd; int V, K, Kt, n_tiles;
  SamplerArgs sa; u64* part; int Mpad; float* logits_out; size_t x_elems; int m_tiles;
  int rows_live;   // the host's bound on the row count: lanes of rows from here on skip their activation loads
};

// bf16, at most 16 rows (launched with MT = 1): each workgroup owns a contiguous range of column tiles; its 8 waves
// take pairs of adjacent tiles round-robin (the two tiles share the activation fragments), keep a running
// (value, index) maximum per row, and the workgroup writes one partial per row.  The k loop has no branches: two
// register buffers, tiles and k tiles beyond the end are clamped on load; columns beyond the vocabulary and rows
// beyond the row count are dropped when the logits are sampled.
template <int MT>
__global__ __launch_bounds__(512) void k_lmhead_bf16(LmArgs a) {
  __shared__ u64 sbest[8][MT * 16];
  __shared__ int s_rb[MT * 16], s_rt[MT * 16];
  const int lane = threadIdx.x & 63, w = wave_index();
  const int tpw = (a.n_tiles + gridDim.x - 1) / gridDim.x;
  const int t0 = blockIdx.x * tpw, t1 = min(t0 + tpw, a.n_tiles);
  const uint4* __restrict__ Wp = (const uint4*)a.W + lane;
  const uint4* __restrict__ Xp = (const uint4*)a.X + lane;
  const int Kt = a.Kt;
  const int n_rows = *a.rd.n_rows;
  constexpr int U = 2;                                    // k tiles per register buffer
  struct Buf { uint4 w[U][2], xh[U][MT]; };
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
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int kc = min(kt + u, Kt - 1);
          b.w[u][0] = Wp[wrow0 + (size_t)kc * 64];
          b.w[u][1] = Wp[wrow1 + (size_t)kc * 64];
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {                 // (a lane holds 8 k of one row: rows that exist in no launch are not fetched,
          if (m0 + mt * 16 + (lane & 15) < a.rows_live) { //  what the registers hold for them only reaches logits that are dropped)
#pragma unroll
            for (int u = 0; u < U; ++u) b.xh[u][mt] = Xp[((size_t)(mtile0 + mt) * Kt + min(kt + u, Kt - 1)) * 64];
          }
        }
      };
      f32x4 acc[2][MT];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[j][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      auto compute = [&](const Buf& b, int kt) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const bool in_k = kt + u < Kt;
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            const uint4 wj = in_k ? b.w[u][j] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[j][mt] = mfma_f16(b.xh[u][mt], wj, acc[j][mt]);
          }
        }
      };
      Buf A, B;
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) A.xh[u][mt] = B.xh[u][mt] = make_uint4(0u, 0u, 0u, 0u);
      load(A, 0);
      for (int kt = 0; kt < Kt; kt += 2 * U) {
        load(B, kt + U);
        __builtin_amdgcn_sched_barrier(0);
        compute(A, kt);
        __builtin_amdgcn_sched_barrier(0);
        load(A, kt + 2 * U);
        __builtin_amdgcn_sched_barrier(0);
        compute(B, kt + U);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = (nt + j) * 16 + (lane & 15);
        const bool col = nt + j < t1 && n < a.V;             // (no branches below: the quad exchange needs every lane)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          if (a.logits_out) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const int m = m0 + mt * 16 + (lane >> 4) * 4 + v;
              if (col && m < n_rows) a.logits_out[(size_t)m * a.V + n] = acc[j][mt][v];
            }
          }
          const int mq = mt * 16 + (lane >> 4) * 4 + (lane & 3);   // the row whose random block this lane computes for its quad
          u64 kj[4];
          sample_keys_quad(acc[j][mt], a.sa, s_rb[mq], s_rt[mq], n, kj);
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int m = m0 + mt * 16 + (lane >> 4) * 4 + v;
            best[mt][v] = umax64(best[mt][v], col && m < n_rows ? kj[v] : 0);
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

// bf16, 17+ rows: the 8 waves of a workgroup take different column tiles (NTW each, 8 NTW tiles per round over the
// workgroup's tile range) and share the activations of MT row tiles through LDS, so a k tile costs the workgroup
// MT KiB of activations once instead of once per wave - at 64 rows per-wave reads would pull three times the
// weight bytes through L2.  KS k tiles per stage, two LDS stages: the loads of stage c + 1 (the wave's weight tiles
// and its share of the activation fragments, into registers) are in flight while the MFMAs of stage c run; one
// barrier per stage.  NTW = 2 where the workgroup's range has more than 8 tiles (large vocabularies), else 1 so
// that every wave has a tile.  Fragment f of a stage = (k tile f / MT, row tile f % MT); wave w
// stages fragments w, w + 8, ...  Tiles and k tiles beyond the end are clamped on load and dropped afterwards; row
// tiles are clamped to the m_tiles the activation buffer holds.  More than 16 MT rows take further passes.
template <int MT, int NTW, int KS>
__global__ __launch_bounds__(512, MT <= 4 ? 4 : 2) void k_lmhead_wide(LmArgs a) {
  constexpr int NF = KS * MT, F = (NF + 7) / 8;             // fragments per stage, per wave (with fewer than 8 the last waves stage none)
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  __shared__ u32x4 xs[2][NF][64];
  __shared__ u64 sbest[8][MT * 16];
  __shared__ int s_rb[MT * 16], s_rt[MT * 16];
  const int lane = threadIdx.x & 63, w = wave_index();
  const int tpw = (a.n_tiles + gridDim.x - 1) / gridDim.x;
  const int t0 = blockIdx.x * tpw, t1 = min(t0 + tpw, a.n_tiles);
  const uint4* __restrict__ Wp = (const uint4*)a.W + lane;
  const int Kt = a.Kt;
  const int n_rows = *a.rd.n_rows;
  struct Regs { u32x4 x[F]; uint4 w[KS][NTW]; };
  for (int m0 = 0; m0 < n_rows; m0 += MT * 16) {
    const int mtile0 = m0 >> 4;
    // running maximum per row: accumulator (row tile mt, register v) of DPP row lq is row mt * 16 + lq * 4 + v; after
    // each round its 16 lanes (columns) are merged and lane l16 = (mt * 4 + v) % 16 keeps the result in slot
    // (mt * 4 + v) / 16 - one or two keys per lane instead of 4 MT
    constexpr int NB = (MT * 4 + 15) / 16;
    u64 best[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) best[q] = 0;
    for (int i = threadIdx.x; i < MT * 16; i += 512) {     // the rows' random streams: batch row, position being generated
      s_rb[i] = m0 + i < n_rows ? a.rd.b[m0 + i] : 0;
      s_rt[i] = m0 + i < n_rows ? a.rd.pos[m0 + i] + 1 : 0;
    }
    const u32x4* xsrc[F];                                    // this wave's fragments of a stage, at k tile 0
    int xu[F];
    bool xlive[F];                                           // (a lane stages 8 k of one row: rows that exist in no launch are not fetched)
#pragma unroll
    for (int i = 0; i < F; ++i) {
      const int f = w + 8 * i, mt = f % MT;
      xu[i] = f / MT;
      xlive[i] = f < NF && m0 + mt * 16 + (lane & 15) < a.rows_live;
      xsrc[i] = (const u32x4*)a.X + (size_t)min(mtile0 + mt, a.m_tiles - 1) * Kt * 64 + lane;
    }
    for (int c0 = t0; c0 < t1; c0 += 8 * NTW) {
      const int nt = c0 + NTW * w;
      size_t wrow[NTW];
#pragma unroll
      for (int j = 0; j < NTW; ++j) wrow[j] = (size_t)min(nt + j, t1 - 1) * Kt * 64;
      auto gload = [&](Regs& r, int kt) {
#pragma unroll
        for (int u = 0; u < KS; ++u) {
          const int kc = min(kt + u, Kt - 1);
#pragma unroll
          for (int j = 0; j < NTW; ++j) r.w[u][j] = Wp[wrow[j] + (size_t)kc * 64];
        }
#pragma unroll
        for (int i = 0; i < F; ++i)
          if (xlive[i]) r.x[i] = xsrc[i][(size_t)min(kt + xu[i], Kt - 1) * 64];
      };
      auto sstore = [&](int stage, const Regs& r) {
#pragma unroll
        for (int i = 0; i < F; ++i)
          if (w + 8 * i < NF) xs[stage][w + 8 * i][lane] = r.x[i];
      };
      f32x4 acc[NTW][MT];
#pragma unroll
      for (int j = 0; j < NTW; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[j][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      auto compute = [&](int stage, const Regs& r, int kt) {
#pragma unroll
        for (int u = 0; u < KS; ++u) {
          const bool in_k = kt + u < Kt;
          uint4 wv[NTW];
#pragma unroll
          for (int j = 0; j < NTW; ++j) wv[j] = in_k ? r.w[u][j] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const u32x4 h = xs[stage][u * MT + mt][lane];
            const uint4 xh = make_uint4(h.x, h.y, h.z, h.w);
#pragma unroll
            for (int j = 0; j < NTW; ++j) {
              acc[j][mt] = mfma_f16(xh, wv[j], acc[j][mt]);
            }
          }
        }
      };
      Regs A, B;
#pragma unroll
      for (int i = 0; i < F; ++i) A.x[i] = B.x[i] = (u32x4){0u, 0u, 0u, 0u};
      gload(A, 0);
      sstore(0, A);                                          // (nobody reads stage 0 any more: the last barrier of the previous round)
      __syncthreads();                                       // also orders s_rb / s_rt before the sampling below
      for (int kt = 0; kt < Kt; kt += 2 * KS) {
        gload(B, kt + KS);
        __builtin_amdgcn_sched_barrier(0);
        compute(0, A, kt);
        sstore(1, B);
        __syncthreads();
        gload(A, kt + 2 * KS);
        __builtin_amdgcn_sched_barrier(0);
        compute(1, B, kt + KS);
        sstore(0, A);
        __syncthreads();
      }
      const int n0 = nt * 16 + (lane & 15);                  // tile j's column: n0 + 16 j
      bool col[NTW];
#pragma unroll
      for (int j = 0; j < NTW; ++j) col[j] = nt + j < t1 && n0 + 16 * j < a.V;
      if (a.logits_out) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int m = m0 + mt * 16 + (lane >> 4) * 4 + v;
#pragma unroll
            for (int j = 0; j < NTW; ++j)
              if (m < n_rows && col[j]) a.logits_out[(size_t)m * a.V + n0 + 16 * j] = acc[j][mt][v];
          }
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int mq = mt * 16 + (lane >> 4) * 4 + (lane & 3);   // the row whose random block this lane computes for its quad
        const int rb = s_rb[mq], rt = s_rt[mq];
        u64 kv[4] = {0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < NTW; ++j) {
          u64 kj[4];
          sample_keys_quad(acc[j][mt], a.sa, rb, rt, n0 + 16 * j, kj);
#pragma unroll
          for (int v = 0; v < 4; ++v) kv[v] = umax64(kv[v], col[j] ? kj[v] : 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int mi = mt * 16 + (lane >> 4) * 4 + v, idx = mt * 4 + v;
          const u64 k = group_umax64_16(m0 + mi < n_rows ? kv[v] : 0);
          if ((lane & 15) == (idx & 15)) best[idx >> 4] = umax64(best[idx >> 4], k);
        }
        __builtin_amdgcn_sched_barrier(0);                   // one row tile's random streams at a time (registers)
      }
    }
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      const int idx = q * 16 + (lane & 15);                  // (row tile, register) this lane kept
      if (idx < MT * 4) sbest[w][(idx >> 2) * 16 + (lane >> 4) * 4 + (idx & 3)] = best[q];
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

void launch_lmhead(int dtype, const void* W, const void* X, size_t x_elems, const RowDesc& rd, int V, int K,
                   const SamplerArgs& sa, unsigned long long* part, int n_wg, int Mpad, float* logits_out, int max_rows,
                   hipStream_t s) {
  LmArgs a;
  a.x_elems = x_elems;
  a.W = W; a.X = X; a.rd = rd; a.V = V; a.K = K; a.Kt = (K + 31) / 32; a.n_tiles = (V + 15) / 16;
  a.sa = sa; a.part = part; a.Mpad = Mpad; a.logits_out = logits_out; a.m_tiles = 0; a.rows_live = max_rows;
  if (dtype == 0) {
    hipLaunchKernelGGL(k_lmhead_f32, dim3(n_wg), dim3(256), 0, s, a);
  } else if (max_rows <= 16) {
    hipLaunchKernelGGL(k_lmhead_bf16<1>, dim3(n_wg), dim3(512), 0, s, a);
  } else {
    a.m_tiles = (int)(x_elems / ((size_t)a.Kt * 512));      // row tiles the activation buffer holds
    const int tpw = (a.n_tiles + n_wg - 1) / n_wg;           // tiles per workgroup
#define SPRINTER_LM(MT, KS1, KS2)                                                                       \
  do {                                                                                                  \
    if (tpw <= 8) hipLaunchKernelGGL((k_lmhead_wide<MT, 1, KS1>), dim3(n_wg), dim3(512), 0, s, a);      \
    else hipLaunchKernelGGL((k_lmhead_wide<MT, 2, KS2>), dim3(n_wg), dim3(512), 0, s, a);               \
  } while (0)
    if (max_rows <= 32) SPRINTER_LM(2, 2, 2);
    else if (max_rows <= 64) SPRINTER_LM(4, 2, 2);
    else SPRINTER_LM(8, 2, 1);                               // more than 128 rows: further passes inside the kernel
#undef SPRINTER_LM
  }
}

// =============================================================== verifier
// Hidden layer of the verifier MLP (Sec. 3.2; the paper's single linear layer when d_hidden == 0) in float32.
// With a hidden layer it is a small matrix product, hidden = relu(hf W1^T + b1), done on the float32 matrix
// pipes: a workgroup owns 16 rows x 16 hidden units, its 8 waves split K; lane (l16, lq) holds four consecutive k of
// row l16 and of unit l16 per 16-byte load, and the four 16x16x4 products of a load take k = 4 lq + 0 .. 3 (any
// assignment of k to products is a valid order of the sum as long as both operands use the same one).  The waves'
// accumulators are added in fixed order through LDS, then relu(. + b1) * w2 is summed over the 16 units and the
// workgroup leaves its share of each row's output logit in part[chunk][row]; the consumer adds the chunks in order.
// (One wave per hidden unit re-read the whole hidden-state matrix per wave - 268 MB through L2 at d = 2048,
// 512 units and 64 rows, 81 us; this form reads 32 MB.)
__global__ __launch_bounds__(512) void k_verifier_part(const float* __restrict__ hf, int d, int d_hidden,
                                                       const float* __restrict__ w1, const float* __restrict__ b1,
                                                       const float* __restrict__ w2, const int* __restrict__ n_rows_p,
                                                       float* __restrict__ part, int max_rows) {
  __shared__ float red[8][4][64];
  const int n_rows = *n_rows_p;
  const int lane = threadIdx.x & 63, w = wave_index();
  if (d_hidden == 0) {                               // (one workgroup)
    for (int m = w; m < n_rows; m += 8) {
      float acc = 0.f;
      for (int k = lane; k < d; k += 64) acc += w2[k] * hf[(size_t)m * d + k];
      acc = wave_sum(acc);
      if (lane == 0) part[m] = acc;
    }
    return;
  }
  const int m0 = blockIdx.y * 16;
  if (m0 >= n_rows) return;
  const int l16 = lane & 15, lq = lane >> 4, j = blockIdx.x * 16 + l16;
  // rows beyond the row count and units beyond the layer are read at the last valid one and dropped below
  const float4* __restrict__ hrow = reinterpret_cast<const float4*>(hf + (size_t)min(m0 + l16, n_rows - 1) * d) + lq;
  const float4* __restrict__ wrow = reinterpret_cast<const float4*>(w1 + (size_t)min(j, d_hidden - 1) * d) + lq;
  const int n16 = d >> 4, g0 = n16 * w / 8, g1 = n16 * (w + 1) / 8;   // this wave's groups of 16 k (d is a multiple of 16)
  f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
  for (int g = g0; g < g1; g += 8) {
    float4 av[8], bv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int gi = min(g + i, g1 - 1);
      av[i] = hrow[gi * 4];
      bv[i] = wrow[gi * 4];
    }
    __builtin_amdgcn_sched_barrier(0);               // all sixteen loads go out before the first product waits
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool on = g + i < g1;                    // (scalar) a group beyond the share contributes zeros
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i].x, on ? bv[i].x : 0.f, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i].y, on ? bv[i].y : 0.f, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i].z, on ? bv[i].z : 0.f, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i].w, on ? bv[i].w : 0.f, acc, 0, 0, 0);
    }
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) red[w][v][lane] = acc[v];
  __syncthreads();
  if (w < 4) {                                       // wave v finishes accumulator register v: row m0 + lq * 4 + v, unit j
    float sum = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) sum += red[q][w][lane];
    const bool unit = j < d_hidden;
    const float t = unit ? fmaxf(sum + b1[min(j, d_hidden - 1)], 0.f) * w2[min(j, d_hidden - 1)] : 0.f;
    const float tot = group_sum<16>(t);
    const int m = m0 + lq * 4 + w;
    if (l16 == 0 && m < n_rows) part[(size_t)blockIdx.x * max_rows + m] = tot;
  }
}
int verifier_num_chunks(int d_hidden) { return d_hidden > 0 ? (d_hidden + 15) / 16 : 1; }
void launch_verifier_part(const float* hf, int d, int d_hidden, const float* w1, const float* b1, const float* w2,
                          const int* n_rows, float* part, int max_rows, hipStream_t s) {
  const dim3 grid = d_hidden > 0 ? dim3(verifier_num_chunks(d_hidden), (max_rows + 15) / 16) : dim3(1);
  hipLaunchKernelGGL(k_verifier_part, grid, dim3(512), 0, s, hf, d, d_hidden, w1, b1, w2, n_rows, part, max_rows);
}

}  // namespace sprinter
