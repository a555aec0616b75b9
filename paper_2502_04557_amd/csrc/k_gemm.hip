// HIP kernels of the batched SPRINTER decode step for gfx950: the projection / FFN GEMMs
// (Alg. 2: the draft's and the target's forward passes).
#include "dev.h"
#include <algorithm>
#include <cstring>

namespace sprinter {

// =================================================================== GEMM
struct GemmArgs {
  const void* W; const void* W2; const void* X; const int* n_rows;
  int N, K, Kt, n_tiles;
  const float* bias; float* out_f32; int ldo; void* out_act; int out_K;
  size_t x_elems;     // elements the activation buffer X holds (bf16 mode)
  int SK; float* part; size_t part_stride;   // k_gemm16_part: K shares, partial outputs [SK][rows][N], floats per share
  int rows_live;      // the host's bound on the row count: rows from here on exist in no launch, their activations are not fetched
};

// bias: the column's bias (0 if none); res: the current value of the output element (residual epilogue only)
template <int EPI, typename AT>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& a, int n_rows, int m, int n, float v, float v2, float bias, float res) {
  if (m >= n_rows || n >= a.N) return;
  if (EPI == EPI_F32) a.out_f32[(size_t)m * a.ldo + n] = v + bias;
  else if (EPI == EPI_RESID) a.out_f32[(size_t)m * a.ldo + n] = res + (v + bias);
  else if (EPI == EPI_GELU) act_store<AT>((AT*)a.out_act, m, n, a.out_K, gelu_tanh(v + bias));
  else act_store<AT>((AT*)a.out_act, m, n, a.out_K, silu(v) * v2);
}


// bf16-mode GEMM (float16 operands) on MFMA for at most 16 rows.  512 threads = 8 waves that split K; each wave owns NTW column tiles
// (16 columns each): D[m][n] += X[m][k] W[n][k].
// All 8 waves leave their partial sums in LDS and every thread then finishes ONE output element: it adds the 8
// partials in fixed order, applies bias / residual / GELU / SwiGLU and stores.  With the element order chosen per
// output layout the 256 x NTW stores of the workgroup are contiguous: one 32-column operand tile for
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
  // A lane holds 8 k of row lane % 16: lanes of rows the host knows not to exist skip their loads (a step with 3
  // rejected rows then pulls 3/16 of the activation bytes through the compute unit's memory pipeline, which carries
  // them next to the weight stream); what their registers hold only reaches output rows that are dropped.
  const bool row_live = (lane & 15) < a.rows_live;
  uint4 xv[U];
#pragma unroll
  for (int u = 0; u < U; ++u) xv[u] = make_uint4(0u, 0u, 0u, 0u);
  auto load_x = [&](int kt) {                               // no dependence on the (device-side) row count
    if (row_live) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int kc = min(kt + u * 8, Kt - 1);
        xv[u] = Xp[(size_t)kc * 64 + lane];
      }
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
      const uint4 ah = in_k ? xv[u] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
      for (int j = 0; j < NTW; ++j) {
        acc[j] = mfma_f16(ah, wv[u][j], acc[j]);
        if (DUAL) {
          acc2[j] = mfma_f16(ah, wv2[u][j], acc2[j]);
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

// bf16-mode GEMM for 17 .. 64 rows per pass (MT row tiles of 16), one column tile per workgroup, K split over
// the 8 waves.  At these row counts a workgroup pulls the whole activation matrix (MT x 1 KiB per k tile,
// from L2) for 1 KiB of weights per k tile, so the kernel lives on memory-level parallelism: two register
// buffers, the loads of chunk c + 1 (weights and all MT row tiles) are in flight while the
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
  size_t wrow[NTW];
#pragma unroll
  for (int j = 0; j < NTW; ++j) wrow[j] = (size_t)min(nt0 + j, a.n_tiles - 1) * Kt * 64;
  struct Buf { uint4 w[U][NWT], xh[U][MT]; };
  // (as in k_gemm16: a lane whose row exists in no launch - the host's bound - skips its activation loads; with 18
  // rows the second row tile costs an eighth of its bytes)
  bool row_live[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) row_live[mt] = (mtile0 + mt) * 16 + (lane & 15) < a.rows_live;
  auto load = [&](Buf& b, int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kc = min(kt + u * 8, k1 - 1);
#pragma unroll
      for (int j = 0; j < NTW; ++j) {
        b.w[u][j] = Wp[wrow[j] + (size_t)kc * 64];
        if (DUAL) b.w[u][NTW + j] = W2p[wrow[j] + (size_t)kc * 64];
      }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      if (row_live[mt]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int kc = min(kt + u * 8, k1 - 1);
          b.xh[u][mt] = Xp[((size_t)mt * Kt + kc) * 64];
        }
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
          acc[j][mt] = mfma_f16(b.xh[u][mt], w1, acc[j][mt]);
        }
      }
    }
  };
  Buf A, B;
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) A.xh[u][mt] = B.xh[u][mt] = make_uint4(0u, 0u, 0u, 0u);
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

// bf16-mode GEMM for 128+ rows (prefill chunks, long work lists): the 8 waves of a workgroup split the COLUMNS (NTW
// column tiles each; SwiGLU: one gate + one up tile) and share the activations of 8 row tiles (128 rows) through LDS,
// so a k tile costs the workgroup 8 KiB of activations (once) + 8 * NWT KiB of weights for
// 8 * NWT * 8 MFMAs - far fewer bytes per MFMA than the K-split kernel above, which reads every operand per wave.
// Two k tiles per stage (one with four weight tiles per wave), two LDS stages: the global loads of stage c + 1 (the activation fragments a thread stages, into
// registers, and the wave's own weight tiles) are in flight while the MFMAs of stage c run; one barrier per stage.
// blockIdx.y = group of 128 rows, blockIdx.z = K share (EPI_PART).  The activation buffer must hold every row
// tile the grid covers (the launcher checks it against the buffer's size).
template <int NTW, int EPI>
__global__ __launch_bounds__(512) void k_gemm_wide(GemmArgs a) {
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int NWT = NTW * (DUAL ? 2 : 1), MT = 8;
  constexpr int KU = NWT >= 4 ? 1 : 2;                 // k tiles per stage (four weight tiles per wave leave registers for one)
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  __shared__ u32x4 xs[2][KU][MT][64];                   // [stage][k tile][row tile][lane]: 16 KiB per k tile of a stage
  const int lane = threadIdx.x & 63, w = wave_index();
  const int Kt = a.Kt, mtile0 = blockIdx.y * MT, nt0 = (blockIdx.x * 8 + w) * NTW;
  const int sk = (EPI == EPI_PART) ? blockIdx.z : 0, SK = (EPI == EPI_PART) ? gridDim.z : 1;
  const int k0 = (int)((long long)Kt * sk / SK), k1 = (int)((long long)Kt * (sk + 1) / SK);
  const uint4* __restrict__ Wp = (const uint4*)a.W + lane;
  const uint4* __restrict__ W2p = DUAL ? (const uint4*)a.W2 + lane : nullptr;
  // staging: wave w fetches row tile w of every k tile of the stage
  const u32x4* __restrict__ Xh = (const u32x4*)a.X + (size_t)(mtile0 + w) * Kt * 64 + lane;
  size_t wrow[NTW];
#pragma unroll
  for (int j = 0; j < NTW; ++j) wrow[j] = (size_t)min(nt0 + j, a.n_tiles - 1) * Kt * 64;
  struct Regs { u32x4 x[KU]; uint4 w[KU][NWT]; };
  auto gload = [&](Regs& r, int kt) {
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      const int kc = min(kt + u, k1 - 1);                // clamped: always a tile of this share
      r.x[u] = Xh[(size_t)kc * 64];
#pragma unroll
      for (int j = 0; j < NTW; ++j) {
        r.w[u][j] = Wp[wrow[j] + (size_t)kc * 64];
        if (DUAL) r.w[u][NTW + j] = W2p[wrow[j] + (size_t)kc * 64];
      }
    }
  };
  auto sstore = [&](int stage, const Regs& r) {
#pragma unroll
    for (int i = 0; i < KU; ++i) xs[stage][i][w][lane] = r.x[i];
  };
  f32x4 acc[NWT][MT];
#pragma unroll
  for (int j = 0; j < NWT; ++j)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[j][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
  auto compute = [&](int stage, const Regs& r, int kt) {
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      const bool in_k = kt + u < k1;
      uint4 wv[NWT];
#pragma unroll
      for (int j = 0; j < NWT; ++j) wv[j] = in_k ? r.w[u][j] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const u32x4 h = xs[stage][u][mt][lane];
        const uint4 xh = make_uint4(h.x, h.y, h.z, h.w);
#pragma unroll
        for (int j = 0; j < NWT; ++j) {
          acc[j][mt] = mfma_f16(xh, wv[j], acc[j][mt]);
        }
      }
    }
  };
  Regs A, B;
  gload(A, k0);
  sstore(0, A);
  const int n_rows = *a.n_rows;                          // only the epilogue needs it
  __syncthreads();
  for (int kt = k0; kt < k1; kt += 2 * KU) {
    gload(B, kt + KU);
    __builtin_amdgcn_sched_barrier(0);
    compute(0, A, kt);
    sstore(1, B);
    __syncthreads();
    gload(A, kt + 2 * KU);
    __builtin_amdgcn_sched_barrier(0);
    compute(1, B, kt + KU);
    sstore(0, A);
    __syncthreads();
  }
  // every wave stores its own 128 x 16 NTW block straight from the accumulators (lane l, register v: column l % 16,
  // row (l / 16) * 4 + v)
  float* part = (EPI == EPI_PART) ? a.part + (size_t)sk * a.part_stride : nullptr;
#pragma unroll
  for (int j = 0; j < NTW; ++j) {
    const int n = (nt0 + j) * 16 + (lane & 15);
    if (n >= a.N) continue;
    const float bias = (EPI != EPI_PART && a.bias) ? a.bias[n] : 0.f;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int m = (mtile0 + mt) * 16 + (lane >> 4) * 4 + v;
        if (m >= n_rows) continue;
        const float s1 = acc[j][mt][v], s2 = DUAL ? acc[NTW + j][mt][v] : 0.f;
        if constexpr (EPI == EPI_PART) {
          part[(size_t)m * a.ldo + n] = s1;
        } else {
          const float res = (EPI == EPI_RESID) ? a.out_f32[(size_t)m * a.ldo + n] : 0.f;
          gemm_epilogue<EPI, bf16_t>(a, n_rows, m, n, s1, s2, bias, res);
        }
      }
  }
}

// Launches k_gemm_wide if the row count calls for it and the activation buffer holds every row tile of the grid.
// min_rows: 128 for outputs that need the whole K in one workgroup; 97 for partial products, where K shares bring the
// workgroup count back up (c4's shapes at 100 rows: FFN-down 4096 x 11008 50.8 -> 42.2 us, O-proj 25.5 -> 18.3 us with one
// 128-row group, while FFN-up and QKV, left with 86 - 96 workgroups, lose: 95 -> 115 us and 56 -> 77 us; at 72 - 88 rows
// FFN-down loses too, 42 -> 46 us, against two passes of 3 row tiles).
template <int EPI>
static bool try_gemm_wide(const GemmArgs& a, int max_rows, int sk, hipStream_t s, int min_rows = 128) {
  if (max_rows < min_rows) return false;
  const int row_groups = (max_rows + 127) / 128;
  if ((size_t)row_groups * 128 * a.Kt * 32 > a.x_elems) return false;
  constexpr bool DUAL = EPI == EPI_SWIGLU;
  const int g2 = (a.n_tiles + 15) / 16, g1 = (a.n_tiles + 7) / 8;
  // too few workgroups for the chip (a 128-row decode batch on a narrow model: 18 column groups): the K-split
  // kernels, which put every column tile in a workgroup of its own, do better there
  if (g1 * row_groups * sk < 128) return false;
  // four weight tiles per wave (SwiGLU: two gate + two up) halve the LDS reads per MFMA, which at two tiles take as
  // long as the MFMAs themselves; two or one tile per wave where that would leave too few workgroups
  const int g4 = (a.n_tiles + 31) / 32;
  if constexpr (DUAL) {
    if (g2 * row_groups * sk >= 160) {
      hipLaunchKernelGGL((k_gemm_wide<2, EPI>), dim3(g2, row_groups, sk), dim3(512), 0, s, a);
      return true;
    }
  } else {
    if (g4 * row_groups * sk >= 160) {
      hipLaunchKernelGGL((k_gemm_wide<4, EPI>), dim3(g4, row_groups, sk), dim3(512), 0, s, a);
      return true;
    }
    if (g2 * row_groups * sk >= 160) {
      hipLaunchKernelGGL((k_gemm_wide<2, EPI>), dim3(g2, row_groups, sk), dim3(512), 0, s, a);
      return true;
    }
  }
  hipLaunchKernelGGL((k_gemm_wide<1, EPI>), dim3(g1, row_groups, sk), dim3(512), 0, s, a);
  return true;
}

// bf16-mode GEMM for at most 16 rows whose output only has to exist as a sum: O-proj and FFN-down add into the
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
  uint4 wv[U][NTW];
  auto load_weights = [&](int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kc = min(kt + u * 8, k1 - 1);                // clamped: always a tile of this share
#pragma unroll
      for (int j = 0; j < NTW; ++j) wv[u][j] = Wp[((size_t)min(nt0 + j, a.n_tiles - 1) * Kt + kc) * 64 + lane];
    }
  };
  const bool row_live = (lane & 15) < a.rows_live;            // (as in k_gemm16: rows that exist in no launch are not fetched)
  uint4 xv[U];
#pragma unroll
  for (int u = 0; u < U; ++u) xv[u] = make_uint4(0u, 0u, 0u, 0u);
  auto load_x = [&](int kt) {
    if (row_live) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int kc = min(kt + u * 8, k1 - 1);
        xv[u] = Xp[(size_t)kc * 64 + lane];
      }
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
      const uint4 ah = in_k ? xv[u] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
      for (int j = 0; j < NTW; ++j) {
        acc[j] = mfma_f16(ah, wv[u][j], acc[j]);
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
  else if (try_gemm_wide<EPI>(a, max_rows, 1, s)) return;
  else {
    // column tiles per wave that share the activation fragments: as many as leave about 192 workgroups
    // as few passes over the weights as 4 row tiles per pass allow, the row tiles spread evenly over them
    // (80 rows: 2 passes of 3 tiles, not 4 + 1)
    const int row_tiles = (max_rows + 15) / 16;
    constexpr bool DUAL = EPI == EPI_SWIGLU;
#define SPRINTER_ROWS(MT_, NTW_) hipLaunchKernelGGL((k_gemm_rows<MT_, NTW_, EPI>), grid, dim3(512), 0, s, a)
    if (row_tiles >= 5 && row_tiles <= 7 && (long long)a.n_tiles * a.Kt <= 24576) {
      // 65 .. 112 rows of a matrix under 24 MiB in ONE pass over the weights (5-7 row tiles per workgroup; the
      // registers allow two column tiles per wave, one for SwiGLU's two matrices) instead of two passes of 3-4 tiles:
      // the fixed cost per pass weighs more than the activation traffic there (an SD round of 80 entries at c2
      // 7.4 -> 6.5 ms; at c4's 4096-wide matrices the single pass is slower, 13.3 -> 14.4 ms per step)
      constexpr int ntw = DUAL ? 1 : 2;
      const dim3 grid((a.n_tiles + ntw - 1) / ntw, 1, 1);
      if (row_tiles == 5) SPRINTER_ROWS(5, ntw); else if (row_tiles == 6) SPRINTER_ROWS(6, ntw); else SPRINTER_ROWS(7, ntw);
      return;
    }
    const int passes = (row_tiles + 3) / 4;
    const int mt = std::max(2, (row_tiles + passes - 1) / passes);
    const int ntw = (!DUAL && mt > 2 && a.n_tiles / 4 >= 192) ? 4 : (a.n_tiles / 2 >= (DUAL ? 256 : 128)) ? 2 : 1;
    const dim3 grid((a.n_tiles + ntw - 1) / ntw, passes, 1);
    if (ntw == 4) { if (mt == 3) SPRINTER_ROWS(3, 4); else SPRINTER_ROWS(4, 4); }
    else if (ntw == 2) { if (mt == 2) SPRINTER_ROWS(2, 2); else if (mt == 3) SPRINTER_ROWS(3, 2); else SPRINTER_ROWS(4, 2); }
    else { if (mt == 2) SPRINTER_ROWS(2, 1); else if (mt == 3) SPRINTER_ROWS(3, 1); else SPRINTER_ROWS(4, 1); }
#undef SPRINTER_ROWS
  }
}

void launch_gemm(int dtype, int epi, const void* W, const void* W2, const void* X, size_t x_elems, const int* n_rows,
                 int N, int K, const float* bias, float* out_f32, int ldo, void* out_act, int out_K,
                 int max_rows, hipStream_t s) {
  GemmArgs a;
  memset(&a, 0, sizeof a);
  a.x_elems = x_elems;
  a.W = W; a.W2 = W2; a.X = X; a.n_rows = n_rows; a.N = N; a.K = K;
  a.Kt = (K + 31) / 32; a.n_tiles = (N + 15) / 16;
  a.bias = bias; a.out_f32 = out_f32; a.ldo = ldo; a.out_act = out_act; a.out_K = out_K; a.rows_live = max_rows;
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

int launch_gemm_part(const void* W, const void* X, size_t x_elems, const int* n_rows, int N, int K, float* part,
                     size_t part_stride, int max_shares, int max_rows, hipStream_t s) {
  GemmArgs a;
  memset(&a, 0, sizeof a);
  a.W = W; a.X = X; a.x_elems = x_elems; a.n_rows = n_rows; a.N = N; a.K = K;
  a.Kt = (K + 31) / 32; a.n_tiles = (N + 15) / 16; a.ldo = N;
  a.part = part; a.part_stride = part_stride; a.rows_live = max_rows;
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
  // 17+ rows: the workgroup's activation traffic (1 KiB per k tile and 16 rows) is what costs, so a wave takes
  // four column tiles (two if that leaves too few workgroups) and K is split until about 256 workgroups exist,
  // with at least two k tiles per wave and share
  if (max_rows >= 97) {            // 97+ rows: column-split workgroups, K shares until about 256 of them exist
    const int row_groups = (max_rows + 127) / 128, s_lim = std::max(1, std::min(max_shares, a.Kt / 16));
    // first with four column tiles per wave (the shares make up for the fewer column groups), then with two
    for (int per_group : {32, 16}) {
      const int groups = (a.n_tiles + per_group - 1) / per_group * row_groups;
      const int sk = std::max(1, std::min(s_lim, (256 + groups - 1) / groups));
      if (per_group == 32 && groups * sk < 160) continue;
      a.SK = sk;
      if (try_gemm_wide<EPI_PART>(a, max_rows, sk, s, 97)) return sk;
    }
  }
  const int row_tiles = (max_rows + 15) / 16;
  const int s_max = std::max(1, std::min(max_shares, a.Kt / 16));
#define SPRINTER_PART(MT_, NTW_) hipLaunchKernelGGL((k_gemm_rows<MT_, NTW_, EPI_PART>), grid, dim3(512), 0, s, a)
  if (row_tiles >= 5 && row_tiles <= 7 && (long long)a.n_tiles * a.Kt <= 24576) {   // small matrix: one pass of 5-7 row tiles
    const int groups = (a.n_tiles + 1) / 2, sk = std::min(s_max, std::max(1, 256 / groups));
    a.SK = sk;
    const dim3 grid(groups, 1, sk);
    if (row_tiles == 5) SPRINTER_PART(5, 2); else if (row_tiles == 6) SPRINTER_PART(6, 2); else SPRINTER_PART(7, 2);
    return sk;
  }
  const int passes = (row_tiles + 3) / 4;
  const int mt = std::max(2, (row_tiles + passes - 1) / passes);
  int ntw = 4, groups = (a.n_tiles + 3) / 4, sk = std::min(s_max, std::max(1, 256 / groups));
  if (groups * sk < 192 || mt == 4) { ntw = 2; groups = (a.n_tiles + 1) / 2; sk = std::min(s_max, std::max(1, 256 / groups)); }
  a.SK = sk;
  const dim3 grid(groups, passes, sk);
  if (ntw == 4) { if (mt == 2) SPRINTER_PART(2, 4); else if (mt == 3) SPRINTER_PART(3, 4); else SPRINTER_PART(4, 4); }
  else { if (mt == 2) SPRINTER_PART(2, 2); else if (mt == 3) SPRINTER_PART(3, 2); else SPRINTER_PART(4, 2); }
#undef SPRINTER_PART
  return sk;
}

}  // namespace sprinter
