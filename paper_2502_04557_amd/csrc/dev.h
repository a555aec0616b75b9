// Device-side helpers shared by the kernels (k_*.hip): bf16 conversion, operand-tile indexing,
// wave reductions, Philox4x32-10 / Gumbel noise, packed arg-max keys.
#pragma once
#include "internal.h"
#include <math.h>

namespace sprinter {

typedef unsigned short bf16_t;   // raw bfloat16 bits (weights as given, KV caches); also the 16-bit element type of an
                                 // activation operand, whose bits are float16 (below)
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned long long u64;

// ------------------------------------------------------------------ scalars
__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((unsigned)v) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {   // round to nearest even
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);   // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<bf16_t>(bf16_t v) { return bf2f(v); }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { return f2bf(v); }

// Activation layout: float32 mode = row-major [m][K]; bf16 mode = MFMA operand tiles.
template <typename T> __device__ __forceinline__ size_t act_idx(int m, int k, int K);
template <> __device__ __forceinline__ size_t act_idx<float>(int m, int k, int K) { return (size_t)m * K + k; }
template <> __device__ __forceinline__ size_t act_idx<bf16_t>(int m, int k, int K) {
  int Kt = (K + 31) >> 5;
  return ((size_t)(m >> 4) * Kt + (k >> 5)) * 512 + ((((k & 31) >> 3) << 4) + (m & 15)) * 8 + (k & 7);
}

// Store one activation.  In bf16 mode the GEMM operands are float16: the weights (bf16 values, converted once when
// they are packed - exact above 2^-14) and the activations, rounded to nearest even with 11 significant bits, so
// that one matrix instruction per product carries eight times the precision of a bf16 activation; the products
// accumulate in float32.  Values beyond the float16 range (65504) become infinities and show as such downstream.
__device__ __forceinline__ unsigned short f2h(float v) {
  const _Float16 h = (_Float16)v;
  return __builtin_bit_cast(unsigned short, h);
}
template <typename T> __device__ __forceinline__ void act_store(T* base, int m, int k, int K, float v);
template <> __device__ __forceinline__ void act_store<float>(float* base, int m, int k, int K, float v) {
  base[act_idx<float>(m, k, K)] = v;
}
template <> __device__ __forceinline__ void act_store<bf16_t>(bf16_t* base, int m, int k, int K, float v) {
  base[act_idx<bf16_t>(m, k, K)] = f2h(v);
}

// Two floats -> packed bf16 pair (v_cvt_pk_bf16_f32, round to nearest even), and the hi + lo split of a pair (the
// attention kernels keep the query and the probabilities as two bf16 operands next to the bf16 keys / values).
typedef float f2v __attribute__((ext_vector_type(2)));
typedef __bf16 b2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pk_bf16(float a, float b) {
  f2v v = {a, b};
  b2v h = __builtin_convertvector(v, b2v);   // v_cvt_pk_bf16_f32, round to nearest even
  return __builtin_bit_cast(unsigned, h);
}
// Two floats -> packed float16 pair of an activation operand (round to nearest even).
typedef _Float16 h2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pk_f16(float a, float b) {
  f2v v = {a, b};
  h2v h = __builtin_convertvector(v, h2v);
  return __builtin_bit_cast(unsigned, h);
}
__device__ __forceinline__ void split2(float a, float b, unsigned& hi, unsigned& lo) {
  hi = pk_bf16(a, b);
  lo = pk_bf16(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}
__device__ __forceinline__ float gelu_tanh(float x) {
  const float c = 0.7978845608028654f;   // sqrt(2/pi)
  return 0.5f * x * (1.0f + tanhf(c * (x + 0.044715f * x * x * x)));
}
__device__ __forceinline__ float silu(float x) { return x / (1.0f + expf(-x)); }

// The wave's index inside its workgroup as a scalar.  Conditions built from it are then scalar too,
// so the compiler branches around matrix instructions instead of masking them with EXEC: the MFMA
// instructions ignore the EXEC mask and would run (on stale registers) inside a masked-off block.
__device__ __forceinline__ int wave_index() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// ------------------------------------------------------------- reductions
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int o) {
  unsigned lo = __shfl_xor((unsigned)v, o), hi = __shfl_xor((unsigned)(v >> 32), o);
  return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 umax64(u64 a, u64 b) { return a > b ? a : b; }

// block-wide reductions for 256-thread blocks; result broadcast to all threads
__device__ __forceinline__ float block_sum256(float v, float* s4) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) s4[threadIdx.x >> 6] = v;
  __syncthreads();
  return ((s4[0] + s4[1]) + s4[2]) + s4[3];
}
__device__ __forceinline__ float block_max256(float v, float* s4) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) s4[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(s4[0], s4[1]), fmaxf(s4[2], s4[3]));
}

// ------------------------------------------------- Philox4x32-10 + Gumbel
// Counter-based generator of Salmon et al. (SC'11).  key = seed, counter =
// (vocab index / 4, position, row, stream); word (vocab index % 4) of the block.  philox_block: the whole block of
// four words (vocabulary indices 4 c0 .. 4 c0 + 3 of one row and position).
__device__ __forceinline__ uint4 philox_block(unsigned k0, unsigned k1, unsigned stream, unsigned b, unsigned t,
                                              unsigned c0) {
  unsigned c1 = t, c2 = b, c3 = stream;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    unsigned hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    unsigned hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    unsigned n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  return make_uint4(c0, c1, c2, c3);
}
__device__ __forceinline__ unsigned philox_word(unsigned k0, unsigned k1, unsigned stream, unsigned b,
                                                unsigned t, unsigned v) {
  const uint4 c = philox_block(k0, k1, stream, b, t, v >> 2);
  const unsigned sel = v & 3u;
  return sel == 0 ? c.x : sel == 1 ? c.y : sel == 2 ? c.z : c.w;
}
// u = ((word >> 9) + 0.5) * 2^-23 is exact in float32 and inside (0,1).
__device__ __forceinline__ float gumbel_from_word(unsigned w) {
  float u = ((float)(w >> 9) + 0.5f) * 1.1920928955078125e-07f;
  return -logf(-logf(u));
}
// (value, index) -> one integer whose order is "larger value first, then smaller index"
__device__ __forceinline__ u64 pack_key(float y, unsigned n) {
  y = y + 0.0f;   // -0 -> +0
  unsigned u = __float_as_uint(y);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((u64)u << 32) | (u64)(0xFFFFFFFFu - n);
}
__device__ __forceinline__ int key_index(u64 k) { return (int)(0xFFFFFFFFu - (unsigned)(k & 0xFFFFFFFFull)); }

// Largest key of row m over the per-workgroup partial results part[n_wg][Mpad] (all 64 lanes get it).
__device__ __forceinline__ u64 merge_partials(const u64* part, int n_wg, int Mpad, int m, int lane) {
  u64 k = 0;
  for (int i0 = lane; i0 < n_wg; i0 += 256) {                  // four loads in flight per lane
    u64 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + 64 * u;
      v[u] = i < n_wg ? part[(size_t)i * Mpad + m] : 0;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) k = umax64(k, v[u]);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) k = umax64(k, shfl_xor_u64(k, o));
  return k;
}

__device__ __forceinline__ u64 sample_key(float logit, const SamplerArgs& sa, int b, int t, int n) {
  float y = logit;
  if (sa.inv_temperature > 0.0f)
    y = logit * sa.inv_temperature + gumbel_from_word(philox_word(sa.seed_lo, sa.seed_hi, sa.stream, b, t, n));
  return pack_key(y, (unsigned)n);
}

// Sampling keys of a matrix-core accumulator: register v of the lane is the logit of (row v of four, column n), and
// the four lanes of a quad hold four consecutive columns 4 c .. 4 c + 3 of the same four rows, i.e. words 0 .. 3 of
// the same four random blocks.  Lane q of the quad computes the block of row q (whose batch row and position the
// caller passes as b_q, t_q) and the quad exchanges words through DPP broadcasts: one block per lane instead of
// four - the integer multiplies of the generator are most of the sampling arithmetic.  Same words as sample_key.
// All 64 lanes must be active.
__device__ __forceinline__ void sample_keys_quad(f32x4 logit, const SamplerArgs& sa, int b_q, int t_q, int n, u64 (&key)[4]) {
  if (!(sa.inv_temperature > 0.0f)) {                 // (uniform)
#pragma unroll
    for (int v = 0; v < 4; ++v) key[v] = pack_key(logit[v], (unsigned)n);
    return;
  }
  const uint4 blk = philox_block(sa.seed_lo, sa.seed_hi, sa.stream, (unsigned)b_q, (unsigned)t_q, (unsigned)n >> 2);
  const int sel = n & 3;
#define SPRINTER_QUAD_ROW(V, CTRL)                                                                     \
  {                                                                                                    \
    const unsigned x = (unsigned)__builtin_amdgcn_update_dpp(0, (int)blk.x, CTRL, 0xF, 0xF, true);     \
    const unsigned y = (unsigned)__builtin_amdgcn_update_dpp(0, (int)blk.y, CTRL, 0xF, 0xF, true);     \
    const unsigned z = (unsigned)__builtin_amdgcn_update_dpp(0, (int)blk.z, CTRL, 0xF, 0xF, true);     \
    const unsigned w = (unsigned)__builtin_amdgcn_update_dpp(0, (int)blk.w, CTRL, 0xF, 0xF, true);     \
    const unsigned word = sel == 0 ? x : sel == 1 ? y : sel == 2 ? z : w;                              \
    key[V] = pack_key(logit[V] * sa.inv_temperature + gumbel_from_word(word), (unsigned)n);            \
  }
  SPRINTER_QUAD_ROW(0, 0x00)   // quad_perm [0,0,0,0]: the block lane 0 of the quad computed (row 0)
  SPRINTER_QUAD_ROW(1, 0x55)   // [1,1,1,1]
  SPRINTER_QUAD_ROW(2, 0xAA)   // [2,2,2,2]
  SPRINTER_QUAD_ROW(3, 0xFF)   // [3,3,3,3]
#undef SPRINTER_QUAD_ROW
}

// Sum over an aligned group of 8 or 16 consecutive lanes, the total in every lane of the group, through DPP
// (quad permutes, then the half-row and row mirrors: after the quad steps every lane of a quad holds the quad's
// sum, so any lane of the other half is a valid partner).  A ds_bpermute butterfly costs about 100 cycles per
// step in a dependent chain; this is four ordinary VALU adds.
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(LANES == 8 || LANES == 16, "one DPP row or half a row");
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));   // row_half_mirror
  if (LANES == 16) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true));   // row_mirror
  return v;
}

// Maximum over an aligned group of 16 consecutive lanes (one DPP row), in every lane of the group.
__device__ __forceinline__ float group_max16(float v) {
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true)));
  return v;
}

// Maximum of 64-bit keys over an aligned group of 16 consecutive lanes, in every lane of the group.
__device__ __forceinline__ u64 group_umax64_16(u64 k) {
#define SPRINTER_DPP_STEP(CTRL)                                                                              \
  {                                                                                                          \
    const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)k, CTRL, 0xF, 0xF, true);    \
    const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(k >> 32), CTRL, 0xF, 0xF, true); \
    k = umax64(k, ((u64)hi << 32) | lo);                                                                     \
  }
  SPRINTER_DPP_STEP(0xB1)    // quad_perm [1,0,3,2]
  SPRINTER_DPP_STEP(0x4E)    // quad_perm [2,3,0,1]
  SPRINTER_DPP_STEP(0x141)   // row_half_mirror
  SPRINTER_DPP_STEP(0x140)   // row_mirror
#undef SPRINTER_DPP_STEP
  return k;
}

// D += X W^T for a 16 x 32 activation tile and a 16 x 32 weight tile, both float16 operands.
__device__ __forceinline__ f32x4 mfma_f16(uint4 x, uint4 w, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<f16x8*>(&x), *reinterpret_cast<f16x8*>(&w), c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma_bf16(uint4 x, uint4 w, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8*>(&x), *reinterpret_cast<bf16x8*>(&w), c, 0,
                                                 0, 0);
}

}  // namespace sprinter
