// HIP kernels of the batched SPRINTER decode step for gfx950: single-query attention over the KV caches.
#include "dev.h"
#include <algorithm>
#include <cstring>

namespace sprinter {

// ============================================================== attention
// One workgroup per (row, KV head): rotary on q and the new k, append k/v to the
// cache, scores against all cached keys, softmax, weighted sum of values.
// The G query heads that share the KV head are processed together.
struct AttnArgs {
  const float* y; const float* rope; RowDesc rd;
  void* kcache; void* vcache; size_t layer_off;
  int H, KVH, dqkv, max_seq, use_rope; float scale;
  void* ao; int ao_K;
  int phase;   // 0 append + attend, 1 append only, 2 attend only, 3 attend only over long runs of one row (launcher only)
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
    act_store<T>(ao, r, kvh * G * DH + idx, a.ao_K, o);
  }
}

// Layout of the bf16 value cache.  The key cache is row-major [slot][DH]: a row is already what the matrix
// instruction wants for S = Q K^T (contraction over DH).  O = P V contracts over the keys, so the values are kept
// as operand tiles of V^T: per (row, KV head) blocks of 32 slots, a block holds DH / 16 tiles of 16 columns x 32
// keys (1 KiB, lane = (key % 32) / 8 * 16 + column % 16, 8 consecutive keys per lane).  A wave then fetches a
// value tile with one coalesced 16-byte-per-lane load and feeds it to the MFMA unchanged; appending one key is
// DH scattered 2-byte stores.  Slots per (row, KV head) are a multiple of 32 (AttnArgs::max_seq in bf16 mode).
__device__ __forceinline__ size_t vt_index(int slot, int d, int DH) {
  return (size_t)(slot >> 5) * (size_t)(32 * DH) + (size_t)(d >> 4) * 512 + (size_t)(((((slot & 31) >> 3) << 4) + (d & 15)) * 8 + (slot & 7));
}
// One operand piece of a value tile (8 consecutive keys from `key0` of one column): keys after `slot` become 0 (the
// cache may hold anything there, and 0 x NaN is NaN on the matrix cores), key == slot becomes `own` (bf16 bits).
__device__ __forceinline__ uint4 vt_fix(uint4 v, int key0, int slot, unsigned own) {
  unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int key = key0 + e;
    unsigned h = (e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffffu);
    h = key > slot ? 0u : (key == slot ? own : h);
    w[e >> 1] = (e & 1) ? ((w[e >> 1] & 0xffffu) | (h << 16)) : ((w[e >> 1] & 0xffff0000u) | h);
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding global access
// of the wave (vmcnt(0)): here that would be the first block's keys and values, requested on purpose long before
// they are needed, and the cache append.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// bf16 single-query attention on the matrix cores: one workgroup of NW waves per (row, KV head); the G query heads
// that share the KV head are rows of one 16-row operand, so a cached key costs the same whatever G is and the
// kernel is left with streaming the cache.  Wave w takes the 32-key blocks w, w + NW, ...; per block
// S = Q K^T (Q rotated, scaled and split into hi + lo bf16 planes in LDS, so it enters at float32
// precision; K fragments straight from the cache), online softmax in float32 on the accumulator layout (the 16 keys
// of a tile sit in one DPP row), P through a wave-private piece of LDS into operand layout (hi + lo), V^T tiles
// straight from the cache, O += P V.  A block's keys and value tiles are requested a whole step ahead (two register
// buffers; the query operand is kept in LDS to make room); nothing in the loop synchronises waves.  The row's own key and value
// (the token being processed) are computed in the prologue, appended to the cache by wave 0 and patched into the
// operands of the block that holds slot `slot`, which is the row's last block; keys beyond it are masked.
// The waves' partial results are merged through LDS at the end.
//   phase 0: append + attend; 1: append only; 2: attend only (the entry is already cached; patching it in again
//   changes nothing).
template <int DH, int NW>
__global__ __launch_bounds__(NW * 64, 2) void k_attn_dec_bf16(AttnArgs a) {
  constexpr int T = DH / 32, CT = DH / 16, PS = 36, HALF = DH / 2, GMAX = 8;
  constexpr float NEG = -1e30f;
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  __shared__ __attribute__((aligned(16))) float lds_p[NW][GMAX * PS];
  __shared__ __attribute__((aligned(16))) bf16_t lds_kn[DH];
  __shared__ uint4 lds_q[2][T][64];
  __shared__ float s_ml[NW][GMAX][2];
  __shared__ float s_o[NW][GMAX][DH];
  const int r = blockIdx.y;
  const int kvh = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = wave_index();
  const int l16 = lane & 15, lq = lane >> 4, G = a.H / a.KVH;
  // What depends on the row index alone is requested first, before the row count and the row's descriptor are
  // known (the projection buffer holds every row the grid covers): the new value per column (every wave), and for
  // wave t < T the 32-column piece t of the query heads and of the new key with their rotary partners and angles.
  // The G query heads form one operand (row l16 = head min(l16, G - 1): rows beyond G repeat the last head and are
  // ignored).  Spread over T waves the preparation is a quarter of the arithmetic per wave and its loads overlap
  // the descriptor's round trips (one wave doing all of it after the descriptor took 3.4 of c2's 7.4 us).
  const float* __restrict__ y = a.y + (size_t)r * a.dqkv;
  const float* __restrict__ rp = a.rope + (size_t)r * DH;
  const float* __restrict__ yq = y + (size_t)(kvh * G + min(l16, G - 1)) * DH;
  const float* __restrict__ yk = y + (size_t)(a.H + kvh) * DH;
  const float* __restrict__ yv = y + (size_t)(a.H + a.KVH + kvh) * DH;
  float vraw[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) vraw[ct] = yv[ct * 16 + l16];
  const int tq = min(w, T - 1);                                  // this wave's piece (waves beyond T repeat the last one and drop it)
  const int d0 = tq * 32 + lq * 8, p0 = d0 ^ HALF;
  float x[8], xp[8], kx[8], kp[8], cs[16];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float4 u = reinterpret_cast<const float4*>(yq + d0)[i], v = reinterpret_cast<const float4*>(yq + p0)[i];
    const float4 ku = reinterpret_cast<const float4*>(yk + d0)[i], kv = reinterpret_cast<const float4*>(yk + p0)[i];
    x[4 * i] = u.x; x[4 * i + 1] = u.y; x[4 * i + 2] = u.z; x[4 * i + 3] = u.w;
    xp[4 * i] = v.x; xp[4 * i + 1] = v.y; xp[4 * i + 2] = v.z; xp[4 * i + 3] = v.w;
    kx[4 * i] = ku.x; kx[4 * i + 1] = ku.y; kx[4 * i + 2] = ku.z; kx[4 * i + 3] = ku.w;
    kp[4 * i] = kv.x; kp[4 * i + 1] = kv.y; kp[4 * i + 2] = kv.z; kp[4 * i + 3] = kv.w;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float4 u = reinterpret_cast<const float4*>(rp + 2 * (d0 % HALF))[i];
    cs[4 * i] = u.x; cs[4 * i + 1] = u.y; cs[4 * i + 2] = u.z; cs[4 * i + 3] = u.w;
  }
  if (r >= *a.rd.n_rows) return;
  const int b = a.rd.b[r], slot = a.rd.slot[r], S = a.max_seq;
  bf16_t* __restrict__ Kc = (bf16_t*)a.kcache + a.layer_off + ((size_t)b * a.KVH + kvh) * (size_t)S * DH;
  bf16_t* __restrict__ Vc = (bf16_t*)a.vcache + a.layer_off + ((size_t)b * a.KVH + kvh) * (size_t)S * DH;
  const int n_steps = (slot + 32 * NW) / (32 * NW);             // blocks 0 .. slot / 32, NW per step
  // Two register buffers: a block's key fragments and value tiles are requested a whole step ahead (the query
  // operand lives in LDS to make room for them).
  // A block beyond the row's last one is read at the last one's address (scalar clamp) and fully masked; inside a
  // block nothing is clamped: the caches hold a multiple of 32 slots per (row, KV head), so every key of a block
  // that exists lies inside the cache.  Per-lane base addresses once, block offsets are scalars.
  struct Blk { u32x4 k[2][T]; u32x4 v[CT]; };
  const bf16_t* const k_lane = Kc + (size_t)l16 * DH + lq * 8;
  const bf16_t* const v_lane = Vc + lane * 8;
  const int kb_last = slot & ~31;
  auto fetch = [&](Blk& B, int kb) {
    const size_t off = (size_t)min(kb, kb_last) * DH;            // elements; the same for keys and value tiles
#pragma unroll
    for (int tile = 0; tile < 2; ++tile)
#pragma unroll
      for (int t = 0; t < T; ++t) B.k[tile][t] = *reinterpret_cast<const u32x4*>(k_lane + off + tile * 16 * DH + t * 32);
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) B.v[ct] = *reinterpret_cast<const u32x4*>(v_lane + off + ct * 512);
  };
  Blk A, B;
  fetch(A, w * 32);
  {
    const bool upper = d0 >= HALF;
    float qv[8], kn[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float c = a.use_rope ? cs[2 * i] : 1.f, sn = a.use_rope ? cs[2 * i + 1] : 0.f;
      qv[i] = (upper ? x[i] * c + xp[i] * sn : x[i] * c - xp[i] * sn) * a.scale;
      kn[i] = upper ? kx[i] * c + kp[i] * sn : kx[i] * c - kp[i] * sn;
    }
    uint4 qh, ql;
    u32x4 knew;
    split2(qv[0], qv[1], qh.x, ql.x);
    split2(qv[2], qv[3], qh.y, ql.y);
    split2(qv[4], qv[5], qh.z, ql.z);
    split2(qv[6], qv[7], qh.w, ql.w);
    knew.x = (unsigned)f2bf(kn[0]) | ((unsigned)f2bf(kn[1]) << 16);
    knew.y = (unsigned)f2bf(kn[2]) | ((unsigned)f2bf(kn[3]) << 16);
    knew.z = (unsigned)f2bf(kn[4]) | ((unsigned)f2bf(kn[5]) << 16);
    knew.w = (unsigned)f2bf(kn[6]) | ((unsigned)f2bf(kn[7]) << 16);
    if (w < T) {                                                 // (scalar)
      lds_q[0][tq][lane] = qh;                                   // hi, lo planes of the query operand, for every wave
      lds_q[1][tq][lane] = ql;
      if (l16 == 0) {                                            // the new key: into LDS for the row's last block, and into the cache
        *reinterpret_cast<u32x4*>(lds_kn + d0) = knew;
        if (a.phase != 2) *reinterpret_cast<u32x4*>(Kc + (size_t)slot * DH + d0) = knew;
      }
    }
  }
  unsigned vnew[CT / 2];                                         // the new value of columns ct * 16 + l16 as bf16 bits, two per register
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    const unsigned h = f2bf(vraw[ct]);
    if (a.phase != 2 && w == 0 && lq == 0) Vc[vt_index(slot, ct * 16 + l16, DH)] = (bf16_t)h;
    if (ct & 1) vnew[ct >> 1] |= h << 16; else vnew[ct >> 1] = h;
  }
  if (a.phase == 1) return;
  lds_barrier();                                                 // the query operand and the new key are in LDS for every wave
  f32x4 O[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) O[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m_run[4] = {NEG, NEG, NEG, NEG}, l_run[4] = {0.f, 0.f, 0.f, 0.f};
  float* myp = lds_p[w];
  auto step = [&](Blk& Bk, int kb) {
    if (kb + 31 >= slot) {                                       // (scalar) the row's last block or beyond: patch the new key in
#pragma unroll
      for (int tile = 0; tile < 2; ++tile)
        if (kb + tile * 16 + l16 == slot) {
#pragma unroll
          for (int t = 0; t < T; ++t) Bk.k[tile][t] = *reinterpret_cast<const u32x4*>(lds_kn + t * 32 + lq * 8);
        }
    }
    f32x4 sc[2];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      sc[tile] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < T; ++t) {
        const u32x4 kk = Bk.k[tile][t];
        const uint4 kf = make_uint4(kk.x, kk.y, kk.z, kk.w);
        sc[tile] = mfma_bf16(lds_q[0][t][lane], kf, sc[tile]);
        sc[tile] = mfma_bf16(lds_q[1][t][lane], kf, sc[tile]);
      }
    }
    // accumulator register v of lane (lq, l16) is head lq * 4 + v, key kb + tile * 16 + l16
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int last = (lq * 4 + v < G) ? slot : -1;             // last valid key of accumulator row v (head lq * 4 + v)
      const bool ok0 = kb + l16 <= last, ok1 = kb + 16 + l16 <= last;
      const float mx = group_max16(fmaxf(ok0 ? sc[0][v] : NEG, ok1 ? sc[1][v] : NEG));
      const float mn = fmaxf(m_run[v], mx);
      const float corr = __expf(m_run[v] - mn);
      const float p0 = ok0 ? __expf(sc[0][v] - mn) : 0.f, p1 = ok1 ? __expf(sc[1][v] - mn) : 0.f;
      l_run[v] = l_run[v] * corr + group_sum<16>(p0 + p1);
      m_run[v] = mn;
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) O[ct][v] *= corr;
      if (lq < 2) {                                              // heads 0 .. 7 (rows beyond G hold zeros)
        myp[(lq * 4 + v) * PS + l16] = p0;
        myp[(lq * 4 + v) * PS + 16 + l16] = p1;
      }
    }
    __builtin_amdgcn_wave_barrier();                             // LDS operations of one wave complete in order
    uint4 ph, pl;                                                // P in operand layout: head l16, keys lq * 8 .. + 8
    {
      const float4 u = *reinterpret_cast<const float4*>(myp + (l16 & 7) * PS + lq * 8);
      const float4 x = *reinterpret_cast<const float4*>(myp + (l16 & 7) * PS + lq * 8 + 4);
      split2(u.x, u.y, ph.x, pl.x);
      split2(u.z, u.w, ph.y, pl.y);
      split2(x.x, x.y, ph.z, pl.z);
      split2(x.z, x.w, ph.w, pl.w);
    }
    __builtin_amdgcn_wave_barrier();
    if (kb + 31 >= slot) {                                       // (scalar) new value in, keys beyond the row's last one out
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        const unsigned own = (ct & 1) ? (vnew[ct >> 1] >> 16) : (vnew[ct >> 1] & 0xffffu);
        const uint4 f = vt_fix(make_uint4(Bk.v[ct].x, Bk.v[ct].y, Bk.v[ct].z, Bk.v[ct].w), kb + lq * 8, slot, own);
        Bk.v[ct].x = f.x; Bk.v[ct].y = f.y; Bk.v[ct].z = f.z; Bk.v[ct].w = f.w;
      }
    }
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      const uint4 vf = make_uint4(Bk.v[ct].x, Bk.v[ct].y, Bk.v[ct].z, Bk.v[ct].w);
      O[ct] = mfma_bf16(ph, vf, O[ct]);
      O[ct] = mfma_bf16(pl, vf, O[ct]);
    }
  };
  for (int i = 0; i < n_steps; i += 2) {
    const int kb = (i * NW + w) * 32;
    fetch(B, kb + 32 * NW);
    __builtin_amdgcn_sched_barrier(0);
    step(A, kb);
    __builtin_amdgcn_sched_barrier(0);
    if (i + 1 < n_steps) {                                       // (scalar condition)
      fetch(A, kb + 64 * NW);
      __builtin_amdgcn_sched_barrier(0);
      step(B, kb + 32 * NW);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // merge the waves: heads lq * 4 + v < G live in the lanes of the first G / 4 (rounded up) DPP rows
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int g = lq * 4 + v;
    if (g < G) {
      if (l16 == 0) { s_ml[w][g][0] = m_run[v]; s_ml[w][g][1] = l_run[v]; }
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) s_o[w][g][ct * 16 + l16] = O[ct][v];
    }
  }
  lds_barrier();
  bf16_t* __restrict__ ao = (bf16_t*)a.ao;
  for (int idx = tid; idx < G * DH; idx += NW * 64) {
    const int g = idx / DH, i = idx % DH;
    float mn = NEG;
#pragma unroll
    for (int q = 0; q < NW; ++q) mn = fmaxf(mn, s_ml[q][g][0]);
    float den = 0.f, num = 0.f;
#pragma unroll
    for (int q = 0; q < NW; ++q) {
      const float c = __expf(s_ml[q][g][0] - mn);
      den += c * s_ml[q][g][1];
      num += c * s_o[q][g][i];
    }
    act_store<bf16_t>(ao, r, kvh * G * DH + idx, a.ao_K, num / den);
  }
}

// Append-only launch of a multi-entry pass: rotate the new key, round key and value to bf16 and write them to the
// entry's cache slot - what k_attn_dec_bf16 does in its prologue, without the attention around it.  One 64-lane
// workgroup per (entry, KV head): the first DH / 8 lanes take the key, the next DH / 8 the value, 8 elements each.
template <int DH>
__global__ __launch_bounds__(64) void k_kv_append_bf16(AttnArgs a) {
  constexpr int LPK = DH / 8;
  const int r = blockIdx.y, lane = threadIdx.x;
  if (r >= *a.rd.n_rows || lane >= 2 * LPK) return;
  const int kvh = blockIdx.x, b = a.rd.b[r], slot = a.rd.slot[r], S = a.max_seq;
  const bool is_v = lane >= LPK;
  const int chunk = lane % LPK, pchunk = chunk ^ (LPK / 2);
  const bool upper = chunk >= LPK / 2;
  const float* __restrict__ y = a.y + (size_t)r * a.dqkv + (size_t)(a.H + (is_v ? a.KVH : 0) + kvh) * DH;
  const float* __restrict__ cs = a.rope + (size_t)r * DH + 2 * (chunk % (LPK / 2)) * 8;
  float x[8], xp[8], c16[16];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float4 u = reinterpret_cast<const float4*>(y + chunk * 8)[i], w = reinterpret_cast<const float4*>(y + pchunk * 8)[i];
    x[4 * i] = u.x; x[4 * i + 1] = u.y; x[4 * i + 2] = u.z; x[4 * i + 3] = u.w;
    xp[4 * i] = w.x; xp[4 * i + 1] = w.y; xp[4 * i + 2] = w.z; xp[4 * i + 3] = w.w;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float4 u = reinterpret_cast<const float4*>(cs)[i];
    c16[4 * i] = u.x; c16[4 * i + 1] = u.y; c16[4 * i + 2] = u.z; c16[4 * i + 3] = u.w;
  }
  const bool rot = a.use_rope && !is_v;
  unsigned pk[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float v2[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int e = 2 * i + j;
      const float c = rot ? c16[2 * e] : 1.f, sn = rot ? c16[2 * e + 1] : 0.f;
      v2[j] = upper ? x[e] * c + xp[e] * sn : x[e] * c - xp[e] * sn;
    }
    pk[i] = (unsigned)f2bf(v2[0]) | ((unsigned)f2bf(v2[1]) << 16);
  }
  bf16_t* __restrict__ dst = (bf16_t*)(is_v ? a.vcache : a.kcache) + a.layer_off + ((size_t)b * a.KVH + kvh) * (size_t)S * DH;
  if (!is_v) {
    *reinterpret_cast<uint4*>(dst + (size_t)slot * DH + chunk * 8) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
  } else {                                                       // value cache: operand tiles of V^T (vt_index)
#pragma unroll
    for (int e = 0; e < 8; ++e)
      dst[vt_index(slot, chunk * 8 + e, DH)] = (bf16_t)((e & 1) ? (pk[e >> 1] >> 16) : (pk[e >> 1] & 0xffffu));
  }
}

// Causal attention on the matrix cores for a multi-entry pass whose entries come in runs of consecutive positions of
// one batch row (prefill); every key and value of the pass is already cached (the append-only launch ran before).
// One wave per (block of 16 entries, query head).  Per block of 32 keys: S = Q K^T (16 x 32 scores, Q as hi + lo bf16
// planes so that it enters at float32 precision, K straight from the cache in operand layout), causal mask per
// query, online softmax in float32 on the accumulator layout (a query's 16 keys of a tile sit in one DPP row),
// P through LDS into operand layout (hi + lo), V^T tiles straight from the cache (keys beyond the run's last one
// zeroed: 0 x NaN is NaN), O += P V.  A block that straddles two batch rows handles its runs one after the other.
template <int DH>
__global__ __launch_bounds__(64) void k_attn_mfma_bf16(AttnArgs a) {
  constexpr int T = DH / 32, CT = DH / 16, PS = 36;
  constexpr float NEG = -1e30f;
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  __shared__ __attribute__((aligned(16))) float lds_p[16 * PS];
  const int n_rows = *a.rd.n_rows, r0 = blockIdx.y * 16;
  if (r0 >= n_rows) return;
  const int h = blockIdx.x, kvh = h / (a.H / a.KVH), lane = threadIdx.x, l16 = lane & 15, lq = lane >> 4, S = a.max_seq;
  const int n_here = min(16, n_rows - r0);
  for (int s0 = 0; s0 < n_here;) {
    const int b = a.rd.b[r0 + s0];
    int s1 = s0 + 1;
    while (s1 < n_here && a.rd.b[r0 + s1] == b) ++s1;            // entries s0 .. s1-1 belong to batch row b
    const bf16_t* __restrict__ Kc = (const bf16_t*)a.kcache + a.layer_off + ((size_t)b * a.KVH + kvh) * (size_t)S * DH;
    const bf16_t* __restrict__ Vc = (const bf16_t*)a.vcache + a.layer_off + ((size_t)b * a.KVH + kvh) * (size_t)S * DH;
    int max_slot = 0;
    for (int e = s0; e < s1; ++e) max_slot = max(max_slot, a.rd.slot[r0 + e]);
    int slot[4];                                                 // of this lane's 4 accumulator rows (queries)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int e = lq * 4 + v;
      slot[v] = (e >= s0 && e < s1) ? a.rd.slot[r0 + e] : -1;    // -1: not a query of this run, every key masked
    }
    // Q in operand layout: row l16 of the block, elements t * 32 + lq * 8 .. + 8, rotated and scaled
    uint4 qh[T], ql[T];
    {
      const int re = r0 + min(max(l16, s0), s1 - 1);
      const float* __restrict__ y = a.y + (size_t)re * a.dqkv + (size_t)h * DH;
      const float* __restrict__ rp = a.rope + (size_t)re * DH;
#pragma unroll
      for (int t = 0; t < T; ++t) {
        const int d0 = t * 32 + lq * 8, p0 = d0 ^ (DH / 2);
        const bool upper = d0 >= DH / 2;
        float x[8], xp[8], cs[16], qv[8];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const float4 u = reinterpret_cast<const float4*>(y + d0)[i], w = reinterpret_cast<const float4*>(y + p0)[i];
          x[4 * i] = u.x; x[4 * i + 1] = u.y; x[4 * i + 2] = u.z; x[4 * i + 3] = u.w;
          xp[4 * i] = w.x; xp[4 * i + 1] = w.y; xp[4 * i + 2] = w.z; xp[4 * i + 3] = w.w;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float4 u = reinterpret_cast<const float4*>(rp + 2 * (d0 % (DH / 2)))[i];
          cs[4 * i] = u.x; cs[4 * i + 1] = u.y; cs[4 * i + 2] = u.z; cs[4 * i + 3] = u.w;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float c = a.use_rope ? cs[2 * i] : 1.f, sn = a.use_rope ? cs[2 * i + 1] : 0.f;
          qv[i] = (upper ? x[i] * c + xp[i] * sn : x[i] * c - xp[i] * sn) * a.scale;
        }
        split2(qv[0], qv[1], qh[t].x, ql[t].x);
        split2(qv[2], qv[3], qh[t].y, ql[t].y);
        split2(qv[4], qv[5], qh[t].z, ql[t].z);
        split2(qv[6], qv[7], qh[t].w, ql[t].w);
      }
    }
    f32x4 O[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) O[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m_run[4] = {NEG, NEG, NEG, NEG}, l_run[4] = {0.f, 0.f, 0.f, 0.f};
    // Two register buffers: the keys (operand fragments) and values (staging pieces) of block kb + 32 are requested
    // before block kb is worked on.  Addresses are clamped to the run's last key, so a block beyond it loads valid
    // memory, has every key masked and every value zeroed, and changes nothing.
    struct Blk { u32x4 k[2][T]; u32x4 v[CT]; };
    auto fetch = [&](Blk& B, int kb) {
#pragma unroll
      for (int tile = 0; tile < 2; ++tile) {
        const bf16_t* kr = Kc + (size_t)min(kb + tile * 16 + l16, max_slot) * DH + lq * 8;
#pragma unroll
        for (int t = 0; t < T; ++t) B.k[tile][t] = *reinterpret_cast<const u32x4*>(kr + t * 32);
      }
      const bf16_t* vb = Vc + (size_t)(min(kb, max_slot & ~31) >> 5) * (32 * DH) + lane * 8;
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) B.v[ct] = *reinterpret_cast<const u32x4*>(vb + ct * 512);
    };
    auto step = [&](Blk& B, int kb) {
      if (kb + 31 > max_slot) {                                   // (scalar) zero the values of keys beyond the run's last one
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          const uint4 f = vt_fix(make_uint4(B.v[ct].x, B.v[ct].y, B.v[ct].z, B.v[ct].w), kb + lq * 8, max_slot + 1, 0u);
          B.v[ct].x = f.x; B.v[ct].y = f.y; B.v[ct].z = f.z; B.v[ct].w = f.w;
        }
      }
      // scores of the two 16-key tiles
      f32x4 sc[2];
#pragma unroll
      for (int tile = 0; tile < 2; ++tile) {
        sc[tile] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < T; ++t) {
          const u32x4 kk = B.k[tile][t];
          const uint4 kf = make_uint4(kk.x, kk.y, kk.z, kk.w);
          sc[tile] = mfma_bf16(qh[t], kf, sc[tile]);
          sc[tile] = mfma_bf16(ql[t], kf, sc[tile]);
        }
      }
      // online softmax: accumulator register v of lane (lq, l16) is query lq * 4 + v, key kb + tile * 16 + l16
      float p[2][4];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const bool ok0 = kb + l16 <= slot[v], ok1 = kb + 16 + l16 <= slot[v];
        const float mx = group_max16(fmaxf(ok0 ? sc[0][v] : NEG, ok1 ? sc[1][v] : NEG));
        const float mn = fmaxf(m_run[v], mx);
        const float corr = __expf(m_run[v] - mn);
        p[0][v] = ok0 ? __expf(sc[0][v] - mn) : 0.f;
        p[1][v] = ok1 ? __expf(sc[1][v] - mn) : 0.f;
        l_run[v] = l_run[v] * corr + group_sum<16>(p[0][v] + p[1][v]);
        m_run[v] = mn;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) O[ct][v] *= corr;
        lds_p[(lq * 4 + v) * PS + l16] = p[0][v];
        lds_p[(lq * 4 + v) * PS + 16 + l16] = p[1][v];
      }
      __syncthreads();
      // P in operand layout: query l16, keys lq * 8 .. + 8 of the block
      uint4 ph, pl;
      {
        const float4 u = *reinterpret_cast<const float4*>(lds_p + l16 * PS + lq * 8);
        const float4 w = *reinterpret_cast<const float4*>(lds_p + l16 * PS + lq * 8 + 4);
        split2(u.x, u.y, ph.x, pl.x);
        split2(u.z, u.w, ph.y, pl.y);
        split2(w.x, w.y, ph.z, pl.z);
        split2(w.z, w.w, ph.w, pl.w);
      }
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        const uint4 vf = make_uint4(B.v[ct].x, B.v[ct].y, B.v[ct].z, B.v[ct].w);
        O[ct] = mfma_bf16(ph, vf, O[ct]);
        O[ct] = mfma_bf16(pl, vf, O[ct]);
      }
      __syncthreads();                                           // LDS is rewritten by the next key block
    };
    Blk A, B;
    fetch(A, 0);
    for (int kb = 0; kb <= max_slot; kb += 64) {
      fetch(B, kb + 32);
      __builtin_amdgcn_sched_barrier(0);
      step(A, kb);
      fetch(A, kb + 64);
      __builtin_amdgcn_sched_barrier(0);
      step(B, kb + 32);
    }
    bf16_t* __restrict__ ao = (bf16_t*)a.ao;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int e = lq * 4 + v;
      if (e < s0 || e >= s1) continue;
      const float inv = 1.0f / l_run[v];
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) act_store<bf16_t>(ao, r0 + e, h * DH + ct * 16 + l16, a.ao_K, O[ct][v] * inv);
    }
    s0 = s1;
  }
}

static size_t attn_smem_bytes(int DH, int G, int max_seq) {
  return (size_t)(G * DH + 2 * DH + 4 * G * DH + G * max_seq) * sizeof(float);
}

template <int DH>
static void launch_attn_bf16(const AttnArgs& a, int G, int max_rows, int ctx_bound, hipStream_t s) {
  if (a.phase == 1) {          // append only
    hipLaunchKernelGGL((k_kv_append_bf16<DH>), dim3(a.KVH, max_rows), dim3(64), 0, s, a);
    return;
  }
  if (a.phase == 3) {          // attend-only over runs of consecutive positions of one row: the matrix-core kernel
    hipLaunchKernelGGL((k_attn_mfma_bf16<DH>), dim3(a.H, (max_rows + 15) / 16), dim3(64), 0, s, a);
    return;
  }
  // NW = waves per workgroup that share one (row, KV head)'s keys: 8 when the launch has no more workgroups than
  // the chip has compute units and the contexts are long, else 4
  dim3 grid(a.KVH, max_rows);
  const bool wide = (long long)a.KVH * max_rows <= 256 && ctx_bound >= 512;
  if (wide) hipLaunchKernelGGL((k_attn_dec_bf16<DH, 8>), grid, dim3(512), 0, s, a);
  else hipLaunchKernelGGL((k_attn_dec_bf16<DH, 4>), grid, dim3(256), 0, s, a);
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
                      int max_rows, hipStream_t s, int phase) {
  AttnArgs a;
  a.phase = (phase == 3 && dtype == 0) ? 2 : phase;      // the run-sharing kernel exists for bf16 only
  a.y = y; a.rope = rope; a.rd = rd; a.kcache = kcache; a.vcache = vcache; a.layer_off = layer_off;
  a.H = md.H; a.KVH = md.KVH; a.dqkv = md.dqkv; a.max_seq = max_seq; a.use_rope = md.arch == 1;
  a.scale = 1.0f / sqrtf((float)md.dh);
  a.ao = ao; a.ao_K = md.H * md.dh;
  int G = md.H / md.KVH;
  if (dtype == 0) {
    if (md.dh == 64) launch_attn_g<float, 64>(a, G, max_rows, s); else launch_attn_g<float, 128>(a, G, max_rows, s);
  } else {
    if (md.dh == 64) launch_attn_bf16<64>(a, G, max_rows, ctx_bound, s); else launch_attn_bf16<128>(a, G, max_rows, ctx_bound, s);
  }
}

}  // namespace sprinter
