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
  void* ao; int ao_K; size_t ao_plane;
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

// Append-only launch of a multi-entry pass: rotate the new key, round key and value to bf16 and write them to the
// entry's cache slot - what k_attn_bf16 does in its prologue, without the attention around it.  One 64-lane
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
  *reinterpret_cast<uint4*>(dst + (size_t)slot * DH + chunk * 8) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
}

// Causal attention on the matrix cores for a multi-entry pass whose entries come in runs of consecutive positions of
// one batch row (prefill); every key and value of the pass is already cached (the append-only launch ran before).
// One wave per (block of 16 entries, query head).  Per block of 32 keys: S = Q K^T (16 x 32 scores, Q as hi + lo bf16
// planes so that it enters at float32 precision, K straight from the cache in operand layout), causal mask per
// query, online softmax in float32 on the accumulator layout (a query's 16 keys of a tile sit in one DPP row),
// P through LDS into operand layout (hi + lo), V through LDS transposed (the MFMA wants 8 consecutive keys per
// lane), O += P V.  A block that straddles two batch rows handles its runs one after the other.
template <int DH>
__global__ __launch_bounds__(64) void k_attn_mfma_bf16(AttnArgs a) {
  constexpr int T = DH / 32, CT = DH / 16, VS = DH + 8, PS = 36;
  constexpr float NEG = -1e30f;
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  __shared__ __attribute__((aligned(16))) bf16_t lds_v[32 * VS];
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
    struct Blk { u32x4 k[2][T]; u32x4 v[DH / 16]; };
    auto fetch = [&](Blk& B, int kb) {
#pragma unroll
      for (int tile = 0; tile < 2; ++tile) {
        const bf16_t* kr = Kc + (size_t)min(kb + tile * 16 + l16, max_slot) * DH + lq * 8;
#pragma unroll
        for (int t = 0; t < T; ++t) B.k[tile][t] = *reinterpret_cast<const u32x4*>(kr + t * 32);
      }
#pragma unroll
      for (int i = 0; i < DH / 16; ++i) {
        const int u = lane + 64 * i, key = u / (DH / 8), piece = u % (DH / 8);
        B.v[i] = *reinterpret_cast<const u32x4*>(Vc + (size_t)min(kb + key, max_slot) * DH + piece * 8);
      }
    };
    auto step = [&](const Blk& B, int kb) {
      // stage V[kb .. kb+31][0 .. DH) in LDS (rows beyond the run's last key as zeros: they may hold anything)
#pragma unroll
      for (int i = 0; i < DH / 16; ++i) {
        const int u = lane + 64 * i, key = u / (DH / 8), piece = u % (DH / 8);
        const u32x4 z = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4*>(lds_v + key * VS + piece * 8) = (kb + key > max_slot) ? z : B.v[i];
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
        // V^T in operand layout: column ct * 16 + l16, keys lq * 8 .. + 8
        const bf16_t* vr = lds_v + (lq * 8) * VS + ct * 16 + l16;
        uint4 vf;
        vf.x = (unsigned)vr[0] | ((unsigned)vr[VS] << 16);
        vf.y = (unsigned)vr[2 * VS] | ((unsigned)vr[3 * VS] << 16);
        vf.z = (unsigned)vr[4 * VS] | ((unsigned)vr[5 * VS] << 16);
        vf.w = (unsigned)vr[6 * VS] | ((unsigned)vr[7 * VS] << 16);
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
      for (int ct = 0; ct < CT; ++ct) act_store<bf16_t>(ao, a.ao_plane, r0 + e, h * DH + ct * 16 + l16, a.ao_K, O[ct][v] * inv);
    }
    s0 = s1;
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
  if (a.phase == 1) {          // append only
    hipLaunchKernelGGL((k_kv_append_bf16<DH>), dim3(a.KVH, max_rows), dim3(64), 0, s, a);
    return;
  }
  if (a.phase == 3) {          // attend-only over runs of consecutive positions of one row: the matrix-core kernel
    hipLaunchKernelGGL((k_attn_mfma_bf16<DH>), dim3(a.H, (max_rows + 15) / 16), dim3(64), 0, s, a);
    return;
  }
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
  a.phase = (phase == 3 && dtype == 0) ? 2 : phase;      // the run-sharing kernel exists for bf16 only
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

}  // namespace sprinter
