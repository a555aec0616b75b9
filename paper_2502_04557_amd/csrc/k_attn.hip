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

// Attention for a multi-entry pass whose entries come in long runs of consecutive positions of one batch row (prefill):
// every key and value of the pass is already in the cache (the append-only launch ran before), so a workgroup takes QB
// consecutive entries x the GH query heads of one KV head (QB * GH = 8 queries) and streams the row's keys and values
// ONCE for all of them - each query masks the keys beyond its own position.  A block that straddles two batch rows
// handles them one after the other.  Same lane layout and online softmax as k_attn_bf16 with 8 query heads.
template <int DH, int GH, int QB>
__global__ __launch_bounds__(256) void k_attn_block_bf16(AttnArgs a) {
  constexpr int NW = 4, VQ = GH * QB, LPK = DH / 8, KPW = 64 / LPK, NB = 4;
  constexpr float NEG = -1e30f;
  __shared__ float s_m[NW][VQ], s_l[NW][VQ], s_o[NW][VQ][DH];
  const int n_rows = *a.rd.n_rows, r0 = blockIdx.y * QB;
  if (r0 >= n_rows) return;
  const int kvh = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = wave_index();
  const int chunk = lane % LPK, kin = lane / LPK, S = a.max_seq;
  const bool upper = chunk >= LPK / 2;
  const int pchunk = chunk ^ (LPK / 2);
  const int n_here = min(QB, n_rows - r0);
  for (int s0 = 0; s0 < n_here;) {
    const int b = a.rd.b[r0 + s0];
    int s1 = s0 + 1;
    while (s1 < n_here && a.rd.b[r0 + s1] == b) ++s1;          // entries s0 .. s1-1 of the block belong to row b
    const bf16_t* __restrict__ Kc = (const bf16_t*)a.kcache + a.layer_off + ((size_t)b * a.KVH + kvh) * (size_t)S * DH;
    const bf16_t* __restrict__ Vc = (const bf16_t*)a.vcache + a.layer_off + ((size_t)b * a.KVH + kvh) * (size_t)S * DH;
    int slot[QB], max_slot = 0;
#pragma unroll
    for (int e = 0; e < QB; ++e) {
      slot[e] = (e >= s0 && e < s1) ? a.rd.slot[r0 + e] : -1;  // -1: not a query of this pass, every key masked
      max_slot = max(max_slot, slot[e]);
    }
    const int n_blocks = (max_slot + 1 + KPW - 1) / KPW;        // a query's own key sits at its slot
    const int n_rounds = (n_blocks + NW * NB - 1) / (NW * NB);
    uint4 kA[NB], vA[NB];
    auto request = [&](int rd) {
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int key = min(((rd * NB + j) * NW + w) * KPW + kin, max_slot);
        kA[j] = *reinterpret_cast<const uint4*>(Kc + (size_t)key * DH + chunk * 8);
        vA[j] = *reinterpret_cast<const uint4*>(Vc + (size_t)key * DH + chunk * 8);
      }
    };
    request(0);
    // the queries: this lane's 8 elements of every (entry, head), rotated by the entry's own angles
    float q[VQ][8];
#pragma unroll
    for (int e = 0; e < QB; ++e) {
      const int re = r0 + min(max(e, s0), s1 - 1);              // entries outside the run re-read a row of the run
      const float* __restrict__ y = a.y + (size_t)re * a.dqkv;
      const float* __restrict__ cs = a.rope + (size_t)re * DH + 2 * (chunk % (LPK / 2)) * 8;
      float csr[16];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float4 t = reinterpret_cast<const float4*>(cs)[i];
        csr[4 * i] = t.x; csr[4 * i + 1] = t.y; csr[4 * i + 2] = t.z; csr[4 * i + 3] = t.w;
      }
#pragma unroll
      for (int g = 0; g < GH; ++g) {
        const float* qs = y + (size_t)(kvh * GH + g) * DH;
        float qx[8], qp[8];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const float4 t = reinterpret_cast<const float4*>(qs + chunk * 8)[i], u = reinterpret_cast<const float4*>(qs + pchunk * 8)[i];
          qx[4 * i] = t.x; qx[4 * i + 1] = t.y; qx[4 * i + 2] = t.z; qx[4 * i + 3] = t.w;
          qp[4 * i] = u.x; qp[4 * i + 1] = u.y; qp[4 * i + 2] = u.z; qp[4 * i + 3] = u.w;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float c = a.use_rope ? csr[2 * i] : 1.f, sn = a.use_rope ? csr[2 * i + 1] : 0.f;
          q[e * GH + g][i] = (upper ? qx[i] * c + qp[i] * sn : qx[i] * c - qp[i] * sn) * a.scale;
        }
      }
    }
    float m[VQ], l[VQ], acc[VQ][8];
#pragma unroll
    for (int v = 0; v < VQ; ++v) {
      m[v] = NEG; l[v] = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[v][i] = 0.f;
    }
    for (int rd = 0; rd < n_rounds; ++rd) {
      if (rd > 0) request(rd);
      float sc[NB][VQ];
      int keyj[NB];
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        keyj[j] = ((rd * NB + j) * NW + w) * KPW + kin;
        const bf16_t* kt = reinterpret_cast<const bf16_t*>(&kA[j]);
        float kf[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) kf[i] = bf2f(kt[i]);
#pragma unroll
        for (int v = 0; v < VQ; ++v) {
          float d = 0.f;
#pragma unroll
          for (int i = 0; i < 8; ++i) d += q[v][i] * kf[i];
          sc[j][v] = group_sum<LPK>(d);
        }
      }
#pragma unroll
      for (int v = 0; v < VQ; ++v) {
        float mn = m[v];
#pragma unroll
        for (int j = 0; j < NB; ++j) mn = keyj[j] <= slot[v / GH] ? fmaxf(mn, sc[j][v]) : mn;
        const float corr = __expf(m[v] - mn);
        m[v] = mn;
        l[v] *= corr;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[v][i] *= corr;
      }
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const bf16_t* vt = reinterpret_cast<const bf16_t*>(&vA[j]);
        float vf[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) vf[i] = bf2f(vt[i]);
#pragma unroll
        for (int v = 0; v < VQ; ++v) {
          const float p = keyj[j] <= slot[v / GH] ? __expf(sc[j][v] - m[v]) : 0.f;
          l[v] += p;
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[v][i] += p * vf[i];
        }
      }
    }
    // merge the KPW lane groups of the wave, then the waves through LDS
#pragma unroll
    for (int v = 0; v < VQ; ++v) {
#pragma unroll
      for (int o = LPK; o < 64; o <<= 1) {
        const float mo = __shfl_xor(m[v], o), lo = __shfl_xor(l[v], o);
        const float mn = fmaxf(m[v], mo);
        const float c1 = __expf(m[v] - mn), c2 = __expf(mo - mn);
        l[v] = l[v] * c1 + lo * c2;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[v][i] = acc[v][i] * c1 + __shfl_xor(acc[v][i], o) * c2;
        m[v] = mn;
      }
      if (kin == 0) {
        if (chunk == 0) { s_m[w][v] = m[v]; s_l[w][v] = l[v]; }
#pragma unroll
        for (int i = 0; i < 8; ++i) s_o[w][v][chunk * 8 + i] = acc[v][i];
      }
    }
    __syncthreads();
    bf16_t* __restrict__ ao = (bf16_t*)a.ao;
    for (int idx = tid; idx < VQ * DH; idx += NW * 64) {
      const int v = idx / DH, i = idx % DH, e = v / GH, g = v % GH;
      if (e < s0 || e >= s1) continue;
      float mn = s_m[0][v];
#pragma unroll
      for (int q4 = 1; q4 < NW; ++q4) mn = fmaxf(mn, s_m[q4][v]);
      float den = 0.f, num = 0.f;
#pragma unroll
      for (int q4 = 0; q4 < NW; ++q4) {
        const float c = __expf(s_m[q4][v] - mn);
        den += c * s_l[q4][v];
        num += c * s_o[q4][v][i];
      }
      act_store<bf16_t>(ao, a.ao_plane, r0 + e, (kvh * GH + g) * DH + i, a.ao_K, num / den);
    }
    __syncthreads();                                            // LDS is reused by the block's next run
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
  if (a.phase == 3) {
    // attend-only over long runs of consecutive positions: 8 queries share a key stream.  Used at head dimension 64
    // (c2's prefill 66 -> 58 ms); at 128 the kernel is bound by its dot products, not by the key stream, and the
    // 8-query variant measured slower (c3's prefill 290 -> 317 ms), as it would with 8 query heads per KV head.
    if constexpr (DH == 64) {
      if (G == 1) { hipLaunchKernelGGL((k_attn_block_bf16<DH, 1, 8>), dim3(a.KVH, (max_rows + 7) / 8), dim3(256), 0, s, a); return; }
      if (G == 2) { hipLaunchKernelGGL((k_attn_block_bf16<DH, 2, 4>), dim3(a.KVH, (max_rows + 3) / 4), dim3(256), 0, s, a); return; }
      if (G == 4) { hipLaunchKernelGGL((k_attn_block_bf16<DH, 4, 2>), dim3(a.KVH, (max_rows + 1) / 2), dim3(256), 0, s, a); return; }
    }
    AttnArgs b = a;
    b.phase = 2;
    launch_attn_bf16<DH>(b, G, max_rows, ctx_bound, s);
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
