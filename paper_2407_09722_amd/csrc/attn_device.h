// Device-side tree attention of float32 models (kernels_attn.hip).
#pragma once
#include "common.h"

#include <type_traits>

namespace mtad {

constexpr int RB = 16;  // query rows per workgroup

template <typename T, int HD>
struct AttnCfg {
  static constexpr int TK = (sizeof(T) == 4 && HD == 128) ? 32 : 64;  // keys per tile (LDS budget)
  static constexpr int KSTRIDE = (sizeof(T) == 2) ? HD + 2 : HD + 1;  // odd dword stride: no bank conflicts
};

__device__ __forceinline__ float wsum(float v) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wmax(float v) {
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

template <typename T, int HD, int NTHR>
struct AttnSmem {
  using C = AttnCfg<T, HD>;
  float q_s[RB][HD];
  __attribute__((aligned(16))) T k_s[C::TK * C::KSTRIDE];
  __attribute__((aligned(16))) T v_s[C::TK * HD];
  float s_s[RB][C::TK];
  float m_s[RB], l_s[RB], a_s[RB];
  unsigned long long mask_s[RB];
  int last_s;
};

// One work item = (key split, head, 16-row chunk, sequence), processed by all NTHR threads of the workgroup.
template <typename T, typename OutT, int HD, int NTHR, bool COH = false>
__device__ __forceinline__ void attn_item(AttnSmem<T, HD, NTHR>& sm, const float* __restrict__ q, int q_stride, const RowDesc& rd,
                                          const KvView& kv, int layer, int B, int R, int n_heads, int n_chunks, float scale,
                                          float* __restrict__ partial, int n_splits, int* __restrict__ counters,
                                          OutT* __restrict__ out, int split, int head, int chunk, int seq) {
  using C = AttnCfg<T, HD>;
  constexpr int TK = C::TK, KS = C::KSTRIDE;
  constexpr int NW = NTHR / 64;
  constexpr int NRG = NTHR / TK, RPT = RB / NRG;    // score phase: row groups, rows per thread
  constexpr int NRG2 = NTHR / HD, RPT2 = RB / NRG2;  // PV phase
  static_assert(RB % NRG == 0 && RB % NRG2 == 0 && RPT >= 1 && RPT2 >= 1, "thread count does not tile the row chunk");

  auto& q_s = sm.q_s; auto& k_s = sm.k_s; auto& v_s = sm.v_s; auto& s_s = sm.s_s;
  auto& m_s = sm.m_s; auto& l_s = sm.l_s; auto& a_s = sm.a_s; auto& mask_s = sm.mask_s; int& last_s = sm.last_s;

  const int t = threadIdx.x;
  const int row0 = chunk * RB;                     // first row (within the sequence) of this chunk
  const int nrows = min(RB, R - row0);
  const int KVH = kv.n_kv_heads;
  const int g = head * KVH / n_heads;
  const int len = kv.len[seq];
  int nspec = rd.nspec[seq];
  nspec = max(0, min(nspec, 64));
  const int cap = kv_capacity(kv);
  const int ktot = min(len + nspec, cap);

  // queries of this chunk and head
  for (int i = t; i < RB * HD; i += NTHR) {
    const int r = i / HD, d = i % HD;
    q_s[r][d] = (r < nrows) ? ld4<COH>(q + (int64_t)(seq * R + row0 + r) * q_stride + (int64_t)head * HD + d) : 0.f;
  }
  if (t < RB) {
    m_s[t] = -INFINITY;
    l_s[t] = 0.f;
    a_s[t] = 0.f;
    mask_s[t] = (t < nrows) ? rd.mask[seq * R + row0 + t] : 0ull;
  }
  float acc[RPT2];
#pragma unroll
  for (int i = 0; i < RPT2; ++i) acc[i] = 0.f;

  int per = (ktot + n_splits - 1) / n_splits;
  per = ((per + TK - 1) / TK) * TK;
  const int kbeg = split * per, kend = min(ktot, kbeg + per);

  const T* kbase = (const T*)kv.k + (int64_t)layer * kv.layer_stride + (int64_t)g * HD;
  const T* vbase = (const T*)kv.v + (int64_t)layer * kv.layer_stride + (int64_t)g * HD;
  constexpr int EPC = 16 / sizeof(T);  // elements per 16-byte chunk
  constexpr int CPK = HD / EPC;        // chunks per key

  for (int tile = kbeg; tile < kend; tile += TK) {
    __syncthreads();  // previous tile fully consumed (and q_s / stats initialised on the first pass)
    for (int c = t; c < TK * CPK; c += NTHR) {
      const int j = c / CPK, e = (c % CPK) * EPC;
      const int kj = tile + j;
      uint4 kk = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
      if (kj < kend) {
        const int64_t off = kv_token_offset(kv, seq, kj) + e;
        kk = *(const uint4*)(kbase + off);  // cache rows are written once per pass, before anyone reads them: no stale copy can exist
        vv = *(const uint4*)(vbase + off);
      }
      uint32_t* kd = (uint32_t*)(k_s + j * KS + e);  // padded stride: 4-byte aligned only
      kd[0] = kk.x; kd[1] = kk.y; kd[2] = kk.z; kd[3] = kk.w;
      *(uint4*)(v_s + j * HD + e) = vv;
    }
    __syncthreads();

    // scores: thread (key j, row group rg)
    {
      const int j = t % TK, rg = t / TK;
      float sacc[RPT];
#pragma unroll
      for (int i = 0; i < RPT; ++i) sacc[i] = 0.f;
      const T* krow = k_s + j * KS;
#pragma unroll 8
      for (int d = 0; d < HD; d += 2) {
        float k0, k1;
        if constexpr (sizeof(T) == 2) {
          typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
          const half2_t w = *(const half2_t*)(krow + d);
          k0 = (float)w[0];
          k1 = (float)w[1];
        } else {
          k0 = krow[d];
          k1 = krow[d + 1];
        }
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
          const float2 qq = *(const float2*)&q_s[rg + NRG * i][d];
          sacc[i] = fmaf(qq.x, k0, sacc[i]);
          sacc[i] = fmaf(qq.y, k1, sacc[i]);
        }
      }
      const int kj = tile + j;
#pragma unroll
      for (int i = 0; i < RPT; ++i) {
        const int r = rg + NRG * i;
        bool vis = kj < kend;
        if (vis && kj >= len) vis = (mask_s[r] >> (kj - len)) & 1ull;
        s_s[r][j] = vis ? sacc[i] * scale : -INFINITY;
      }
    }
    __syncthreads();

    // running softmax statistics: wave w owns rows w, w+4, ...
    {
      const int lane = t & 63, w = t >> 6;
      for (int r = w; r < RB; r += NW) {
        const float s = (lane < TK) ? s_s[r][lane] : -INFINITY;
        const float m_old = m_s[r];
        const float m_new = fmaxf(m_old, wmax(s));
        const float p = (s == -INFINITY) ? 0.f : expf(s - m_new);
        const float alpha = (m_old == -INFINITY) ? 0.f : expf(m_old - m_new);
        const float l_new = l_s[r] * alpha + wsum(p);
        if (lane < TK) s_s[r][lane] = p;
        if (lane == 0) {
          m_s[r] = m_new;
          l_s[r] = l_new;
          a_s[r] = alpha;
        }
      }
    }
    __syncthreads();

    // output accumulation: thread (dim d, row group rg2)
    {
      const int d = t % HD, rg2 = t / HD;
#pragma unroll
      for (int i = 0; i < RPT2; ++i) acc[i] *= a_s[rg2 + NRG2 * i];
      for (int j = 0; j < TK; ++j) {
        const float v = (float)v_s[j * HD + d];
#pragma unroll
        for (int i = 0; i < RPT2; ++i) acc[i] = fmaf(s_s[rg2 + NRG2 * i][j], v, acc[i]);
      }
    }
  }
  __syncthreads();

  // partial[seq][head][row][split][HD+2] = (m, l, acc[HD]).  Partials travel between workgroups (possibly on
  // different XCDs, whose L2s are not coherent with each other) as device-scope relaxed atomics: write-through
  // stores and cache-bypassing loads, no L2 flush.
  {
    const int d = t % HD, rg2 = t / HD;
#pragma unroll
    for (int i = 0; i < RPT2; ++i) {
      const int r = rg2 + NRG2 * i;
      if (r < nrows) {
        float* p = partial + ((((int64_t)seq * n_heads + head) * R + row0 + r) * n_splits + split) * (HD + 2);
        __hip_atomic_store(p + 2 + d, acc[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (d == 0) {
          __hip_atomic_store(p, m_s[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(p + 1, l_s[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
  }

  // the workgroup that arrives last merges the splits of its rows
  __builtin_amdgcn_s_waitcnt(0);  // the stores have been acknowledged
  __syncthreads();
  if (t == 0) {
    int* c = counters + ((int64_t)seq * n_heads + head) * n_chunks + chunk;
    const int prev = __hip_atomic_fetch_add(c, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    last_s = (prev == n_splits - 1);
    if (last_s) __hip_atomic_store(c, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // clean for the next launch
  }
  __syncthreads();
  if (!last_s) return;
  {
    const int d = t % HD, rg2 = t / HD;
    const int64_t lo_plane = (int64_t)B * R * n_heads * HD;
#pragma unroll
    for (int i = 0; i < RPT2; ++i) {
      const int r = rg2 + NRG2 * i;
      if (r >= nrows) continue;
      const float* p = partial + (((int64_t)seq * n_heads + head) * R + row0 + r) * n_splits * (HD + 2);
      // running merge in split order, eight splits' loads in flight at a time (deterministic)
      float M = -INFINITY, L = 0.f, o = 0.f;
      for (int s2 = 0; s2 < n_splits; s2 += 8) {
        float mm[8], ll[8], oo[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const bool ok = s2 + j < n_splits;
          const float* ps = p + (int64_t)(ok ? s2 + j : 0) * (HD + 2);
          mm[j] = ok ? __hip_atomic_load(ps, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : -INFINITY;
          ll[j] = ok ? __hip_atomic_load(ps + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
          oo[j] = ok ? __hip_atomic_load(ps + 2 + d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          if (mm[j] == -INFINITY) continue;
          const float Mn = fmaxf(M, mm[j]);
          const float ws = (M == -INFINITY) ? 0.f : expf(M - Mn), wj = expf(mm[j] - Mn);
          L = L * ws + ll[j] * wj;
          o = o * ws + oo[j] * wj;
          M = Mn;
        }
      }
      const float y = (L > 0.f) ? o / L : 0.f;
      const int64_t idx = (int64_t)(seq * R + row0 + r) * n_heads * HD + (int64_t)head * HD + d;
      if constexpr (sizeof(OutT) == 2) {  // hi / lo planes
        bf16_t hi, lo;
        split_bf16(y, hi, lo);
        if constexpr (COH) {  // 2-byte values: pair up with the neighbouring dim so that the store is a whole dword
          const uint32_t hi2 = (uint32_t)hi | ((uint32_t)__shfl_down((int)hi, 1, 64) << 16);
          const uint32_t lo2 = (uint32_t)lo | ((uint32_t)__shfl_down((int)lo, 1, 64) << 16);
          if ((d & 1) == 0) {
            __hip_atomic_store((uint32_t*)(out + idx), hi2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store((uint32_t*)(out + lo_plane + idx), lo2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
        } else {
          out[idx] = hi;
          out[lo_plane + idx] = lo;
        }
      } else {
        out[idx] = y;
      }
    }
  }
}

}  // namespace mtad
