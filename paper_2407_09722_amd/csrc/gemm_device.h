// Device-side pieces of the skinny bf16 matrix product shared by the stand-alone kernel (kernels_gemm.hip)
// and the one-launch pass (kernels_flow.hip): fragment types, operand loads and the epilogues.
#pragma once
#include "common.h"
#include "gemm.h"

namespace mtad {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float floatx4;
typedef __attribute__((ext_vector_type(4))) unsigned int uintx4;

union Frag {
  uint4 u;
  uintx4 n;  // native vector: the form the nontemporal-load builtin accepts
  bf16x8 v;
};

constexpr int GW = 8;  // waves per workgroup of the stand-alone product kernel

// ---- operand loads shared by the product kernels ---------------------------------------------------------------

template <int U>
__device__ __forceinline__ void gemm_load_w(Frag (&w)[U], const char* strip, int KT, int kt, unsigned voff) {
  const char* base = strip + ((size_t)kt << 10);  // tiles are 1 KiB each, k-major within the strip
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (kt + u * GW < KT) w[u].n = __builtin_nontemporal_load((const uintx4*)(base + (size_t)u * (GW << 10) + voff));
}

// Activation fragments of k tiles kt + u*GW for NG row groups.  X + xoff is this lane's 16 bytes of (row group 0, k tile 0);
// a k tile is kstride bytes further, a row group gstride bytes (plane layout: 64 and 16 K; fragment order: 1024 x the
// pass's row groups and 1024).
template <int NG, int U>
__device__ __forceinline__ void gemm_load_b(Frag (&b)[U][NG], const char* X, unsigned xoff, size_t kstride, size_t gstride, int KT, int kt,
                                            int rows_here, int c) {
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      b[u][g].u = make_uint4(0, 0, 0, 0);
      const char* base = X + (size_t)g * gstride + (size_t)(kt + u * GW) * kstride;
      if (kt + u * GW < KT && g * 8 + (c & 7) < rows_here) b[u][g].u = *(const uint4*)(base + xoff);
    }
}

// (X base of the launch's first row, lane offset, k tile stride, row group stride) for either activation layout
struct ActAddr {
  const char* X;
  unsigned xoff;
  size_t kstride, gstride;
};
__device__ __forceinline__ ActAddr act_addr(const GemmArgs& a, int lane) {
  const int c = lane & 15, kg = lane >> 4;
  ActAddr r;
  if (a.ncg == 0) {
    r.X = (const char*)a.X + (size_t)a.row0 * a.K * 2;
    r.xoff = (unsigned)((((size_t)(c >> 3) * a.R + (c & 7)) * a.K + kg * 8) * 2);  // plane c/8, row c%8, k group kg
    r.kstride = 64;
    r.gstride = (size_t)16 * a.K;
  } else if (a.R <= ACT_COMPACT_ROWS) {  // fragments without the unused row slots (act_offset); one launch, row0 = 0
    r.X = (const char*)a.X;
    r.xoff = (unsigned)(((kg * 2 + (c >> 3)) * a.R + (c & 7)) * 16);  // lanes of rows past R are never loaded
    r.kstride = (size_t)a.R * 128;
    r.gstride = 128;  // the next 8 rows of the same (k group, plane)
  } else {
    r.X = (const char*)a.X + (size_t)(a.row0 >> 3) * 1024;  // launches start at multiples of 8 rows
    r.xoff = (unsigned)lane * 16u;
    r.kstride = (size_t)a.ncg * 1024;
    r.gstride = 1024;
  }
  return r;
}

// Epilogue of one row group of one strip.  s: this lane's four sums (packed features kg*4 .. +3 of strip nt, row m;
// hi and lo already folded), live: the lane holds a real row, inv: the row's fused-RMSNorm factor (1 if none).
// Every lane of the wave must call it (it shuffles).
// pre_h, pre_gn: the RESID epilogue's residual row and next-norm gain for this lane if the kernel requested them ahead
// (HAVE_PRE), else they are loaded here.
template <int EPI, bool COH = false, bool HAVE_PRE = false>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& a, int nt, floatx4 s, int m, bool live, float inv, int kg,
                                              float4 pre_h = float4{0.f, 0.f, 0.f, 0.f}, float4 pre_gn = float4{0.f, 0.f, 0.f, 0.f}) {
  const int NT = a.N >> 4, R = a.R;
    if constexpr (EPI == EPI_STORE) {
      const int n = nt * 16 + kg * 4;
      float4 o = make_float4(s[0] * inv, s[1] * inv, s[2] * inv, s[3] * inv);
      if (live) {
        float4* y = (float4*)(a.Y + (int64_t)m * a.ldy + n);
        if (a.accumulate) {
          const float4 p = *y;
          o.x += p.x; o.y += p.y; o.z += p.z; o.w += p.w;
        }
        *y = o;
      }
      if (a.lse_part) {  // (max, sum exp) over this strip's 16 features of row m, merged over the four lane groups
        float mx = fmaxf(fmaxf(o.x, o.y), fmaxf(o.z, o.w));
        float sm = expf(o.x - mx) + expf(o.y - mx) + expf(o.z - mx) + expf(o.w - mx);
        for (int off = 16; off <= 32; off <<= 1) {
          const float omx = __shfl_xor(mx, off, 64), osm = __shfl_xor(sm, off, 64);
          const float nm = fmaxf(mx, omx);
          sm = sm * expf(mx - nm) + osm * expf(omx - nm);
          mx = nm;
        }
        if (live && kg == 0) ((float2*)a.lse_part)[(int64_t)m * NT + nt] = make_float2(mx, sm);
      }
    } else if constexpr (EPI == EPI_RESID) {
      const int n = nt * 16 + kg * 4;
      float4 hn = make_float4(0.f, 0.f, 0.f, 0.f);
      if (live) {
        float4* hp = (float4*)(a.h + (int64_t)m * a.N + n);
        float4 p;
        if constexpr (HAVE_PRE) {
          p = pre_h;
        } else if constexpr (COH) {  // written by a workgroup of this kernel (an earlier step's strip owner)
          const uint4 u = ld16<true>(hp);
          p = make_float4(__uint_as_float(u.x), __uint_as_float(u.y), __uint_as_float(u.z), __uint_as_float(u.w));
        } else {
          p = *hp;
        }
        hn = make_float4(p.x + s[0], p.y + s[1], p.z + s[2], p.w + s[3]);
        if constexpr (COH) {
          st8<true>(hp, make_uint2(__float_as_uint(hn.x), __float_as_uint(hn.y)));
          st8<true>((float*)hp + 2, make_uint2(__float_as_uint(hn.z), __float_as_uint(hn.w)));
        } else {
          *hp = hn;
        }
        const float4 gn = HAVE_PRE ? pre_gn : *(const float4*)(a.g_next + n);
        ushort4 hi, lo;
        split_bf16(hn.x * gn.x, hi.x, lo.x);
        split_bf16(hn.y * gn.y, hi.y, lo.y);
        split_bf16(hn.z * gn.z, hi.z, lo.z);
        split_bf16(hn.w * gn.w, hi.w, lo.w);
        st8<COH>(a.planes_out + act_offset(a.ncg, R, a.N, 0, m, n), *(uint2*)&hi);
        st8<COH>(a.planes_out + act_offset(a.ncg, R, a.N, 1, m, n), *(uint2*)&lo);
      }
      float q = hn.x * hn.x + hn.y * hn.y + hn.z * hn.z + hn.w * hn.w;
      q += __shfl_xor(q, 16, 64);
      q += __shfl_xor(q, 32, 64);
      if (live && kg == 0) st4<COH>(a.ssq_out + (int64_t)m * NT + nt, q);
    } else {
      // paired strips: packed features 0..7 (kg 0, 1) and their partners 8..15 (kg 2, 3 = lane + 32)
      floatx4 t;
#pragma unroll
      for (int i = 0; i < 4; ++i) t[i] = __shfl_xor(s[i], 32, 64);
      if (kg < 2 && live) {
        const int i0 = kg * 4;  // 0 or 4 within the strip's 8 pairs
        if constexpr (EPI == EPI_SWIGLU) {
          const int f = a.N >> 1;
          ushort4 hi, lo;
          bf16_t* hip = (bf16_t*)&hi;
          bf16_t* lop = (bf16_t*)&lo;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float gate = s[e] * inv, up = t[e] * inv;
            split_bf16(gate / (1.0f + expf(-gate)) * up, hip[e], lop[e]);
          }
          st8<COH>(a.act_out + act_offset(a.ncg, R, f, 0, m, nt * 8 + i0), *(uint2*)&hi);
          st8<COH>(a.act_out + act_offset(a.ncg, R, f, 1, m, nt * 8 + i0), *(uint2*)&lo);
        } else {  // EPI_QKV
          const int hd = a.kv.head_dim, half = hd >> 1, tph = hd >> 4;
          const int head = nt / tph, i = (nt % tph) * 8 + i0;
          const int H = a.n_heads, KVH = a.kv.n_kv_heads;
          float x1[4], x2[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) { x1[e] = s[e] * inv; x2[e] = t[e] * inv; }
          if (head < H + KVH) {  // q and k heads are rotated
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float2 cs = a.rope[(int64_t)m * half + i + e];
              const float y1 = x1[e] * cs.x - x2[e] * cs.y, y2 = x2[e] * cs.x + x1[e] * cs.y;
              x1[e] = y1;
              x2[e] = y2;
            }
          }
          if (head < H) {
            float* q = a.q_out + (int64_t)m * H * hd + (int64_t)head * hd + i;
            st8<COH>(q, make_uint2(__float_as_uint(x1[0]), __float_as_uint(x1[1])));
            st8<COH>(q + 2, make_uint2(__float_as_uint(x1[2]), __float_as_uint(x1[3])));
            st8<COH>(q + half, make_uint2(__float_as_uint(x2[0]), __float_as_uint(x2[1])));
            st8<COH>(q + half + 2, make_uint2(__float_as_uint(x2[2]), __float_as_uint(x2[3])));
          } else {
            const int slot = a.slot[m];
            if (slot >= 0) {
              if (slot >= kv_capacity(a.kv)) {
                atomicOr(a.status, (uint32_t)ST_KV_CAP);
              } else {
                const bool is_k = head < H + KVH;
                const int gh = is_k ? head - H : head - H - KVH;
                kv16_t* dst = (kv16_t*)(is_k ? a.kv.k : a.kv.v) + (int64_t)a.layer * a.kv.layer_stride +
                              kv_token_offset(a.kv, m / a.Rseq, slot) + (int64_t)gh * hd + i;
                typedef kv16_t half4_t __attribute__((ext_vector_type(4)));
                half4_t v1, v2;
#pragma unroll
                for (int e = 0; e < 4; ++e) { v1[e] = (kv16_t)x1[e]; v2[e] = (kv16_t)x2[e]; }
                st8<COH>(dst, *(uint2*)&v1);
                st8<COH>(dst + half, *(uint2*)&v2);
              }
            }
          }
        }
      }
    }
}

// Sum of the NWAVES partial sums of row group g (in wave order).  Called by wave g < NG after the partial sums are in
// `red` ([wave][g][lane]) and a workgroup barrier.
template <int NG, int NWAVES = GW>
__device__ __forceinline__ floatx4 gemm_sum_waves(int g, const floatx4* red, int lane) {
  floatx4 s = red[g * 64 + lane];
  for (int w2 = 1; w2 < NWAVES; ++w2) {
    const floatx4 t2 = red[(w2 * NG + g) * 64 + lane];
    s[0] += t2[0]; s[1] += t2[1]; s[2] += t2[2]; s[3] += t2[3];
  }
  return s;
}

// The RESID epilogue's inputs of (strip nt, row group g) for this lane: residual values and next-norm gain (zeros for
// lanes without a row).  Requested for several epilogues at once, their latencies overlap instead of adding up.
__device__ __forceinline__ void gemm_resid_inputs(const GemmArgs& a, int nt, int g, int rows_here, int lane, float4& h, float4& gn) {
  const int c = lane & 15, kg = lane >> 4;
  const int mrel = g * 8 + (c & 7);
  h = float4{0.f, 0.f, 0.f, 0.f};
  gn = h;
  if (c < 8 && mrel < rows_here) {
    const int n = nt * 16 + kg * 4;
    h = *(const float4*)(a.h + (int64_t)(a.row0 + mrel) * a.N + n);
    gn = *(const float4*)(a.g_next + n);
  }
}

// hi + lo fold of a row group's sums, then the epilogue.
template <int EPI, bool COH = false, bool HAVE_PRE = false>
__device__ __forceinline__ void gemm_finish_sum(const GemmArgs& a, int nt, int g, floatx4 s, const float* inv_s, int rows_here, int lane,
                                                float4 pre_h = float4{0.f, 0.f, 0.f, 0.f}, float4 pre_gn = float4{0.f, 0.f, 0.f, 0.f}) {
  const int c = lane & 15, kg = lane >> 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) s[i] += __shfl_xor(s[i], 8, 64);  // columns c and c + 8 are the hi and lo terms of one row
  const int mrel = g * 8 + (c & 7);
  const bool live = c < 8 && mrel < rows_here;
  const float inv = (a.ssq && live) ? inv_s[mrel] : 1.0f;
  gemm_epilogue<EPI, COH, HAVE_PRE>(a, nt, s, a.row0 + mrel, live, inv, kg, pre_h, pre_gn);
}

// Both steps for a workgroup that holds a strip's whole reduction dimension.
template <int NG, int EPI, bool COH = false, int NWAVES = GW, bool HAVE_PRE = false>
__device__ __forceinline__ void gemm_finish_group(const GemmArgs& a, int nt, int g, const floatx4* red, const float* inv_s,
                                                  int rows_here, int lane, float4 pre_h = float4{0.f, 0.f, 0.f, 0.f},
                                                  float4 pre_gn = float4{0.f, 0.f, 0.f, 0.f}) {
  const int c = lane & 15, kg = lane >> 4;
  floatx4 s = gemm_sum_waves<NG, NWAVES>(g, red, lane);
#pragma unroll
  for (int i = 0; i < 4; ++i) s[i] += __shfl_xor(s[i], 8, 64);  // columns c and c + 8 are the hi and lo terms of one row
  const int mrel = g * 8 + (c & 7);
  const bool live = c < 8 && mrel < rows_here;
  const float inv = (a.ssq && live) ? inv_s[mrel] : 1.0f;
  gemm_epilogue<EPI, COH, HAVE_PRE>(a, nt, s, a.row0 + mrel, live, inv, kg, pre_h, pre_gn);
}

// Row factors of a fused RMSNorm into inv_s[0 .. rows_here): 1/sqrt(sum of the producer's partial sums of squares / K + eps).
// All waves of the workgroup take part; the caller synchronises afterwards.  A wave takes rows wave, wave + n_waves, ...
// RB of them at a time with all their loads in flight together: one row after the other is one memory latency per row,
// 21 in a row for a 164-row pass (measured: 16 and 23 us of the 13B-shaped QKV and gate/up products).
template <bool COH = false, int RB = 1>
__device__ __forceinline__ void gemm_row_factors(const GemmArgs& a, float* inv_s, int rows_here, int wave, int lane, int n_waves) {
  if (!a.ssq) return;
  constexpr int NPI = 8;  // partial sums per lane held at once: rows of up to 512 partial sums
  if (RB == 1 || a.NP > NPI * 64) {
    for (int m = wave; m < rows_here; m += n_waves) {
      float s = 0.f;
      for (int p = lane; p < a.NP; p += 64) s += ld4<COH>(a.ssq + (int64_t)(a.row0 + m) * a.NP + p);
      for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
      if (lane == 0) inv_s[m] = 1.0f / sqrtf(s / (float)a.K + a.eps);
    }
    return;
  }
  const int npi = (a.NP + 63) >> 6;  // uniform
  for (int m0 = wave; m0 < rows_here; m0 += n_waves * RB) {
    float v[RB][NPI];
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      const int m = min(m0 + r * n_waves, rows_here - 1);  // past the end: an existing row once more, dropped below
#pragma unroll
      for (int i = 0; i < NPI; ++i)
        if (i < npi) v[r][i] = ld4<COH>(a.ssq + (int64_t)(a.row0 + m) * a.NP + min(lane + 64 * i, a.NP - 1));
    }
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < NPI; ++i)
        if (i < npi && lane + 64 * i < a.NP) s += v[r][i];
      for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
      const int m = m0 + r * n_waves;
      if (lane == 0 && m < rows_here) inv_s[m] = 1.0f / sqrtf(s / (float)a.K + a.eps);
    }
  }
}

}  // namespace mtad
