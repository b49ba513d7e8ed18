// Skinny matrix products Y[R][N] = X[R][K] * W[N][K]^T for the few-row projections, FFN and lm_head of the
// draft and target passes: the weight stream that dominates one target pass.
//
// bf16 path.  Weights are tile-packed (pack_matrix_kernel): the 16x32 tile (nt, kt) of the matrix is 1 KiB
// contiguous, laid out exactly as the A operand of v_mfma_f32_16x16x32_bf16 wants it (lane l holds row l%16,
// k = (l/16)*8 .. +8), and the tiles of one 16-feature strip follow each other along k.  A wave therefore
// fetches every A fragment as one fully coalesced 1 KiB read and a workgroup streams one contiguous strip.
// Activations are the B operand, carried as two bf16 planes (hi + lo): the 16 columns of one MFMA hold the hi
// and lo terms of 8 rows, so a weight tile costs one MFMA per 8 rows.
// One workgroup owns one strip; its waves split the k tiles and add their partial sums in a fixed order
// (deterministic).  The epilogue variants fold the neighbouring element-wise work in:
//   STORE   plain store / accumulate; optional per-strip (max, sum-exp) partials of each row (lm_head)
//   RESID   residual add, then the next RMSNorm's input: planes of h*gain and per-strip sums of squares
//   SWIGLU  strips hold 8 gate + 8 up features: silu(gate)*up written as planes
//   QKV     strips hold features i..i+8 and i+hd/2.. of one head: rotary rotation, q to a buffer, k/v to the cache
// A product whose input is RMS-normalised takes planes of h*gain and multiplies its rows by
// 1/sqrt(mean h^2 + eps) afterwards (the factor is common to the whole row, so it commutes with the product).
//
// fp32 path (the tiny all-float32 workload): one wave per output feature, plain FMA, shuffle reduction.
#include "common.h"
#include "gemm.h"
#include "gemm_device.h"

#include <stdlib.h>

namespace mtad {

// ---- packing ------------------------------------------------------------------------------------------

// original row of packed row (nt*16 + j)
__device__ __forceinline__ int packed_src_row(int kind, int nt, int j, int head_dim, int d_ffn) {
  if (kind == PACK_QKV) {
    const int tph = head_dim / 16, head = nt / tph, u = nt % tph;
    return head * head_dim + (j < 8 ? 8 * u + j : head_dim / 2 + 8 * u + (j - 8));
  }
  if (kind == PACK_GATE_UP) return j < 8 ? 8 * nt + j : d_ffn + 8 * nt + (j - 8);
  return nt * 16 + j;
}

__global__ void pack_matrix_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int N, int K, int kind, int head_dim) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // one thread per 8-element lane fragment
  const int KT = K / 32;
  if (idx >= (int64_t)(N / 16) * KT * 64) return;
  const int lane = (int)(idx & 63);
  const int64_t tile = idx >> 6;
  const int kt = (int)(tile % KT), nt = (int)(tile / KT);
  const int row = packed_src_row(kind, nt, lane & 15, head_dim, N / 2);
  const uint4 v = *(const uint4*)(src + (int64_t)row * K + kt * 32 + (lane >> 4) * 8);
  *(uint4*)(dst + idx * 8) = v;
}

hipError_t launch_pack_matrix(const void* src, void* dst, int N, int K, int kind, int head_dim, hipStream_t s) {
  const int64_t n = (int64_t)(N / 16) * (K / 32) * 64;
  hipLaunchKernelGGL(pack_matrix_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const bf16_t*)src, (bf16_t*)dst, N, K,
                     kind, head_dim);
  return hipGetLastError();
}

// ---- the product -----------------------------------------------------------------------------------------


// One workgroup = one strip of 16 output features; its GW waves interleave over the k tiles (wave w takes tiles
// w, w + GW, ...) in batches of U tiles, and their partial sums meet in LDS in a fixed order (deterministic).
// Columns of the B operand: c < 8 = hi term of row g*8 + c, c >= 8 = lo term of row g*8 + c - 8, so one MFMA per
// weight tile covers 8 rows (NG = ceil(rows / 8) MFMAs per tile).  Wave g < NG finishes row group g.
// Each wave keeps TWO batches in flight (register sets 0 and 1): when a batch has been consumed its registers take
// the batch two places ahead.  Loads complete in issue order, so a wave that waits for its newest load has waited
// for all of them; the activation fragments of a batch (L2 hits) are therefore issued BEFORE its weight tiles, two
// batches ahead of their use, never between a batch's weight loads and its use.  Workgroups are small (512 threads,
// few registers) so that several are resident per compute unit: while one runs its epilogue or waits for its first
// tiles, the others keep the memory pipe full.
// TAG only names the call site (0 draft pass, 1 target pass, 2 component entry point) in kernel traces.

template <int NG, int EPI, int TAG>
__global__ __launch_bounds__(GW * 64) __attribute__((amdgpu_waves_per_eu((NG <= 1 && EPI != EPI_RESID) ? 6 : 4))) void gemm_bf16_kernel(GemmArgs a) {
  constexpr int U = (NG <= 2) ? 4 : (NG <= 4 ? 2 : 1);  // weight tiles per batch and wave
  __shared__ floatx4 red[GW * NG * 64];
  __shared__ float inv_s[NG * 8];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform by construction: keep it scalar
  const int nt = blockIdx.x;
  const int K = a.K, KT = K >> 5;
  const int R = a.R, row0 = a.row0;
  const int rows_here = min(NG * 8, R - row0);
  const int c = lane & 15, kg = lane >> 4;

  // (wave-uniform base) + (32-bit lane offset): the scalar-base addressing mode, one offset register per stream
  const char* strip = (const char*)a.W + (((size_t)nt * KT) << 10);
  const unsigned voff = (unsigned)lane * 16u;
  const ActAddr xa = act_addr(a, lane);

  constexpr int span = U * GW;
  Frag w[2][U], b[2][U][NG];
  gemm_load_b<NG, U>(b[0], xa.X, xa.xoff, xa.kstride, xa.gstride, KT, wave, rows_here, c);
  gemm_load_w<U>(w[0], strip, KT, wave, voff);
  gemm_load_b<NG, U>(b[1], xa.X, xa.xoff, xa.kstride, xa.gstride, KT, wave + span, rows_here, c);
  gemm_load_w<U>(w[1], strip, KT, wave + span, voff);

  floatx4 acc[NG];
#pragma unroll
  for (int g = 0; g < NG; ++g) acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};
  // RESID: the finishing wave requests its residual values and the next norm's gain now.  Products with this epilogue
  // (o, down) have about one workgroup per compute unit, so nothing else covers that latency after the stream.
  float4 pre_h = float4{0.f, 0.f, 0.f, 0.f}, pre_gn = pre_h;
  if constexpr (EPI == EPI_RESID) {
    const int mrel = wave * 8 + (c & 7);
    if (wave < NG && c < 8 && mrel < rows_here) {
      pre_h = *(const float4*)(a.h + (int64_t)(row0 + mrel) * a.N + nt * 16 + kg * 4);
      pre_gn = *(const float4*)(a.g_next + nt * 16 + kg * 4);
    }
  }

  for (int kt = wave; kt < KT; kt += 2 * span) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int k0 = kt + h * span;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (k0 + u * GW < KT) {
#pragma unroll
          for (int g = 0; g < NG; ++g) acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[h][u].v, b[h][u][g].v, acc[g], 0, 0, 0);
        }
      if (k0 + 2 * span < KT) {
        gemm_load_b<NG, U>(b[h], xa.X, xa.xoff, xa.kstride, xa.gstride, KT, k0 + 2 * span, rows_here, c);
        gemm_load_w<U>(w[h], strip, KT, k0 + 2 * span, voff);
      }
    }
  }
#pragma unroll
  for (int g = 0; g < NG; ++g) red[(wave * NG + g) * 64 + lane] = acc[g];
  gemm_row_factors<false, (NG > 1 ? NG : 1)>(a, inv_s, rows_here, wave, lane, GW);  // after the stream: its loads are L2 hits by now for most workgroups
  __syncthreads();
  if (wave < NG) gemm_finish_group<NG, EPI, false, GW, EPI == EPI_RESID>(a, nt, wave, red, inv_s, rows_here, lane, pre_h, pre_gn);
}

// The same kernel for S strips per workgroup: the activation fragments of a k tile are loaded once and multiplied with
// the S weight tiles of that k tile, so the L2 -> compute-unit traffic of the fragments per weight byte is 1/S of the
// one-strip kernel's (which spends 12 to 15 % of its time on them at 5 rows: measured by knocking the loads out).
// U tiles per batch and strip, two batches in flight as above; the S strips are reduced and finished at the
// same time by different waves.  Used with S = 3 for 4 to 8 rows (U = 2) and 9 to 24 rows (U = 1).
template <int NG, int EPI, int TAG, int S, int U>
__global__ __launch_bounds__(GW * 64) __attribute__((amdgpu_waves_per_eu((S + NG) * U * 8 + S * NG * 4 > 100 ? 2 : 4))) void gemm_bf16_strips_kernel(GemmArgs a) {
  __shared__ floatx4 red[S * GW * NG * 64];
  __shared__ float inv_s[NG * 8];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int K = a.K, KT = K >> 5, NT = a.N >> 4;
  const int R = a.R, row0 = a.row0;
  const int rows_here = min(NG * 8, R - row0);
  const int c = lane & 15;
  const int nt0 = blockIdx.x * S, ns = min(S, NT - nt0);
  const size_t strip_bytes = (size_t)KT << 10;
  const char* strip0 = (const char*)a.W + (size_t)nt0 * strip_bytes;
  const unsigned voff = (unsigned)lane * 16u;
  const ActAddr xa = act_addr(a, lane);

  constexpr int span = U * GW;
  Frag w[2][U][S], b[2][U][NG];
  auto load_w = [&](Frag (&ws)[U][S], int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int s2 = 0; s2 < S; ++s2)
        if (kt + u * GW < KT)  // a strip past the last one reads the last one again: never finished
          ws[u][s2].n = __builtin_nontemporal_load((const uintx4*)(strip0 + (size_t)min(s2, ns - 1) * strip_bytes + ((size_t)(kt + u * GW) << 10) + voff));
  };
  gemm_load_b<NG, U>(b[0], xa.X, xa.xoff, xa.kstride, xa.gstride, KT, wave, rows_here, c);
  load_w(w[0], wave);
  gemm_load_b<NG, U>(b[1], xa.X, xa.xoff, xa.kstride, xa.gstride, KT, wave + span, rows_here, c);
  load_w(w[1], wave + span);

  floatx4 acc[S][NG];
#pragma unroll
  for (int s2 = 0; s2 < S; ++s2)
#pragma unroll
    for (int g = 0; g < NG; ++g) acc[s2][g] = floatx4{0.f, 0.f, 0.f, 0.f};

  for (int kt = wave; kt < KT; kt += 2 * span) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int k0 = kt + h * span;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (k0 + u * GW < KT) {
#pragma unroll
          for (int s2 = 0; s2 < S; ++s2)
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[s2][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[h][u][s2].v, b[h][u][g].v, acc[s2][g], 0, 0, 0);
        }
      if (k0 + 2 * span < KT) {
        gemm_load_b<NG, U>(b[h], xa.X, xa.xoff, xa.kstride, xa.gstride, KT, k0 + 2 * span, rows_here, c);
        load_w(w[h], k0 + 2 * span);
      }
    }
  }
  gemm_row_factors<false, (NG > 1 ? NG : 1)>(a, inv_s, rows_here, wave, lane, GW);
  // all strips' sums to LDS at once; wave s2 * NG + g then finishes row group g of strip s2, the strips side by side
  // (one after the other, each epilogue's dependent loads, the rotary table, cache slots and residual rows, added up)
#pragma unroll
  for (int s2 = 0; s2 < S; ++s2)
#pragma unroll
    for (int g = 0; g < NG; ++g) red[((s2 * GW + wave) * NG + g) * 64 + lane] = acc[s2][g];
  __syncthreads();
  for (int item = wave; item < S * NG; item += GW) {  // (a ninth item falls to wave 0 again)
    const int s2 = item / NG, g = item % NG;
    if (s2 < ns) gemm_finish_group<NG, EPI>(a, nt0 + s2, g, red + s2 * GW * NG * 64, inv_s, rows_here, lane);
  }
}

// Several strips per workgroup, for passes of more than 8 rows.  With NG row groups a weight tile needs NG activation
// fragments of its own size from L2; a workgroup that works on S strips at once loads the fragments of a k tile
// once and uses them for S weight tiles, so the L2 -> compute-unit traffic per weight byte drops from 1 + NG to
// 1 + NG/S.  Same wave layout as above with one k tile per batch and wave; the S strips are reduced and finished one
// after the other through the same LDS buffer.  A product with about one strip per compute unit or fewer would leave
// most units idle at S > 1: its reduction dimension is then also cut into KS ranges (grid.y); every workgroup leaves
// its sums in global memory (device-scope write-through stores) and the one that arrives last for a group of strips
// adds the KS partial sums in range order and runs the epilogues (deterministic, same protocol as the attention splits).  S * NG <= 12 (16 for 48 and 64 rows) bounds the accumulator registers.
template <int NG, int EPI>
__global__ __launch_bounds__(GW * 64) void gemm_bf16_multi_kernel(GemmArgs a, int S) {
  __shared__ int last_s;
  constexpr int SM = NG <= 4 ? 12 / NG : (NG <= 6 ? 3 : 4);  // most strips per workgroup
  __shared__ floatx4 red[GW * NG * 64];
  __shared__ float inv_s[NG * 8];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int K = a.K, KT_all = K >> 5, NT = a.N >> 4;
  const int R = a.R, row0 = a.row0;
  const int rows_here = min(NG * 8, R - row0);
  const int c = lane & 15, kg = lane >> 4;
  const int nt0 = blockIdx.x * S, ns = min(S, NT - nt0);
  // this workgroup's range of k tiles [k_lo, KT)
  const int KS = gridDim.y, ks = blockIdx.y;
  const int per = (KT_all + KS - 1) / KS;
  const int k_lo = ks * per, KT = min(KT_all, k_lo + per);

  const char* strip0 = (const char*)a.W + (((size_t)nt0 * KT_all) << 10);
  const size_t strip_bytes = (size_t)KT_all << 10;
  const unsigned voff = (unsigned)lane * 16u;
  const ActAddr xa = act_addr(a, lane);

  Frag w[2][SM], b[2][1][NG];
  auto load_w = [&](Frag (&ws)[SM], int kt) {
#pragma unroll
    for (int s2 = 0; s2 < SM; ++s2)
      if (s2 < ns && kt < KT) ws[s2].n = __builtin_nontemporal_load((const uintx4*)(strip0 + s2 * strip_bytes + ((size_t)kt << 10) + voff));
  };
  gemm_load_b<NG, 1>(b[0], xa.X, xa.xoff, xa.kstride, xa.gstride, KT, k_lo + wave, rows_here, c);
  load_w(w[0], k_lo + wave);
  gemm_load_b<NG, 1>(b[1], xa.X, xa.xoff, xa.kstride, xa.gstride, KT, k_lo + wave + GW, rows_here, c);
  load_w(w[1], k_lo + wave + GW);

  floatx4 acc[SM][NG];
#pragma unroll
  for (int s2 = 0; s2 < SM; ++s2)
#pragma unroll
    for (int g = 0; g < NG; ++g) acc[s2][g] = floatx4{0.f, 0.f, 0.f, 0.f};

  for (int kt = k_lo + wave; kt < KT; kt += 2 * GW) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int k0 = kt + h * GW;
      if (k0 < KT) {
#pragma unroll
        for (int s2 = 0; s2 < SM; ++s2)
          if (s2 < ns) {
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[s2][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[h][s2].v, b[h][0][g].v, acc[s2][g], 0, 0, 0);
          }
      }
      if (k0 + 2 * GW < KT) {
        gemm_load_b<NG, 1>(b[h], xa.X, xa.xoff, xa.kstride, xa.gstride, KT, k0 + 2 * GW, rows_here, c);
        load_w(w[h], k0 + 2 * GW);
      }
    }
  }
  gemm_row_factors<false, (NG > 1 ? 8 : 1)>(a, inv_s, rows_here, wave, lane, GW);  // after the stream (see the single-strip kernel)
  // partial sums of (group, strip s2, row group g, range ks): 64 lanes x 4 floats
  float* const mypart = a.part ? a.part + ((((size_t)blockIdx.x * SM) * NG) * KS) * 256 : nullptr;
  // The strips are reduced through LDS one after the other; (strip s2, row group g) = item s2 * NG + g goes to wave
  // item % GW, which keeps the sum and runs its epilogue after the last reduction, so that the epilogues of all items
  // (dependent loads of rotary table, cache slots, residual rows) overlap instead of queueing behind NG waves.
  constexpr int HELD = (SM * NG + GW - 1) / GW;
  floatx4 held[HELD];
#pragma unroll
  for (int s2 = 0; s2 < SM; ++s2) {
    if (s2 < ns) {  // uniform over the workgroup
      if (s2 > 0) __syncthreads();  // the previous strip's sums have been read
#pragma unroll
      for (int g = 0; g < NG; ++g) red[(wave * NG + g) * 64 + lane] = acc[s2][g];
      __syncthreads();
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const int item = s2 * NG + g;
        if (wave == item % GW) {
          const floatx4 sum = gemm_sum_waves<NG>(g, red, lane);
          if (KS == 1) {
            held[item / GW] = sum;
          } else {
            float* p = mypart + ((((size_t)s2 * NG + g) * KS + ks) * 64 + lane) * 4;
            st8<true>(p, make_uint2(__float_as_uint(sum[0]), __float_as_uint(sum[1])));
            st8<true>(p + 2, make_uint2(__float_as_uint(sum[2]), __float_as_uint(sum[3])));
          }
        }
      }
    }
  }
  if (KS == 1) {
#pragma unroll
    for (int h = 0; h < HELD; ++h) {
      const int item = h * GW + wave, s2 = item / NG, g = item % NG;
      if (item < SM * NG && s2 < ns) gemm_finish_sum<EPI>(a, nt0 + s2, g, held[h], inv_s, rows_here, lane);
    }
    return;
  }
  // the workgroup that arrives last for this group of strips adds the ranges in order and finishes
  __builtin_amdgcn_s_waitcnt(0);  // the stores have been acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    const int prev = __hip_atomic_fetch_add(a.counters + blockIdx.x, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    last_s = (prev == KS - 1);
    if (last_s) __hip_atomic_store(a.counters + blockIdx.x, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // clean for the next launch
  }
  __syncthreads();
  if (!last_s) return;
  // (strip s2, row group g) = item s2 * NG + g goes to wave item % GW, as above: all waves share the merges
  for (int item = wave; item < ns * NG; item += GW) {
    const int s2 = item / NG, g = item % NG;
    const float* p = mypart + ((((size_t)s2 * NG + g) * KS) * 64 + lane) * 4;
    floatx4 sum = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int k2 = 0; k2 < KS; ++k2) {
      const uint4 v = ld16<true>(p + (size_t)k2 * 256);
      sum[0] += __uint_as_float(v.x); sum[1] += __uint_as_float(v.y); sum[2] += __uint_as_float(v.z); sum[3] += __uint_as_float(v.w);
    }
    gemm_finish_sum<EPI>(a, nt0 + s2, g, sum, inv_s, rows_here, lane);
  }
}

template <int RB>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ W, const float* __restrict__ X,
                                                       float* __restrict__ Y, int R, int N, int K, int ldy,
                                                       int accumulate) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = blockIdx.x * 4 + wave;
  const int r0 = blockIdx.y * RB;
  if (n >= N) return;
  float acc[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r) acc[r] = 0.f;
  const float* wrow = W + (int64_t)n * K;
  for (int k = lane * 4; k < K; k += 256) {
    const float4 w = *(const float4*)(wrow + k);
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      if (r0 + r < R) {
        const float4 x = *(const float4*)(X + (int64_t)(r0 + r) * K + k);
        acc[r] = fmaf(w.x, x.x, acc[r]);
        acc[r] = fmaf(w.y, x.y, acc[r]);
        acc[r] = fmaf(w.z, x.z, acc[r]);
        acc[r] = fmaf(w.w, x.w, acc[r]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    float v = acc[r];
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if (lane == 0 && r0 + r < R) {
      float* y = Y + (int64_t)(r0 + r) * ldy + n;
      *y = accumulate ? (*y + v) : v;
    }
  }
}

hipError_t launch_gemm_f32(const void* W, const void* X, float* Y, int R, int N, int K, int ldy, bool accumulate, hipStream_t s) {
  if (R <= 0) return hipSuccess;
  if (K % 4) return hipErrorInvalidValue;
  constexpr int RB = 8;
  hipLaunchKernelGGL((gemm_f32_kernel<RB>), dim3((N + 3) / 4, (R + RB - 1) / RB), dim3(256), 0, s, (const float*)W, (const float*)X,
                     Y, R, N, K, ldy, accumulate ? 1 : 0);
  return hipGetLastError();
}

template <int NG, int EPI, int TAG>
static hipError_t run_one(const GemmArgs& a, hipStream_t s) {
  hipLaunchKernelGGL((gemm_bf16_kernel<NG, EPI, TAG>), dim3(a.N / 16), dim3(GW * 64), 0, s, a);
  return hipGetLastError();
}

template <int NG, int EPI>
static hipError_t run_tag(const GemmArgs& a, int tag, hipStream_t s) {
  if constexpr (NG <= 3) {
    if (tag == 1) return run_one<NG, EPI, 1>(a, s);
    if (tag == 2) return run_one<NG, EPI, 2>(a, s);
  }
  return run_one<NG, EPI, 0>(a, s);
}

template <int NG, int EPI, int S, int U>
static hipError_t run_strips(const GemmArgs& a, int tag, hipStream_t s) {
  const int NT = a.N / 16;
  const dim3 grid((NT + S - 1) / S), block(GW * 64);
  if (tag == 1) hipLaunchKernelGGL((gemm_bf16_strips_kernel<NG, EPI, 1, S, U>), grid, block, 0, s, a);
  else if (tag == 2) hipLaunchKernelGGL((gemm_bf16_strips_kernel<NG, EPI, 2, S, U>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((gemm_bf16_strips_kernel<NG, EPI, 0, S, U>), grid, block, 0, s, a);
  return hipGetLastError();
}

template <int NG, int EPI>
static hipError_t run_multi(const GemmArgs& a, int S, int KS, hipStream_t s) {
  const int NT = a.N / 16;
  hipLaunchKernelGGL((gemm_bf16_multi_kernel<NG, EPI>), dim3((NT + S - 1) / S, KS), dim3(GW * 64), 0, s, a, S);
  return hipGetLastError();
}

static int device_cus() {
  static const int n_cus = [] {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
    return cus > 0 ? cus : 256;
  }();
  return n_cus;
}

// Products with at most SPLIT_MAX_STRIPS strips (about one per compute unit) take 4 strips per workgroup and cut the
// reduction dimension 4 ways when a workspace is offered; the workspace is sized for that.
constexpr int SPLIT_MAX_STRIPS = 384, SPLIT_S = 4, SPLIT_KS = 4, SPLIT_NG_MAX = 8;
size_t gemm_split_floats(int N) {
  const int NT = N / 16;
  const size_t skinny = NT > SPLIT_MAX_STRIPS ? 0 : (size_t)((NT + SPLIT_S - 1) / SPLIT_S) * SPLIT_S * SPLIT_NG_MAX * SPLIT_KS * 256;
  const size_t tiled = gemm_tiled_split_floats(N);
  return skinny > tiled ? skinny : tiled;
}
int gemm_split_counters(int N) {
  const int skinny = N / 16 > SPLIT_MAX_STRIPS ? 0 : (N / 16 + 1) / 2;  // groups of at least 2 strips
  const int tiled = gemm_tiled_split_counters(N);
  return skinny > tiled ? skinny : tiled;
}

// Strips per workgroup for a product with NT strips and NG row groups.  Cost model (fits the measured times at 17, 41
// and 64 rows): the busiest compute unit works on rounds * S strips, and a strip costs in proportion to the bytes
// that reach the compute unit per weight byte, 1 + NG/S; so minimise rounds * (S + NG), larger S on ties.
static int strips_per_group(int NT, int NG) {
  const int n_cus = device_cus();
  if (NG < 2) return 1;
  const int smax = NG <= 4 ? 12 / NG : (NG <= 6 ? 3 : 4);
  int best = 1, best_cost = 0x7fffffff;
  for (int S = 1; S <= smax; ++S) {
    const int groups = (NT + S - 1) / S;
    const int cost = ((groups + n_cus - 1) / n_cus) * (S + NG);
    if (cost <= best_cost) {
      best = S;
      best_cost = cost;
    }
  }
  return best;
}

template <int EPI>
static hipError_t run_epi(GemmArgs a, int tag, hipStream_t s) {
  // at most 64 rows per launch (8 row groups); more rows re-stream the weights per 64-row slab
  for (int r0 = 0; r0 < a.R; r0 += 64) {
    a.row0 = r0;
    const int ng = ((a.R - r0 < 64 ? a.R - r0 : 64) + 7) / 8;
    hipError_t e;
    const int ngt = ng <= 4 ? ng : (ng <= 6 ? 6 : 8);
    int S = strips_per_group(a.N / 16, ngt), KS = 1;
    const int smax = ngt <= 4 ? 12 / ngt : (ngt <= 6 ? 3 : 4);
    // worth its exchange when every wave keeps at least 8 k tiles, or with 64 rows (measured at 17, 41 and 64 rows)
    if (ng >= 2 && a.part && a.counters && a.N / 16 <= SPLIT_MAX_STRIPS && ((a.K >> 5) >= SPLIT_KS * GW * 8 || (ng >= 7 && (a.K >> 5) >= SPLIT_KS * GW * 2))) {
      S = smax < SPLIT_S ? smax : SPLIT_S;  // share the fragments between strips, keep every compute unit busy by cutting k
      KS = SPLIT_KS;
      if (ng <= 3) S = KS = 2;  // 9 to 24 rows: two strips and two ranges (C4 verify 4.12 -> 4.05 ms; 3 x 2, 4 x 2, 2 x 3 and 2 x 4
                                // slower; the same cut for the o projection, 128 k tiles, slower too)
      // the exchange must fit what the caller offers ((group, strip slot, row group, range) x 256 floats, a counter per group)
      const int groups = (a.N / 16 + S - 1) / S;
      if ((size_t)groups * smax * ngt * KS * 256 > a.part_floats || groups > a.counters_n) {
        S = strips_per_group(a.N / 16, ngt);
        KS = 1;
      }
    }
    // 9 to 24 rows, no k split, at least two strips per compute unit: the three-strip kernel with two or three row
    // groups, whose epilogues run side by side (C3 target at 9 and 12 rows: 3.47 -> 3.39 ms per pass; C4, 17 rows:
    // 4.22 -> 4.12 ms)
    if (KS == 1 && (ng == 2 || ng == 3) && a.N / 16 >= 2 * device_cus()) {
      e = ng == 2 ? run_strips<2, EPI, 3, 1>(a, tag, s) : run_strips<3, EPI, 3, 1>(a, tag, s);
      if (e != hipSuccess) return e;
      continue;
    }
    if (S > 1) {
      if (ng <= 2) e = run_multi<2, EPI>(a, S, KS, s);
      else if (ng <= 3) e = run_multi<3, EPI>(a, S, KS, s);
      else if (ng <= 4) e = run_multi<4, EPI>(a, S, KS, s);
      else if (ng <= 6) e = run_multi<6, EPI>(a, S, KS, s);
      else e = run_multi<8, EPI>(a, S, KS, s);
      if (e != hipSuccess) return e;
      continue;
    }
    // 4 to 8 rows and at least two strips per compute unit: three strips per workgroup share the activation fragments
    // (measured on the 7B-shaped QKV, gate/up and lm_head products: 6, 10 and 4 % faster at 5 rows, 17, 19 and 15 % at 8;
    // slower at 1 row; two, four, five or six strips per workgroup all slower than three; no gain at 9 to 24 rows over
    // the kernel below that already shares fragments there)
    if (ng <= 1 && a.R - r0 >= 4 && a.N / 16 >= 2 * device_cus()) e = run_strips<1, EPI, 3, 2>(a, tag, s);
    else if (ng <= 1) e = run_tag<1, EPI>(a, tag, s);
    else if (ng <= 2) e = run_tag<2, EPI>(a, tag, s);
    else if (ng <= 3) e = run_tag<3, EPI>(a, tag, s);
    else if (ng <= 4) e = run_tag<4, EPI>(a, tag, s);
    else if (ng <= 6) e = run_tag<6, EPI>(a, tag, s);
    else e = run_tag<8, EPI>(a, tag, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// Passes of many rows stage both operands through LDS (kernels_gemm_tiled.hip).  Measured against the kernels above at
// the 7B- and 13B-shaped products: it wins from 65 rows up everywhere, and from 25 rows up for products wide enough
// to give every compute unit a workgroup of 8 strips (at 17 rows it loses also with activations that are already in
// fragment order: C4 verify 4.50 against 4.24 ms).
static bool use_tiled(const GemmArgs& a) {
  if (!a.ncg && (!a.xfrag || a.xfrag_elems < gemm_tiled_xfrag_elems(a.R, a.K))) return false;  // needs fragment order or its scratch
  return a.R >= 65 || (a.R >= 25 && gemm_tiled_wide(a.N));
}

hipError_t launch_gemm_bf16(const GemmArgs& a, int epi, int tag, hipStream_t s) {
  if (a.R <= 0) return hipSuccess;
  if ((a.N % 16) || (a.K % 32) || a.R > 256) return hipErrorInvalidValue;
  if (use_tiled(a) && (epi != EPI_STORE || (a.ldy % 4) == 0)) return launch_gemm_bf16_tiled(a, epi, s);
  switch (epi) {
    case EPI_STORE: return (a.ldy % 4) ? hipErrorInvalidValue : run_epi<EPI_STORE>(a, tag, s);
    case EPI_RESID: return run_epi<EPI_RESID>(a, tag, s);
    case EPI_SWIGLU: return run_epi<EPI_SWIGLU>(a, tag, s);
    case EPI_QKV: return run_epi<EPI_QKV>(a, tag, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace mtad
