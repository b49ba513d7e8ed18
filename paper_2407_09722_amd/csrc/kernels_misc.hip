// Row-wise pieces of the decoder pass: embedding gather, RMSNorm (wavefront reductions), the rotary
// table, rotary + KV-cache write, SwiGLU gating and the row-wise logsumexp of the logits.
// All of them move a few KB..MB per launch; they are latency bound, not bandwidth bound.
#include "common.h"

namespace mtad {

__device__ __forceinline__ float wave_sum(float v) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// block-wide reductions for 256-thread blocks; every thread gets the result
__device__ __forceinline__ float block_sum(float v, float* sh) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = sh[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) t += sh[w];
  return t;
}
__device__ __forceinline__ float block_max(float v, float* sh) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = sh[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) t = fmaxf(t, sh[w]);
  return t;
}

// The inputs of a pass, one workgroup per row: h[row] = E[tok[row]]; bf16 models: also planes of h*g0 (input of the
// first fused RMSNorm) and ssq[row] = sum h^2; and the row's rotary table, table[row][i] = (cos, sin)(pos[row] *
// theta^(-2i/head_dim)), evaluated in double so that positions in the thousands keep float32-exact angles.
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T* __restrict__ E, const int32_t* __restrict__ tok, float* __restrict__ h, int d,
                                                    int vocab, const float* __restrict__ g0, bf16_t* __restrict__ planes,
                                                    float* __restrict__ ssq, const int32_t* __restrict__ pos, float2* __restrict__ table,
                                                    int half, float theta, int ncg) {
  __shared__ float sh[4];
  const int row = blockIdx.x;
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    const double inv_freq = pow((double)theta, -(double)i / (double)half);
    const double ang = (double)pos[row] * inv_freq;
    double sn, cs;
    sincos(ang, &sn, &cs);
    table[(int64_t)row * half + i] = make_float2((float)cs, (float)sn);
  }
  int t = tok[row];
  if (t < 0 || t >= vocab) t = 0;  // inactive rows carry no meaningful token
  const T* e = E + (int64_t)t * d;
  float ss = 0.f;
  for (int i = threadIdx.x * 4; i < d; i += blockDim.x * 4) {  // d is a multiple of 4 (checked at create)
    float v[4];
    if constexpr (sizeof(T) == 2) {
      const ushort4 b = *(const ushort4*)(e + i);
      v[0] = bf16_to_f32(b.x); v[1] = bf16_to_f32(b.y); v[2] = bf16_to_f32(b.z); v[3] = bf16_to_f32(b.w);
    } else {
      const float4 f = *(const float4*)(e + i);
      v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
    }
    *(float4*)(h + (int64_t)row * d + i) = make_float4(v[0], v[1], v[2], v[3]);
    if (planes) {
      const float4 g = *(const float4*)(g0 + i);
      ushort4 hi, lo;
      split_bf16(v[0] * g.x, hi.x, lo.x);
      split_bf16(v[1] * g.y, hi.y, lo.y);
      split_bf16(v[2] * g.z, hi.z, lo.z);
      split_bf16(v[3] * g.w, hi.w, lo.w);
      ss += v[0] * v[0];
      ss += v[1] * v[1];
      ss += v[2] * v[2];
      ss += v[3] * v[3];
      *(ushort4*)(planes + act_offset(ncg, (int)gridDim.x, d, 0, row, i)) = hi;
      *(ushort4*)(planes + act_offset(ncg, (int)gridDim.x, d, 1, row, i)) = lo;
    }
  }
  if (planes) {
    ss = block_sum(ss, sh);
    if (threadIdx.x == 0) ssq[row] = ss;
  }
}

hipError_t launch_embed(int dtype, const void* E, const int32_t* tok, float* h, int rows, int d, int vocab, const float* g0,
                        void* planes, float* ssq, const int32_t* pos, float2* table, int head_dim, float theta, int ncg, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dtype == 1)
    hipLaunchKernelGGL((embed_kernel<bf16_t>), dim3(rows), dim3(256), 0, s, (const bf16_t*)E, tok, h, d, vocab, g0, (bf16_t*)planes, ssq, pos,
                       table, head_dim / 2, theta, ncg);
  else
    hipLaunchKernelGGL((embed_kernel<float>), dim3(rows), dim3(256), 0, s, (const float*)E, tok, h, d, vocab, nullptr, nullptr, nullptr, pos,
                       table, head_dim / 2, theta, 0);
  return hipGetLastError();
}

// out[row][i] = h[row][i] / sqrt(mean(h[row]^2) + eps) * g[i]
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ h, const float* __restrict__ g, T* __restrict__ out,
                                                      int d, float eps) {
  __shared__ float sh[4];
  const int row = blockIdx.x;
  const int64_t lo_plane = (int64_t)gridDim.x * d;
  const float* x = h + (int64_t)row * d;
  float ss = 0.f;
  for (int i = threadIdx.x * 4; i < d; i += 1024) {
    const float4 v = *(const float4*)(x + i);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = block_sum(ss, sh);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x * 4; i < d; i += 1024) {
    const float4 v = *(const float4*)(x + i);
    const float4 gg = *(const float4*)(g + i);
    const float o0 = v.x * inv * gg.x, o1 = v.y * inv * gg.y, o2 = v.z * inv * gg.z, o3 = v.w * inv * gg.w;
    if constexpr (sizeof(T) == 2) {
      ushort4 hi, lo;
      split_bf16(o0, hi.x, lo.x);
      split_bf16(o1, hi.y, lo.y);
      split_bf16(o2, hi.z, lo.z);
      split_bf16(o3, hi.w, lo.w);
      *(ushort4*)(out + (int64_t)row * d + i) = hi;
      *(ushort4*)(out + lo_plane + (int64_t)row * d + i) = lo;
    } else {
      *(float4*)(out + (int64_t)row * d + i) = make_float4(o0, o1, o2, o3);
    }
  }
}

hipError_t launch_rmsnorm(int dtype, const float* h, const float* g, void* out, int rows, int d, float eps, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (d % 4) return hipErrorInvalidValue;
  if (dtype == 1) hipLaunchKernelGGL((rmsnorm_kernel<bf16_t>), dim3(rows), dim3(256), 0, s, h, g, (bf16_t*)out, d, eps);
  else hipLaunchKernelGGL((rmsnorm_kernel<float>), dim3(rows), dim3(256), 0, s, h, g, (float*)out, d, eps);
  return hipGetLastError();
}

// grid (rows, n_heads + 2*n_kv_heads), block head_dim/2.  q heads: rotated in place (float32).
// k heads: rotated and stored to the cache in its storage type; v heads: stored to the cache.
template <typename T>
__global__ void rope_kv_kernel(float* __restrict__ qkv, const float2* __restrict__ table, RowDesc rd, KvView kv, int layer, int R,
                               int n_heads, uint32_t* __restrict__ status) {
  const int row = blockIdx.x, head = blockIdx.y, i = threadIdx.x;
  const int hd = kv.head_dim, half = hd >> 1, KVH = kv.n_kv_heads;
  const int width = (n_heads + 2 * KVH) * hd;
  float* p = qkv + (int64_t)row * width + (int64_t)head * hd;
  const float x1 = p[i], x2 = p[i + half];
  const float2 cs = table[(int64_t)row * half + i];
  if (head < n_heads) {
    p[i] = x1 * cs.x - x2 * cs.y;
    p[i + half] = x2 * cs.x + x1 * cs.y;
    return;
  }
  const int slot = rd.slot[row];
  if (slot < 0) return;
  if (slot >= kv_capacity(kv)) {
    if (i == 0) atomicOr(status, (uint32_t)ST_KV_CAP);
    return;
  }
  const int seq = row / R;
  const bool is_k = head < n_heads + KVH;
  const int g = is_k ? head - n_heads : head - n_heads - KVH;
  const int64_t off = (int64_t)layer * kv.layer_stride + kv_token_offset(kv, seq, slot) + (int64_t)g * hd;
  T* dst = (T*)(is_k ? kv.k : kv.v) + off;
  float y1 = x1, y2 = x2;
  if (is_k) { y1 = x1 * cs.x - x2 * cs.y; y2 = x2 * cs.x + x1 * cs.y; }
  dst[i] = (T)y1;
  dst[i + half] = (T)y2;
}

hipError_t launch_rope_kv(int dtype, float* qkv, const float2* table, const RowDesc& rd, KvView kv, int layer, int B, int R,
                          int n_heads, uint32_t* status, hipStream_t s) {
  const int rows = B * R;
  if (rows <= 0) return hipSuccess;
  dim3 grid(rows, n_heads + 2 * kv.n_kv_heads), block(kv.head_dim / 2);
  if (dtype == 1) return hipErrorInvalidValue;  // bf16 models rotate and store in the QKV product's epilogue
  else hipLaunchKernelGGL((rope_kv_kernel<float>), grid, block, 0, s, qkv, table, rd, kv, layer, R, n_heads, status);
  return hipGetLastError();
}

// act[row][j] = silu(gu[row][j]) * gu[row][f + j]
template <typename T>
__global__ void silu_mul_kernel(const float* __restrict__ gu, T* __restrict__ act, int rows, int f) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)rows * f) return;
  const int row = (int)(idx / f), j = (int)(idx % f);
  const float g = gu[(int64_t)row * 2 * f + j], u = gu[(int64_t)row * 2 * f + f + j];
  const float a = g / (1.0f + expf(-g)) * u;
  if constexpr (sizeof(T) == 2) split_bf16(a, act[idx], act[(int64_t)rows * f + idx]);
  else act[idx] = a;
}

hipError_t launch_silu_mul(int dtype, const float* gu, void* act, int rows, int f, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  const int64_t n = (int64_t)rows * f;
  const int blocks = (int)((n + 255) / 256);
  if (dtype == 1) hipLaunchKernelGGL((silu_mul_kernel<bf16_t>), dim3(blocks), dim3(256), 0, s, gu, (bf16_t*)act, rows, f);
  else hipLaunchKernelGGL((silu_mul_kernel<float>), dim3(blocks), dim3(256), 0, s, gu, (float*)act, rows, f);
  return hipGetLastError();
}

// lse[row] = log(sum_v exp(logits[row][v])), max-shifted; one block per row
__global__ __launch_bounds__(256) void row_lse_kernel(const float* __restrict__ logits, float* __restrict__ lse, int vocab) {
  __shared__ float sh[4];
  const float* x = logits + (int64_t)blockIdx.x * vocab;
  float m = -INFINITY;
  for (int i = threadIdx.x; i < vocab; i += 256) m = fmaxf(m, x[i]);
  m = block_max(m, sh);
  float sum = 0.f;
  for (int i = threadIdx.x; i < vocab; i += 256) sum += expf(x[i] - m);
  sum = block_sum(sum, sh);
  if (threadIdx.x == 0) lse[blockIdx.x] = m + logf(sum);
}

hipError_t launch_row_lse(const float* logits, float* lse, int rows, int vocab, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(row_lse_kernel, dim3(rows), dim3(256), 0, s, logits, lse, vocab);
  return hipGetLastError();
}

// lse[row] = log sum exp over the row from per-strip partials (max, sum exp), merged in strip order
__global__ __launch_bounds__(256) void lse_finish_kernel(const float2* __restrict__ part, float* __restrict__ lse, int NP) {
  __shared__ float sh[4];
  const float2* p = part + (int64_t)blockIdx.x * NP;
  float m = -INFINITY;
  for (int i = threadIdx.x; i < NP; i += 256) m = fmaxf(m, p[i].x);
  m = block_max(m, sh);
  float sum = 0.f;
  for (int i = threadIdx.x; i < NP; i += 256) sum += p[i].y * expf(p[i].x - m);
  sum = block_sum(sum, sh);
  if (threadIdx.x == 0) lse[blockIdx.x] = m + logf(sum);
}

// The same, fused with the gather of the tree nodes' conditional log-likelihoods: workgroup (sequence s, row c) writes
// lse[s][c] and, for c > 0, logp_cond[s][c] = logits[s][parent(c)][tok(c)] - lse[s][parent(c)], reducing the
// parent row's partials itself (same code, same order: the value equals the one the parent's workgroup writes).
__device__ __forceinline__ float lse_of_row(const float2* __restrict__ p, int NP, float* sh) {
  float m = -INFINITY;
  for (int i = threadIdx.x; i < NP; i += 256) m = fmaxf(m, p[i].x);
  m = block_max(m, sh);
  float sum = 0.f;
  for (int i = threadIdx.x; i < NP; i += 256) sum += p[i].y * expf(p[i].x - m);
  sum = block_sum(sum, sh);
  return m + logf(sum);
}

__global__ __launch_bounds__(256) void lse_gather_kernel(const float2* __restrict__ part, float* __restrict__ lse, int NP,
                                                         const float* __restrict__ logits, int M, int V, const int32_t* __restrict__ parent,
                                                         const int32_t* __restrict__ tok, float* __restrict__ logp_cond) {
  __shared__ float sh[4];
  const int idx = blockIdx.x, s = idx / M, c = idx % M;
  const float own = lse_of_row(part + (int64_t)idx * NP, NP, sh);
  if (threadIdx.x == 0) lse[idx] = own;
  float out = 0.f;
  if (c > 0) {  // uniform over the workgroup
    const int p = parent[idx], t = tok[idx];
    if (p >= 0 && p < M && t >= 0 && t < V) {
      __syncthreads();  // sh is reused
      const float lp = lse_of_row(part + ((int64_t)s * M + p) * NP, NP, sh);
      out = logits[((int64_t)s * M + p) * V + t] - lp;
    }
  }
  if (threadIdx.x == 0) logp_cond[idx] = out;
}

hipError_t launch_lse_gather(const float* lse_part, float* lse, int B, int M, int NP, const float* logits, int V, const int32_t* parent,
                             const int32_t* tok, float* logp_cond, hipStream_t s) {
  if (B * M <= 0) return hipSuccess;
  hipLaunchKernelGGL(lse_gather_kernel, dim3(B * M), dim3(256), 0, s, (const float2*)lse_part, lse, NP, logits, M, V, parent, tok, logp_cond);
  return hipGetLastError();
}

hipError_t launch_lse_finish(const float* lse_part, float* lse, int rows, int NP, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(lse_finish_kernel, dim3(rows), dim3(256), 0, s, (const float2*)lse_part, lse, NP);
  return hipGetLastError();
}

// Plain streaming copy of n 16-byte words: the reference point for hardware byte counters (it reads and writes
// exactly 16*n bytes) and for the bandwidth a trivially coalesced kernel reaches.
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

hipError_t launch_copy(const void* src, void* dst, int64_t bytes, hipStream_t s) {
  const int64_t n = bytes / 16;
  if (n <= 0) return hipSuccess;
  const int64_t want = (n + 255) / 256;
  const int blocks = (int)(want < 256 * 16 ? want : 256 * 16);
  hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n);
  return hipGetLastError();
}

}  // namespace mtad
