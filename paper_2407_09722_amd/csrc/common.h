// Internal declarations shared by the kernel files and the C-ABI layer of libmtad.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mtad {

typedef uint16_t bf16_t;  // bfloat16 bit pattern
typedef _Float16 kv16_t;  // storage type of the KV cache of a bfloat16 model: IEEE half (3 more mantissa bits at the same size)

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// float32 -> bfloat16, round to nearest even (NaN not expected on this path)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float round_bf16(float f) { return bf16_to_f32(f32_to_bf16(f)); }
// Two-term bfloat16 split of a float32 activation: x ~= hi + lo with a relative error of about 2^-17.
// Matrix-product inputs are carried this way so that their rounding stays far below the weights' own.
__device__ __forceinline__ void split_bf16(float x, bf16_t& hi, bf16_t& lo) {
  hi = f32_to_bf16(x);
  lo = f32_to_bf16(x - bf16_to_f32(hi));
}

// Element offset of activation (plane, row, feature k) of a pass of R rows and K features.  ncg == 0: two planes
// [2][R][K].  ncg > 0 (= ceil(R / 8)): operand-fragment order, the B operand of v_mfma_f32_16x16x32_bf16 for 8 rows at a
// time, where lane (k%32)/8 * 16 + plane * 8 + row % 8 holds 8 consecutive features of fragment (k / 32, row / 8):
//   R > 24   [K/32][ncg][64 lanes][8]: whole fragments, the slots of rows past R unused (the many-row kernel copies
//            them to LDS line by line);
//   R <= 24  [K/32][4 k groups][2 planes][R rows][8]: the same order with the unused row slots left out: a k tile's
//            fragments are 128 R contiguous bytes (5 cache lines at 5 rows instead of 8, 17 at 17 rows instead of 24);
//            row group g of a (k group, plane) block starts 128 g bytes into it.
// Products read this order (whole cache lines per fragment instead of 64-byte pieces of 16 rows); whatever produces
// their input writes it.
constexpr int ACT_COMPACT_ROWS = 24;  // passes of up to this many rows leave the unused row slots out
__host__ __device__ __forceinline__ int64_t act_offset(int ncg, int R, int K, int plane, int row, int k) {
  if (ncg == 0) return ((int64_t)plane * R + row) * K + k;
  if (R <= ACT_COMPACT_ROWS) return ((((int64_t)(k >> 5) * 4 + ((k >> 3) & 3)) * 2 + plane) * R + row) * 8 + (k & 7);
  return ((((int64_t)(k >> 5) * ncg + (row >> 3)) * 64 + ((k >> 3) & 3) * 16 + plane * 8 + (row & 7)) << 3) + (k & 7);
}

// Device-scope ("coherent") accesses for data that workgroups of ONE kernel hand to each other.  The XCDs' L2
// caches are not coherent with each other; relaxed device-scope atomics compile to write-through stores and
// cache-bypassing loads, which avoids flushing or invalidating whole caches.  COH = false: plain accesses (data
// produced by an earlier kernel).
template <bool COH>
__device__ __forceinline__ uint4 ld16(const void* p) {
  if constexpr (COH) {
    const unsigned long long* q = (const unsigned long long*)p;
    const unsigned long long a = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long b = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_uint4((uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32));
  } else {
    return *(const uint4*)p;
  }
}
template <bool COH>
__device__ __forceinline__ float ld4(const float* p) {
  if constexpr (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return *p;
}
template <bool COH>
__device__ __forceinline__ void st8(void* p, uint2 v) {
  if constexpr (COH)
    __hip_atomic_store((unsigned long long*)p, (unsigned long long)v.x | ((unsigned long long)v.y << 32), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
  else
    *(uint2*)p = v;
}
template <bool COH>
__device__ __forceinline__ void st4(float* p, float v) {
  if constexpr (COH) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = v;
}

// Device status bits (sticky, OR-ed by kernels that refuse an out-of-range access)
enum : uint32_t { ST_KV_CAP = 1u, ST_SPEC_WINDOW = 2u, ST_BAD_CATCHUP = 4u, ST_TIMEOUT = 8u };

// Paged KV addressing: element offset of (layer, logical position pos, kv head 0, dim 0)
struct KvView {
  void* k;
  void* v;
  const int32_t* page_table;  // [B][max_pages]
  int32_t* len;               // [B]
  int32_t page_size, max_pages, n_pages;
  int32_t n_kv_heads, head_dim;
  int64_t layer_stride;  // elements per layer = n_pages*page_size*n_kv_heads*head_dim
};

__device__ __forceinline__ int64_t kv_token_offset(const KvView& kv, int seq, int pos) {
  int page = kv.page_table[(int64_t)seq * kv.max_pages + pos / kv.page_size];
  return ((int64_t)page * kv.page_size + pos % kv.page_size) * kv.n_kv_heads * kv.head_dim;
}
__device__ __forceinline__ int kv_capacity(const KvView& kv) { return kv.page_size * kv.max_pages; }

// Row descriptors of one pass (R rows per sequence, B sequences), device arrays in the workspace
struct RowDesc {
  int32_t* tok;    // [B*R] token id of the row
  int32_t* pos;    // [B*R] rotary position
  int32_t* slot;   // [B*R] logical KV position the row's K/V are written to, -1 = inactive row
  uint64_t* mask;  // [B*R] visible speculative slots: bit j <=> logical position len+j
  int32_t* nspec;  // [B]   speculative slots in use after this pass (keys len .. len+nspec-1 exist)
};

// ---- launchers (kernels_*.hip) ----------------------------------------------------------------
// h = E[tok]; bf16 models also get the first RMSNorm's input: h*g0 as two bf16 terms (layout: act_offset with ncg) and ssq[rows] = sum h^2;
// and the rotary table of the rows' positions, table[rows][head_dim/2] = (cos, sin)
hipError_t launch_embed(int dtype, const void* E, const int32_t* tok, float* h, int rows, int d, int vocab, const float* g0,
                        void* planes, float* ssq, const int32_t* pos, float2* table, int head_dim, float theta, int ncg, hipStream_t s);
// out = rmsnorm(h) * g, written as hi/lo bf16 planes [2][rows][d] (dtype 1) or f32 [rows][d] (dtype 0)
hipError_t launch_rmsnorm(int dtype, const float* h, const float* g, void* out, int rows, int d, float eps, hipStream_t s);
// rotate q (in place in qkv, float32), rotate k and write k, v to the cache in its storage type
hipError_t launch_rope_kv(int dtype, float* qkv, const float2* table, const RowDesc& rd, KvView kv, int layer, int B, int R,
                          int n_heads, uint32_t* status, hipStream_t s);
// q: [rows][q_stride] float32 with head h at column h*head_dim; counters: zeroed ints [B][n_heads][ceil(R/16)], used by
// the float32 kernel only (its last workgroup per item merges the key splits; bf16 models merge in a kernel of their own)
hipError_t launch_attention(int dtype, const float* q, int q_stride, const RowDesc& rd, KvView kv, int layer, int B, int R, int n_heads,
                            float* partial, int n_splits, int* counters, void* out, int ncg, hipStream_t s);
// bf16 models (kernels_attn_mfma.hip): half-precision cache, output = bf16 hi / lo terms (layout: act_offset with ncg);
// n_splits = upper bound on the key splits (the kernel uses fewer for short contexts)
hipError_t launch_attention_mfma(const float* q, int q_stride, const RowDesc& rd, KvView kv, int layer, int B, int R, int n_heads,
                                 float* partial, int n_splits, void* out, int ncg, hipStream_t s);
// lse[row] from per-strip (max, sum exp) partials [rows][NP]
hipError_t launch_lse_finish(const float* lse_part, float* lse, int rows, int NP, hipStream_t s);
// lse as above for B*M rows, plus logp_cond[s][c] = logits[s][parent(c)][tok(c)] - lse[s][parent(c)] (0 for c = 0)
hipError_t launch_lse_gather(const float* lse_part, float* lse, int B, int M, int NP, const float* logits, int V, const int32_t* parent,
                             const int32_t* tok, float* logp_cond, hipStream_t s);
hipError_t launch_silu_mul(int dtype, const float* gu, void* act, int rows, int f, hipStream_t s);
hipError_t launch_copy(const void* src, void* dst, int64_t bytes, hipStream_t s);
hipError_t launch_row_lse(const float* logits, float* lse, int rows, int vocab, hipStream_t s);

size_t attention_partial_floats(int B, int R, int n_heads, int head_dim, int n_splits);

}  // namespace mtad
