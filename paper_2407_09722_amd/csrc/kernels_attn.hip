// Tree-masked paged attention for the rows of one pass (Section 3.3: tree attention gives every tree
// token its conditional likelihood in one pass).  Every row sees the whole committed cache of its
// sequence plus the speculative rows named in its ancestor mask.
//
// Split-KV "flash decoding": grid = (key split, head x row chunk, sequence).  A workgroup stages 64-key
// K and V tiles in LDS once and reuses them for its (up to 16) query rows, keeps running max / sum /
// output per row, and writes one partial per split; the workgroup that finishes last for a (sequence, head,
// row chunk) merges the partials in split order (deterministic) and writes the attention output, so no second
// kernel is needed.  Everything is float32 arithmetic; K/V are read in their storage type (half or float32).
#include "attn_device.h"
#include "common.h"

#include <stdlib.h>

namespace mtad {

template <typename T, typename OutT, int HD, int NTHR>
__global__ __launch_bounds__(NTHR) void tree_attn_kernel(const float* __restrict__ q, int q_stride, RowDesc rd, KvView kv, int layer,
                                                        int R, int n_heads, int n_chunks, float scale, float* __restrict__ partial,
                                                        int n_splits, int* __restrict__ counters, OutT* __restrict__ out) {
  __shared__ AttnSmem<T, HD, NTHR> sm;
  attn_item<T, OutT, HD, NTHR>(sm, q, q_stride, rd, kv, layer, gridDim.z, R, n_heads, n_chunks, scale, partial, n_splits, counters, out,
                              blockIdx.x, blockIdx.y / n_chunks, blockIdx.y % n_chunks, blockIdx.z);
}

size_t attention_partial_floats(int B, int R, int n_heads, int head_dim, int n_splits) {
  return (size_t)B * R * n_heads * n_splits * (head_dim + 2);
}

template <typename T, int HD>
static hipError_t run_attn(const float* q, int q_stride, const RowDesc& rd, KvView kv, int layer, int B, int R, int n_heads,
                           float* partial, int n_splits, int* counters, void* out, hipStream_t s) {
  using OutT = typename std::conditional<sizeof(T) == 2, bf16_t, float>::type;  // bf16 hi/lo planes or float32
  const int n_chunks = (R + RB - 1) / RB;
  const float scale = 1.0f / sqrtf((float)HD);
  hipLaunchKernelGGL((tree_attn_kernel<T, OutT, HD, 256>), dim3(n_splits, n_heads * n_chunks, B), dim3(256), 0, s, q, q_stride, rd,
                       kv, layer, R, n_heads, n_chunks, scale, partial, n_splits, counters, (OutT*)out);
  return hipGetLastError();
}

hipError_t launch_attention(int dtype, const float* q, int q_stride, const RowDesc& rd, KvView kv, int layer, int B, int R, int n_heads,
                            float* partial, int n_splits, int* counters, void* out, int ncg, hipStream_t s) {
  if (B * R <= 0) return hipSuccess;
  const int hd = kv.head_dim;
  if (dtype == 1) return launch_attention_mfma(q, q_stride, rd, kv, layer, B, R, n_heads, partial, n_splits, out, ncg, s);
  if (dtype == 0 && hd == 128) return run_attn<float, 128>(q, q_stride, rd, kv, layer, B, R, n_heads, partial, n_splits, counters, out, s);
  if (dtype == 0 && hd == 64) return run_attn<float, 64>(q, q_stride, rd, kv, layer, B, R, n_heads, partial, n_splits, counters, out, s);
  return hipErrorInvalidValue;
}

}  // namespace mtad
