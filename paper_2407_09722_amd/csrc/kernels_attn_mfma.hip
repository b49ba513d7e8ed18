// Tree-masked paged attention for bf16 models (half-precision K/V cache), few query rows per sequence
// (Section 3.3: tree attention gives every tree token its conditional likelihood in one pass): the stand-alone kernels.
// The work item itself (tile loop on the matrix cores, online softmax, merge of the waves) is in attn_mfma_device.h.
//
// Work item = (key split, KV head, chunk of 16 or 32 (query head, row) pairs, sequence) = one workgroup of AW waves (4 in
// all configurations used; 8 measured no faster).  A context of fewer than 2 x waves x 32 keys is one workgroup,
// which writes the attention output itself: no exchange through global memory.  Longer contexts are cut into splits
// (at least one tile per wave each, at most as many as fill the machine once, or every resident slot where once is an
// uneven fill); every split leaves (max, sum, output)
// per row in global memory (same partial layout as the generic kernel) and a small second kernel, one wave per row,
// merges them in split order.
#include "attn_mfma_device.h"
#include "common.h"

#include <type_traits>

namespace mtad {

namespace {

template <int HD, int NRG, int AW>
__global__ __launch_bounds__(AW * 64) __attribute__((amdgpu_waves_per_eu(2))) void tree_attn_mfma_kernel(const float* __restrict__ q, int q_stride, RowDesc rd, KvView kv, int layer,
                                                               int R, int n_heads, int n_chunks, float scale, float* __restrict__ partial,
                                                               int n_splits, bf16_t* __restrict__ out, int want_splits, int ncg) {
  using Smem = MfmaAttnSmem<HD, NRG, AW>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];  // dynamic: an 8-wave variant needs more than 64 KiB
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
  // the kernels with registers to spare (head dim 64, or a single row group) hold two register sets for K and V
  constexpr int NSET = (HD == 64 || NRG == 1) ? 2 : 1;
  tree_attn_item<HD, NRG, AW, NSET, AW * 64, false>(sm, q, q_stride, rd, kv, layer, (int)gridDim.z, R, n_heads, n_chunks, scale, partial, n_splits,
                                                   out, want_splits, ncg, (int)blockIdx.x, (int)blockIdx.y / n_chunks, (int)blockIdx.y % n_chunks,
                                                   (int)blockIdx.z, (int)threadIdx.x);
}

// Merge of the key splits, a kernel of its own: one wave per (sequence, query head, row).  As a separate launch it is
// spread over the whole machine and costs about the same for any number of
// splits, where the last workgroup of an item merging inside the attention kernel (the first design: 3.3 us of 13.1 at
// 4 splits and 5 rows, 8 us of 28 at 8 splits and 17 rows) made more splits cost more than they gained.
template <int HD>
__global__ __launch_bounds__(256) void attn_merge_kernel(RowDesc rd, KvView kv, int B, int R, int n_heads, const float* __restrict__ partial,
                                                         int n_splits, int want_splits, bf16_t* __restrict__ out, int ncg) {
  const int lane = threadIdx.x & 63;
  const int item = blockIdx.x * 4 + (threadIdx.x >> 6);  // (seq, head, row)
  if (item >= B * n_heads * R) return;
  const int row = item % R, head = (item / R) % n_heads, seq = item / (R * n_heads);
  const int eff = attn_splits(attn_keys(kv, rd, seq), n_splits, want_splits);
  if (eff == 1) return;  // the attention kernel wrote the output itself
  const float* pp = partial + (((int64_t)seq * n_heads + head) * R + row) * n_splits * (HD + 2);
  attn_merge_row<HD, false>(pp, eff, out, ncg, B * R, n_heads * HD, seq * R + row, head, lane);
}

template <int HD, int NRG, int AW>
hipError_t run_mfma(const float* q, int q_stride, const RowDesc& rd, const KvView& kv, int layer, int B, int R, int n_heads, float* partial,
                    int n_splits, void* out, int ncg, hipStream_t s) {
  const int KVH = kv.n_kv_heads, G = n_heads / KVH;
  const int n_chunks = (G * R + NRG * 16 - 1) / (NRG * 16);  // chunks of (query head, row) pairs per KV head
  const float scale = 1.0f / sqrtf((float)HD);
  auto kern = tree_attn_mfma_kernel<HD, NRG, AW>;
  constexpr size_t lds = sizeof(MfmaAttnSmem<HD, NRG, AW>);
  static const hipError_t attr = lds > 64 * 1024 ? hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                                                 : hipSuccess;
  if (attr != hipSuccess) return attr;
  // splits: enough workgroups to fill the machine once (twice and four times over measured no faster at 512, 2048 and 4096
  // keys when once is an even fill)
  static const int n_cus = [] {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
    return cus > 0 ? cus : 256;
  }();
  const int items = KVH * n_chunks * B;
  const int fill = items >= n_cus ? 1 : (n_cus + items - 1) / items;
  // an uneven fill (C5's target pass: 160 items x 2 splits on 256 compute units) runs as long as the compute units that
  // hold two workgroups; splits up to the number of resident slots shorten every workgroup instead (41 rows x 40 heads x
  // 4 sequences at 4096 keys: 99 -> 80 us with 3 splits)
  static const int per_cu = [&] {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, (const void*)kern, AW * 64, lds) != hipSuccess) n = 1;
    return n > 0 ? n : 1;
  }();
  const int more = (items * fill > n_cus && per_cu >= 2) ? (n_cus * per_cu) / items : 0;
  const int fill8 = fill < 255 ? fill : 255, more8 = more < 255 ? more : 255;
  const int want = fill8 | (more8 << 8);
  const int widest = fill8 > more8 ? fill8 : more8;
  const int gx = n_splits < widest ? n_splits : widest;
  hipLaunchKernelGGL(kern, dim3(gx, KVH * n_chunks, B), dim3(AW * 64), lds, s, q, q_stride, rd, kv, layer, R, n_heads, n_chunks, scale,
                     partial, n_splits, (bf16_t*)out, want, ncg);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || gx == 1) return e;  // one split: every workgroup wrote its output
  hipLaunchKernelGGL((attn_merge_kernel<HD>), dim3((B * n_heads * R + 3) / 4), dim3(256), 0, s, rd, kv, B, R, n_heads, (const float*)partial,
                     n_splits, want, (bf16_t*)out, ncg);
  return hipGetLastError();
}

}  // namespace


// bf16 models: q float32 [B*R][q_stride], half-precision cache, output = bf16 hi / lo planes [2][B*R][n_heads*hd].
// Passes of up to 16 rows per sequence use 16-row work items, larger ones 32-row items (K and V are read once per item).
hipError_t launch_attention_mfma(const float* q, int q_stride, const RowDesc& rd, KvView kv, int layer, int B, int R, int n_heads,
                                 float* partial, int n_splits, void* out, int ncg, hipStream_t s) {
  const int hd = kv.head_dim;
  if (kv.n_kv_heads < 1 || n_heads % kv.n_kv_heads) return hipErrorInvalidValue;
  const int pairs = n_heads / kv.n_kv_heads * R;  // (query head, row) pairs that share a KV head
  if (hd == 128 && pairs <= 16) return run_mfma<128, 1, 4>(q, q_stride, rd, kv, layer, B, R, n_heads, partial, n_splits, out, ncg, s);
  if (hd == 128 && pairs > 32 && pairs <= 48)  // one item instead of two that would each read K and V
    return run_mfma<128, 3, 4>(q, q_stride, rd, kv, layer, B, R, n_heads, partial, n_splits, out, ncg, s);
  if (hd == 128) return run_mfma<128, 2, 4>(q, q_stride, rd, kv, layer, B, R, n_heads, partial, n_splits, out, ncg, s);
  if (hd == 64 && pairs <= 16) return run_mfma<64, 1, 4>(q, q_stride, rd, kv, layer, B, R, n_heads, partial, n_splits, out, ncg, s);
  if (hd == 64) return run_mfma<64, 2, 4>(q, q_stride, rd, kv, layer, B, R, n_heads, partial, n_splits, out, ncg, s);
  return hipErrorInvalidValue;
}

}  // namespace mtad
