// Arguments and launchers of the skinny matrix products (kernels_gemm.hip).
#pragma once
#include "common.h"

namespace mtad {

enum { PACK_PLAIN = 0, PACK_QKV = 1, PACK_GATE_UP = 2 };
enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_QKV = 3 };

struct GemmArgs {
  const bf16_t* W;   // tile-packed [N/16][K/32][64 lanes][8]
  const bf16_t* X;   // activation = hi + lo, two bf16 terms: planes [2][R][K] (ncg == 0) or operand-fragment order (act_offset)
  int R, N, K;
  int ncg;           // 0, or ceil(R / 8): X, planes_out and act_out are in operand-fragment order
  int row0;          // first row handled by this launch (set by the launcher; 64 rows per launch)
  // rows are multiplied by 1/sqrt(sum_p ssq[m][p] / K + eps) when ssq != null (fused RMSNorm of the input)
  const float* ssq;
  int NP;
  float eps;
  // EPI_STORE
  float* Y;
  int ldy;
  int accumulate;
  float* lse_part;   // float2 [R][N/16] (max, sum exp) per strip, or null
  // EPI_RESID: h += product; planes_out = split(h * g_next); ssq_out[R][N/16] = per-strip sums of h^2
  float* h;
  const float* g_next;
  bf16_t* planes_out;
  float* ssq_out;
  // EPI_SWIGLU: act_out planes [2][R][N/2]
  bf16_t* act_out;
  // EPI_QKV: rotary rotation of q and k, q to q_out [R][n_heads*head_dim] (float32), k / v to the cache
  float* q_out;
  const float2* rope;   // [R][head_dim/2] (cos, sin)
  const int32_t* slot;  // [R] logical cache position of each row, -1 = do not store
  KvView kv;
  int layer, Rseq, n_heads;
  uint32_t* status;
  // k split across workgroups (products with few strips and more than 8 rows): partial sums [group][strip][row group][split]
  // of 256 floats, and one zeroed counter per group (left zeroed); null = no split
  float* part;
  int* counters;
  size_t part_floats;  // capacity of `part` in floats and of `counters` in ints: a launch that would need more does not split
  int counters_n;
  // scratch for the many-row kernel: the pass's activations rewritten in B-operand fragment order; null = not offered
  // (such products then run on the skinny kernels)
  bf16_t* xfrag;
  size_t xfrag_elems;
};

hipError_t launch_gemm_bf16(const GemmArgs& a, int epi, int tag, hipStream_t s);
// the same product for passes of many rows, activations staged through LDS (kernels_gemm_tiled.hip); chosen by launch_gemm_bf16
hipError_t launch_gemm_bf16_tiled(const GemmArgs& a, int epi, hipStream_t s);
bool gemm_tiled_wide(int N);  // enough strips for workgroups of 8
size_t gemm_tiled_split_floats(int N);
size_t gemm_tiled_xfrag_elems(int R, int K);  // scratch elements a product with R rows and reduction width K wants
int gemm_tiled_split_counters(int N);
// workspace a context should offer for the k split of a product with N outputs (0 if it would never be split)
size_t gemm_split_floats(int N);
int gemm_split_counters(int N);
hipError_t launch_gemm_f32(const void* W, const void* X, float* Y, int R, int N, int K, int ldy, bool accumulate, hipStream_t s);
hipError_t launch_pack_matrix(const void* src, void* dst, int N, int K, int kind, int head_dim, hipStream_t s);

}  // namespace mtad
