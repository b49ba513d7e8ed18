// The persistent decoder pass: all layers of one pass (and the lm_head) in ONE kernel launch (kernels_pass.hip).
#pragma once
#include "common.h"

namespace mtad {

constexpr int PASS_MAX_LAYERS = 60;
constexpr int PASS_MAX_ROWS = 32;  // rows (all sequences together) the persistent kernel takes

// What the kernel does between two grid barriers.  The step list of a model lives in device memory, is written
// by the host before the launch, and is read by the kernel with scalar loads, one step at a time.
enum : int { STEP_QKV = 0, STEP_ATTN = 1, STEP_O = 2, STEP_GATE_UP = 3, STEP_DOWN = 4, STEP_HEAD = 5 };

struct PassStep {
  const void* W;        // tile-packed weights of a product step
  const float* g_next;  // O / DOWN: gains of the RMSNorm that follows
  const bf16_t* X;      // product steps: input planes [2][rows][K]
  bf16_t* out;          // planes this step writes (ATTN, O, GATE_UP, DOWN)
  int kind;
  int N, K;   // output features, reduction width of a product step
  int layer;
  int next;   // index of the next product step (its first weight tiles are prefetched), -1 = none
  int np;     // QKV / GATE_UP / HEAD: partial sums of squares per row left by the producer of the input
  int pad[2];
};
static_assert(sizeof(PassStep) == 64, "PassStep is read as a 64-byte record");

constexpr int pass_steps(int n_layers, bool head) { return 5 * n_layers + (head ? 1 : 0); }

// Activation planes of one pass.  Every buffer is written by exactly one step and read by the next product step, and
// no two steps of a pass share a buffer: a workgroup therefore never holds a stale cached copy of a line it reads
// (the caches start clean at every launch), and the planes can be read with ordinary cached loads.
// Layout: x0 = planes of embedding*gain (written before the launch); then per layer
// [attention output | h*g_ffn | FFN activation | h*g_next], each [2][max_rows][width] bf16.
constexpr size_t pass_act_elems_per_layer(int d, int hhd, int f, int max_rows) { return (size_t)2 * max_rows * ((size_t)hhd + d + f + d); }

// Fills steps[0 .. pass_steps(n_layers, true)) from a model's weight list (order of mtad_model.weights); host code.
void pass_build_steps(PassStep* steps, const void* const* weights, int n_layers, int d, int f, int H, int KVH, int hd, int vocab,
                      const bf16_t* x0, bf16_t* act, int max_rows);

struct PassArgs {
  const PassStep* steps;
  int n_steps;  // pass_steps(n_layers, with or without the lm_head)
  int d, f, H, KVH, hd, vocab;
  int rows, Rseq, B, n_splits;
  float eps;
  KvView kv;
  RowDesc rd;
  float* h;         // [rows][d] residual stream (already holds the embeddings)
  float* ssq;       // per-strip sums of squares (already holds the embeddings': 1 partial per row)
  float* q;         // [rows][H*hd]
  const float2* rope;
  float* partial;   // attention split partials
  int* attn_cnt;
  float* logits;    // [rows][vocab] (when the step list ends with the lm_head)
  float* lse_part;  // float2 [rows][vocab/16]
  uint32_t* status;
  unsigned long long* bar;  // grid barrier counter, zero at launch; bar[1] = abort flag
#ifdef MTAD_PASS_PROFILE
  unsigned long long* prof;  // [3 workgroups][512 steps][3] timestamps (development builds only)
#endif
};

// rows <= PASS_MAX_ROWS, bf16 model.  grid = number of compute units.  dev_args: device memory for one PassArgs, which
// a small kernel fills on the stream just before the pass (it also zeroes the barrier).
hipError_t launch_pass(const PassArgs& a, PassArgs* dev_args, int n_cus, hipStream_t s);
bool pass_supported(int rows, int n_layers);

}  // namespace mtad
