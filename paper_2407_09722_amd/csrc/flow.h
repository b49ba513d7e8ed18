// The one-launch decoder pass for bf16 models with few rows (kernels_flow.hip): every product and the attention of
// every layer as work units of ONE kernel: numbered in dependency order, workgroup b of G runs units b, b + G, ...
#pragma once
#include "common.h"

namespace mtad {

constexpr int FLOW_MAX_LAYERS = 48;  // weight pointers travel in the kernel arguments
constexpr int FLOW_MAX_ROWS = 8;     // rows of a pass (all sequences together): one row group of the product kernels
constexpr int FLOW_NS = 5 * FLOW_MAX_LAYERS + 2;

// Steps of a pass: layer l is steps 5l .. 5l+4 (QKV product, attention, o product, gate/up product, down product), the
// lm_head is step 5 * n_layers.  Every unit of a step needs every unit of the step before it.
enum : int { FK_QKV = 0, FK_ATTN = 1, FK_O = 2, FK_GU = 3, FK_DOWN = 4, FK_HEAD = 5 };

// Synchronisation words of a pass (device ints, zeroed before the pass's first launch).  Read-modify-write operations
// that workgroups on different XCDs aim at ONE address are served one after the other, some tens of nanoseconds each, and
// a pass has tens of thousands of units: a single counter of finished units per step (or a ticket counter) costs more
// than the whole weight stream.  So a step's finished units are counted in FLOW_SHARDS counters, each in a cache line of
// its own (unit u counts in shard u % FLOW_SHARDS); the unit that completes a shard counts it in the step's top counter,
// and the unit that completes that one raises the step's flag, FLOW_FLAGS copies of it in lines of their own, of which a
// waiting workgroup polls the one its index selects.
//   [0]                                         abort flag (a bounded wait gave up: nobody waits any more)
//   [8 + s]                                     top counter of step s: complete shards
//   [FLOW_SHARD_BASE + (s * FLOW_SHARDS + j) * 32]   shard j of step s: finished units
//   [FLOW_FLAG_BASE + (s * FLOW_FLAGS + c) * 32]     copy c of the flag "step s is complete"
//   [FLOW_ITEM_BASE + item]                     attention: splits of item (sequence, KV head, chunk) that have left their partial results
constexpr int FLOW_SHARDS = 16, FLOW_FLAGS = 8;
constexpr int FLOW_SHARD_BASE = 256;
static_assert(8 + FLOW_NS <= FLOW_SHARD_BASE, "top counters fit below the shards");
constexpr int FLOW_FLAG_BASE = FLOW_SHARD_BASE + FLOW_NS * FLOW_SHARDS * 32;
constexpr int FLOW_ITEM_BASE = FLOW_FLAG_BASE + FLOW_NS * FLOW_FLAGS * 32;
constexpr int flow_sync_ints(int max_items) { return FLOW_ITEM_BASE + max_items; }

struct FlowArgs {
  const void* w[FLOW_MAX_LAYERS * 6 + 3];  // the model's weight list (order of mtad_model.weights)
  int n_layers, d, f, H, KVH, hd, vocab;
  float eps;
  int rows, Rseq, B;
  int ncg;  // activation layout of the pass (act_offset)
  KvView kv;
  RowDesc rd;
  float* h;  // [rows][d] residual stream (holds the embeddings at launch)
  // Buffers that many workgroups read back through the caches exist once per producing step ("versions"): a line of
  // them is written exactly once per pass and read only after its step has finished, so no cache can hold a stale copy.
  bf16_t* xg;     // h * gain as hi / lo terms: version 0 from the embedding, 2l+1 from layer l's o product, 2l+2 from its down product
  float* ssq;     // partial sums of squares of h, same versions ([rows][1] for version 0, [rows][d/16] after)
  bf16_t* xattn;  // attention output, one version per layer
  bf16_t* xffn;   // silu(gate) * up, one version per layer
  float* q;       // rotated queries [rows][H*hd], one version per layer
  size_t xg_stride, ssq_stride, xattn_stride, xffn_stride, q_stride;  // elements per version
  float* partial;  // attention split partials (read with cache-bypassing loads: one buffer serves all layers)
  const float2* rope;
  float* logits;    // [rows][vocab], or null: the pass ends after the last layer
  float* lse_part;  // float2 [rows][vocab/16]
  uint32_t* status;
  int* sync;
  int units[6];        // work units of a step of each kind (FK_*)
  int strips[6];       // product kinds: strips of 16 output features per unit (1 or 3)
  int attn_gx, attn_want, attn_chunks, n_splits;  // attention: splits offered per item, split policy, chunks per KV head, partial stride
#ifdef MTAD_FLOW_PROFILE
  unsigned long long* prof;  // development builds: [unit][4] wall-clock stamps (start, wait over, stream over, end)
#endif
};

// Before the first launch of a pass: copies the record to `dev` (device memory, where the pass kernel reads it) and
// zeroes the n synchronisation words (a kernel: the pass must be recordable into a graph, and memset nodes misbehave there).
hipError_t launch_flow_setup(const FlowArgs& a, FlowArgs* dev, int* sync, int n, hipStream_t s);
// steps [s_begin, s_end) of the pass described by `a` (host copy) = `dev` (device copy) in one launch.  head_dim 64 or 128.
hipError_t launch_flow(const FlowArgs& a, const FlowArgs* dev, int s_begin, int s_end, hipStream_t s);
// (splits offered per attention item, split policy word) for a pass of B sequences of R rows
void flow_attention_plan(int KVH, int n_chunks, int B, int n_splits, int* gx, int* want);

}  // namespace mtad
