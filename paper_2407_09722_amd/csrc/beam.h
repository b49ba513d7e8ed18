// Internal views of the caller's beam history, tree and accept buffers, and the launchers of kernels_beam.hip.
#pragma once
#include "common.h"

#define MTAD_MAX_ROWS 64
#define MTAD_MAX_GAMMA 64

namespace mtad {

struct BeamView {
  int32_t* tok;
  int32_t* parent;
  float* cum;
};
struct TreeView {
  int32_t M;
  int32_t *tok, *parent, *depth, *src_beam;
  uint64_t* anc_mask;
  float* qref;
};
struct AcceptView {
  int32_t *eta, *path, *bonus_row, *bonus_tok, *out_tok, *out_cnt;
};

hipError_t launch_draft_rows(const RowDesc& rd, const int32_t* len, BeamView hist, const int32_t* cu_tok, const int32_t* cu_cnt,
                             int step, int B, int R, int gamma, int beam, int cap, uint32_t* status, hipStream_t s);
hipError_t launch_verify_rows(const RowDesc& rd, const int32_t* len, const int32_t* root_tok, TreeView tree, int B, int cap,
                              uint32_t* status, hipStream_t s);
hipError_t launch_prefill_rows(const RowDesc& rd, const int32_t* len, const int32_t* tokens, int n, int c0, int B, int R, int cap,
                               uint32_t* status, hipStream_t s);
hipError_t launch_advance_len(int32_t* len, const int32_t* nspec, int B, int cap, hipStream_t s);
hipError_t launch_topb(const float* logits, const float* lse, BeamView hist, const int32_t* cu_cnt, const int32_t* len, int step,
                       int B, int R, int gamma, int beam, int V, int sample, uint64_t seed, float* part_key, int* part_idx, int G,
                       hipStream_t s);
hipError_t launch_build_tree(BeamView hist, TreeView tree, int B, int gamma, int beam, int mode, hipStream_t s);
// vanilla speculative decoding: keep log q of a width-1 draft step's live row; token-wise acceptance + next token
hipError_t launch_save_logq_row(const float* logits, const float* lse, const int32_t* cu_cnt, int step, int B, int R, int gamma, int V,
                                float* qrows, hipStream_t s);
hipError_t launch_accept_spd(TreeView tree, const float* logits, const float* lse, const float* qrows, int V, const int32_t* len, int B,
                             int gamma, uint64_t seed, AcceptView out, hipStream_t s);
// multi-token joint decoding: the chain in `tree` as an accept record (all gamma tokens emitted)
hipError_t launch_accept_chain(TreeView tree, int B, int gamma, AcceptView out, hipStream_t s);
// rows of logits -> rows of log p~ (top_k, then top_p prefix; 1 <= top_k <= 16), lse -> 0; in place
hipError_t launch_warp_rows(float* logits, float* lse, int rows, int V, int top_k, float top_p, hipStream_t s);
hipError_t launch_gather_logp(const float* logits, const float* lse, TreeView tree, int B, int V, float* logp_cond, hipStream_t s);
hipError_t launch_accept(TreeView tree, const float* logp_cond, const float* logits, int V, const int32_t* len, float log_tau, int mode,
                         int B, int gamma, int sample, uint64_t seed, AcceptView out, hipStream_t s);
hipError_t launch_kv_gather(int dtype, KvView kv, int n_layers, int B, const int32_t* eta, const int32_t* path, const int32_t* src_beam,
                            const int32_t* cu_cnt, int M, int gamma, int beam, int is_draft, hipStream_t s);
hipError_t launch_commit_state(int32_t* tlen, int32_t* dlen, TreeView tree, AcceptView acc, int32_t* root_tok, int32_t* cu_tok,
                               int32_t* cu_cnt, int B, int gamma, int tcap, int dcap, hipStream_t s);

constexpr int TOPB_BLOCKS = 64;  // stage-1 workgroups per sequence

}  // namespace mtad
