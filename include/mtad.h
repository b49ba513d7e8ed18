/*
 * mtad.h - C ABI of the MI355X hot path of multi-token assisted decoding (MTAD) and its
 * multi-candidate variant (MMTAD), arXiv 2407.09722.
 *
 * One iteration of the method (Algorithm 1, appendix "Pseudocode of MTAD"; Section 3.3 for
 * the tree variant) is cut at its four seams:
 *
 *   mtad_draft_beam_step   x, q <- beamSample(M_q, input)      (Section 2.1, Eq. 2; one beam step)
 *   mtad_build_tree        rows of the target pass from the beam history (Section 3.3, Fig. 3a/b)
 *   mtad_verify_tree       P <- M_p(input, X) in one pass        (Algorithm 1; Section 3.3)
 *   mtad_accept            longest passing prefix eta, bonus token t ~ P_{eta+1}
 *   mtad_kv_commit         keep [x_1..x_eta], drop the rest      ("rollback", Section 4)
 *
 * Conventions
 *   - Plain C.  Every function returns 0 (MTAD_OK) or a negative mtad_status code; nothing
 *     throws.  Shapes and pointers are validated on the host before anything is enqueued, so
 *     a call that returns an error has had no effect on device memory.
 *   - "device" pointers are HIP device memory owned by the caller and BORROWED for the
 *     duration of the enqueued work; "host" pointers are read during the call only.
 *     The library allocates device memory nowhere: the caller binds one workspace.
 *   - All hot calls only enqueue work on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and return; results are valid once the caller synchronises.  No call
 *     synchronises the device.
 *   - Lengths live on the device (mtad_kv.len) so that an iteration needs no host round trip.
 *     A kernel that would step outside a KV cache or outside the 64-row speculative window
 *     writes nothing there and sets a sticky bit readable with mtad_device_status().
 *   - A context is not thread safe; use one context per stream.
 *   - Matrices are row-major [out_features, in_features].  dtype 0 = float32 everywhere.
 *     dtype 1 = bfloat16 weights; KV cache in IEEE half (16 bits per value, round to nearest
 *     even); an activation entering a weight matrix product is carried as the sum of two
 *     bfloat16 terms hi = bf16(x), lo = bf16(x - hi); accumulation, queries, residual stream,
 *     softmax, logits and all scores are float32.
 */
#ifndef MTAD_H
#define MTAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MTAD_OK = 0,
  MTAD_EINVAL = -1, /* null pointer, bad enum, bad step */
  MTAD_ESHAPE = -2, /* shape the kernels do not support (rows > 64, beam > 8, K % 32, ...) */
  MTAD_ECAP = -3,   /* workspace or cache too small for the request */
  MTAD_EHIP = -4,   /* a HIP call failed; see mtad_last_hip_error() */
  MTAD_ENOSYS = -5  /* not built */
} mtad_status;

#define MTAD_MAX_ROWS 64  /* rows per sequence in one pass (width of the tree attention mask) */
#define MTAD_MAX_BEAM 8
#define MTAD_MODE_MTAD 0  /* verify the output beam only (chain of gamma tokens)            */
#define MTAD_MODE_MMTAD 1 /* verify every intermediate beam (tree of beam*gamma tokens)     */

typedef struct mtad_ctx mtad_ctx; /* opaque; owns the workspace descriptor, never weights or caches */

/* A decoder: pre-RMSNorm, rotary positions (pairs (i, i+head_dim/2), angle pos*theta^(-2i/head_dim)),
 * grouped-query attention (query head j reads kv head j*n_kv_heads/n_heads), SwiGLU FFN, no biases.
 * weights: HOST array of 3 + 6*n_layers DEVICE pointers in this order:
 *   embed [vocab, d_model];
 *   per layer: g_attn [d_model] f32, w_qkv [(n_heads+2*n_kv_heads)*head_dim, d_model] (q heads, k heads,
 *   v heads), w_o [d_model, n_heads*head_dim], g_ffn [d_model] f32, w_gu [2*d_ffn, d_model] (gate rows,
 *   then up rows), w_d [d_model, d_ffn];
 *   g_final [d_model] f32; unembed [vocab, d_model].
 * Matrices are in `dtype`; norm gains are always float32.
 * dtype 0: every matrix row-major [out_features][in_features].
 * dtype 1: embed row-major; every other matrix in the tile-packed layout written by mtad_pack_matrix
 * (w_qkv with MTAD_PACK_QKV, w_gu with MTAD_PACK_GATE_UP, the rest MTAD_PACK_PLAIN). */
typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t dtype; /* 0 float32, 1 bfloat16 */
  float rms_eps, rope_theta;
  const void *const *weights;
} mtad_model;

/* Paged KV cache of one model, device memory owned by the caller.
 * k, v: [n_layers][n_pages][page_size][n_kv_heads][head_dim], float32 (dtype 0) or IEEE half (dtype 1).
 * page_table: int32 [batch][max_pages], logical page -> physical page (each < n_pages).
 * len: int32 [batch], tokens whose K/V are committed.  Token position t of sequence s lives in
 * page page_table[s][t / page_size], slot t % page_size.  Rows of a pass that are not committed yet
 * (speculative rows) are written at logical positions len, len+1, ... in row order. */
typedef struct {
  void *k, *v;
  const int32_t *page_table;
  int32_t *len;
  int32_t page_size, max_pages, n_pages;
} mtad_kv;

/* Beam history of one draft phase, device memory owned by the caller, all [batch][gamma][beam]:
 * tok = token of survivor j of step i, parent = the step i-1 beam it extends (0 at step 0),
 * cum_logq = log q(branch | context), the likelihood beam sampling stores per beam (Section 2.1).
 * Survivors of a step are listed best first. */
typedef struct {
  int32_t *tok, *parent;
  float *cum_logq;
} mtad_beam;

/* Rows of one target pass, device memory owned by the caller, M rows per sequence, row 0 = the root
 * (last committed token, not cached yet).  tok/parent/depth/src_beam: int32 [batch][M]; parent is a row
 * index (-1 for the root); src_beam = the beam index the node had in its step.  anc_mask: uint64
 * [batch][M], bit j set iff row j is the row itself or one of its ancestors (the tree attention mask,
 * Fig. 3b).  qref: float [batch][gamma], log q(x**_{1:i} | context) of the output beam x** (Eq. 9). */
typedef struct {
  int32_t M;
  int32_t *tok, *parent, *depth, *src_beam;
  uint64_t *anc_mask;
  float *qref;
} mtad_tree;

/* Result of the accept step, device memory owned by the caller.
 * eta [batch]; path [batch][gamma] = tree rows of the accepted branch, depth 1.. (-1 padded);
 * bonus_row [batch] = tree row whose target distribution the bonus token was drawn from;
 * bonus_tok [batch]; out_tok [batch][gamma+1] = [x_1..x_eta, t]; out_cnt [batch] = eta+1. */
typedef struct {
  int32_t *eta, *path, *bonus_row, *bonus_tok, *out_tok, *out_cnt;
} mtad_accept_out;

/* Per-sequence decoding state carried between iterations, device memory owned by the caller.
 * root_tok [batch]: last committed token (row 0 of the next target pass).
 * catchup_tok [batch][gamma+1], catchup_cnt [batch]: committed tokens the draft model has not
 * run yet (the last of them is root_tok); 1..gamma+1 of them. */
typedef struct {
  int32_t *root_tok, *catchup_tok, *catchup_cnt;
} mtad_state;

typedef struct {
  int32_t batch, gamma, beam;
  int32_t mode;         /* MTAD_MODE_* : fixes the rows of the target pass (1+gamma or 1+beam*gamma) */
  int32_t prefill_rows; /* rows per sequence in one prefill chunk, 1..64 */
  int32_t max_context;  /* upper bound on committed + speculative tokens per sequence */
} mtad_config;

/* ---- life cycle -------------------------------------------------------------------------------- */

/* Creates a context for one (target, draft) pair of shapes; the weights pointers are not read here.
 * Errors: EINVAL null; ESHAPE beam > 8, rows > 64, beam > vocab, head_dim not 64/128, bf16 with
 * d_model/d_ffn/(n_heads*head_dim) not multiples of 32 or output widths not multiples of 16. */
int mtad_create(mtad_ctx **ctx, const mtad_config *cfg, const mtad_model *target, const mtad_model *draft);
void mtad_destroy(mtad_ctx *ctx);
/* Bytes of device workspace the context needs; bind exactly one buffer (256-byte aligned) before
 * any hot call.  The contents need no initialisation.  ECAP if too small. */
size_t mtad_workspace_bytes(const mtad_ctx *ctx);
int mtad_bind_workspace(mtad_ctx *ctx, void *device_buf, size_t bytes);
/* bf16 passes of at most 8 rows (all sequences together) can run every product and the attention of every layer as work
 * units of ONE kernel launch, handed out in dependency order, instead of one kernel per step (same arithmetic; the form every
 * larger pass takes).  on = 0: never; 1 (the default): for models whose layers hold at least 64 MiB of weights, where
 * it is the faster form; 2: for every such pass.  Waits inside the one-launch pass are bounded: one that gives up sets status
 * bit 3 and the pass runs to its end.  The environment variable MTAD_FUSED_PASS=0|1|2 sets the same at context creation. */
int mtad_set_fused_pass(mtad_ctx *ctx, int32_t on);
/* Warped distributions (appendix "Hyper-parameter Details"; the footnote of Section 3.2 allows approximating p~ with
 * q~): with top_k > 0 every next-token distribution of both models is warped before it is used: the top_k most likely
 * tokens keep their probabilities and are normalised; of those, in descending order, the shortest prefix whose cumulative
 * probability exceeds top_p is kept and normalised again.  mtad_draft_beam_step then scores with log q~;
 * mtad_verify_tree returns rows of log p~ in `logits` (minus infinity outside the support), 0 in `row_lse`, and
 * log p~ of the draft tokens in `logp_cond` (minus infinity for a token outside the target's support: such a branch
 * passes no positive threshold); mtad_accept, given those rows, draws the bonus token from p~.  1 <= top_k <= 16,
 * top_p > 0 (a top_p of 1 or more keeps all top_k tokens); top_k = 0 turns warping off (the default). */
int mtad_set_warp(mtad_ctx *ctx, int32_t top_k, float top_p);
const char *mtad_strerror(int status);
int mtad_last_hip_error(const mtad_ctx *ctx); /* hipError_t of the last failed HIP call, 0 if none */
/* Copies the sticky device status word to *host_bits after synchronising `stream` (the only call that
 * synchronises).  Bit 0: KV capacity exceeded; bit 1: speculative window (64 rows) exceeded;
 * bit 2: bad catch-up count; bit 3: a bounded wait inside the one-launch pass gave up.  0 = clean. */
int mtad_device_status(mtad_ctx *ctx, uint32_t *host_bits, void *stream);

/* Repacks a row-major bfloat16 matrix [N][K] (device) into the layout the matrix-core kernels stream: the 16x32
 * tile (nt, kt) is 1 KiB contiguous at element offset (nt*(K/32) + kt)*512, lane l of a wavefront owning the 8
 * elements of packed row l%16 at k = kt*32 + (l/16)*8.  Packed row j of strip nt is source row
 *   PLAIN    nt*16 + j
 *   QKV      head*head_dim + (j < 8 ? 8u + j : head_dim/2 + 8u + j-8), head = nt / (head_dim/16), u = nt % (head_dim/16)
 *            (a strip holds rotary pairs, so the rotation happens in the product's epilogue)
 *   GATE_UP  j < 8 ? 8nt + j : N/2 + 8nt + j-8   (a strip holds 8 gate and the matching 8 up features)
 * Done once per matrix when a model is loaded; not part of an iteration.  src != dst.  N % 16 == 0, K % 32 == 0. */
#define MTAD_PACK_PLAIN 0
#define MTAD_PACK_QKV 1
#define MTAD_PACK_GATE_UP 2
int mtad_pack_matrix(int32_t kind, const void *src, void *dst, int32_t N, int32_t K, int32_t head_dim, void *stream);

/* ---- prompt ------------------------------------------------------------------------------------ */

/* Runs tokens[batch][n_tokens] (device, int32) through `model` in causal chunks and commits all of
 * them to `kv` (kv.len += n_tokens).  No logits are produced.  This is the target pass on a chain
 * whose rows are all kept (Section 2.2: the context is the input of every iteration). */
int mtad_prefill(mtad_ctx *ctx, const mtad_model *model, mtad_kv *kv, const int32_t *tokens, int32_t n_tokens,
                 void *stream);

/* ---- the iteration ----------------------------------------------------------------------------- */

/* One step (0 <= step < gamma) of beam sampling on the auxiliary model (Section 2.1, Eq. 2).
 * step 0 runs the catch-up tokens st->catchup_tok[s][0..cnt) as a causal chain on top of dkv and
 * expands the single beam "context"; step i >= 1 runs the survivors of step i-1, each attending to the
 * context and to its own ancestors, and expands them.  Candidate (beam r, token v) scores
 * cum_logq[r] + log q(v | beam r); the beam best (sample_beam = 0, ties to the lowest r*vocab+v) or
 * beam draws without replacement in proportion to p_beam (sample_beam = 1, Gumbel noise keyed by
 * (seed, sequence, absolute position, r*vocab+v)) are written to hist[.][step][.], best first.
 * dkv.len is not changed; speculative rows accumulate after it until mtad_kv_commit. */
int mtad_draft_beam_step(mtad_ctx *ctx, const mtad_model *draft, mtad_kv *dkv, mtad_beam *hist, int32_t step,
                         const mtad_state *st, int32_t sample_beam, uint64_t seed, void *stream);

/* Rows of the target pass from a finished beam history (Section 3.3; Fig. 3a): mode MTAD = the chain
 * of the output beam x** (the final beam with the largest cum_logq, ties to the lowest index); mode
 * MMTAD = every survivor of every step, row 1 + i*beam + j.  Fills every array of `tree`. */
int mtad_build_tree(mtad_ctx *ctx, const mtad_beam *hist, int32_t mode, mtad_tree *tree, void *stream);

/* Target pass over the M rows of every sequence in one go (Algorithm 1: P <- M_p(input, X); Section 3.3:
 * tree attention).  Row r sits at position tkv.len + depth[r], attends to the committed cache and to the
 * rows in anc_mask[r]; its K/V go to logical slot tkv.len + r.  Outputs (device, float32):
 *   logits   [batch][M][vocab]  unnormalised next-token scores after every row (row i of P, as logits)
 *   row_lse  [batch][M]         logsumexp of each row
 *   logp_cond[batch][M]         log p(tok[c] | branch of c) = logits[parent(c)][tok[c]] - row_lse[parent(c)];
 *                               0 for the root.
 * tkv.len is not changed. */
int mtad_verify_tree(mtad_ctx *ctx, const mtad_model *target, mtad_kv *tkv, const int32_t *root_tok,
                     const mtad_tree *tree, float *logp_cond, float *row_lse, float *logits, void *stream);

/* Joint-likelihood acceptance (Section 3.2, Algorithm 1; Section 3.3, Eq. 9).  log p of a branch = sum of
 * logp_cond from the first level down.  mode MTAD: eta = the largest depth i with
 * min(0, log p_i - qref[i]) > log tau (every prefix is examined); mode MMTAD: a node passes iff
 * log p - qref[depth] >= log tau; the deepest passing node wins, then the larger log p, then the lower
 * row.  eta = 0 if nothing passes.  tau in [0,1); tau = 0 passes everything.  The bonus token comes from
 * the logits row of the accepted node (root row if eta = 0): argmax (sample_bonus = 0, ties to the
 * lowest id) or argmax(logit + Gumbel noise) keyed by (seed, sequence, position tkv.len+1+eta, id). */
int mtad_accept(mtad_ctx *ctx, const mtad_tree *tree, const float *logp_cond, const float *logits, int32_t vocab,
                const mtad_kv *tkv, float tau, int32_t mode, int32_t sample_bonus, uint64_t seed,
                mtad_accept_out *out, void *stream);

/* Multi-token joint decoding (Section 3.1) as the paper runs it: beam sampling on the target model itself, gamma = K tokens
 * per step.  A context whose "draft" model is the target runs the K beam steps with mtad_draft_beam_step on that model's
 * cache and builds the chain of the most likely final beam with mtad_build_tree (mode MTAD); this call writes the chain
 * as an accept record that emits all K tokens (out_tok[0..K-1], out_cnt = K), and mtad_kv_commit with tkv = NULL and that
 * cache as dkv commits them: the rows of the first K - 1 tokens are gathered into place, the last token, which the beam
 * steps never ran, becomes the pending token of the next step.  No target pass is involved.
 * MTAD_ESHAPE unless tree->M == gamma + 1. */
int mtad_accept_chain(mtad_ctx *ctx, const mtad_tree *tree, mtad_accept_out *out, void *stream);
/* Vanilla speculative decoding (Section 2.2), the baseline the paper compares with, on the same entry points: a
 * context created with beam = 1 and mode MTAD drafts a chain token by token (mtad_draft_beam_step with sample_beam = 1 is
 * ancestral sampling; it also keeps log q of every step in the workspace), mtad_verify_tree runs the target over the
 * chain, and this call replaces mtad_accept: draft token x_t passes with probability min(1, p(x_t)/q(x_t)) (a uniform
 * number keyed by seed, sequence and the token's absolute position), the tokens before the first failure are kept, and
 * the next token is drawn from the residual distribution norm(max(0, p - q)) of the failed position, or from the
 * target's row after the last token when all passed.  p and q are the warped distributions when mtad_set_warp is on.
 * `logits` [B][gamma+1][vocab] and `row_lse` [B][gamma+1] as mtad_verify_tree wrote them; `out` as mtad_accept;
 * mtad_kv_commit follows unchanged.  MTAD_ESHAPE unless beam == 1, tree->M == gamma + 1 and both models share `vocab`. */
int mtad_accept_spd(mtad_ctx *ctx, const mtad_tree *tree, const float *logits, const float *row_lse, int32_t vocab, const mtad_kv *tkv,
                    uint64_t seed, mtad_accept_out *out, void *stream);
/* Commit / rollback.  Target cache: the root row and the accepted branch are moved to logical slots
 * len .. len+eta (a no-op copy for a chain) and tkv.len += eta + 1; everything else in the speculative
 * window is dropped.  Draft cache: catch-up rows and the rows of the accepted branch the
 * draft has run (depth <= gamma-1) are kept likewise.  Either cache may be NULL (not both): plain decoding has no
 * draft cache, multi-token joint decoding no target cache.  `st` is rewritten for the next iteration:
 * root_tok = t, catchup = [x_gamma, t] if eta == gamma else [t]. */
int mtad_kv_commit(mtad_ctx *ctx, mtad_kv *tkv, mtad_kv *dkv, const mtad_tree *tree, const mtad_accept_out *acc,
                   mtad_state *st, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MTAD_H */
