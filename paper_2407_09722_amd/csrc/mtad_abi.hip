// C-ABI layer of libmtad: context, workspace carving, host-side validation and the sequencing of the
// kernels for the draft beam step, the target pass, accept and commit (see include/mtad.h).
#include "../../include/mtad.h"
#include "../../include/mtad_kernels.h"
#include "beam.h"
#include "common.h"
#include "gemm.h"
#include "flow.h"

#include <math.h>
#include <mutex>
#include <new>
#include <stdlib.h>
#include <string.h>

using namespace mtad;

struct mtad_ctx {
  mtad_config cfg;
  mtad_model tshape, dshape;  // shapes only (weights pointer cleared)
  int M;                      // rows per sequence of the target pass
  int Rmax;                   // most rows per sequence of any pass
  int draft_rows;             // rows per sequence of a draft step (max over steps)
  size_t ws_need;
  char* ws;
  // workspace carve-up
  float *h, *qkv, *gu, *dlogits, *lse, *partial, *part_key, *ssq, *lse_part;
  float* qrows;  // [batch][gamma][draft vocab]: log q of every draft step's live row when the beam is one wide (mtad_accept_spd)
  void *xn, *xg;  // xn: attention output / FFN activation; xg: h*gain planes feeding the next normalised product
  int* attn_cnt;
  float* gemm_part;  // k-split partial sums of the product kernel (products with few strips, more than 8 rows)
  size_t gemm_part_n;  // floats
  int* gemm_cnt;
  int gemm_cnt_n;
  int pass_ncg;    // activation layout of the pass in flight (0 planes, else row groups of the fragment order): its lm_head reads it
  int warp_k;      // > 0: next-token distributions of both models are warped (mtad_set_warp)
  float warp_p;
  bf16_t* gemm_xfrag;  // scratch of the many-row product kernel: a pass's activations in operand-fragment order
  size_t gemm_xfrag_n;
  size_t attn_cnt_n;
  float2* rope;
  int* part_idx;
  RowDesc rd;
  uint32_t* status;
  int n_cus;                // compute units of the device
  // one-launch pass (kernels_flow.hip) for bf16 passes of at most FLOW_MAX_ROWS rows: 0 never, 1 where a layer's
  // weights are large enough for the stream to matter (the default), 2 always
  int flow_on;
  bf16_t *flow_xg, *flow_xattn, *flow_xffn;  // per-step versions of the activation terms (see flow.h)
  float *flow_ssq, *flow_q;
  int* flow_sync;
  int flow_sync_n;
  FlowArgs* flow_args;  // device copy of the arguments of the pass in flight
#ifdef MTAD_FLOW_PROFILE
  unsigned long long* flow_prof;
#endif
  // set by mtad_verify_tree around its pass: the logsumexp kernel of a bf16 pass then also gathers logp_cond
  const mtad_tree* gather_tree;
  float* gather_out;
  int last_hip;
};

namespace {

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline int imax(int a, int b) { return a > b ? a : b; }
inline int imin(int a, int b) { return a < b ? a : b; }
inline size_t imax64(size_t a, size_t b) { return a > b ? a : b; }

int shape_ok(const mtad_model* m) {
  if (m->n_layers < 1 || m->d_model < 1 || m->n_heads < 1 || m->n_kv_heads < 1 || m->d_ffn < 1 || m->vocab < 1) return 0;
  if (m->head_dim != 64 && m->head_dim != 128) return 0;
  if (m->n_heads % m->n_kv_heads) return 0;
  if (m->dtype != 0 && m->dtype != 1) return 0;
  const int hhd = m->n_heads * m->head_dim, qkv = (m->n_heads + 2 * m->n_kv_heads) * m->head_dim;
  if (m->d_model % 4 || m->d_ffn % 4) return 0;
  if (m->dtype == 1) {
    if (m->d_model % 32 || m->d_ffn % 32 || hhd % 32) return 0;           // reduction widths
    if (m->d_model % 16 || qkv % 16 || (2 * m->d_ffn) % 16 || m->vocab % 16) return 0;  // output widths
  }
  return 1;
}

int splits_for(const mtad_ctx* c, const mtad_model* m, int R) {
  const int chunks = (R + 15) / 16;
  const int blocks = c->cfg.batch * m->n_heads * chunks;
  int s = (1024 + blocks - 1) / blocks;
  s = imin(s, (c->cfg.max_context + 127) / 128);
  return imax(1, imin(32, s));
}

struct Carver {
  size_t off = 0;
  char* base;
  explicit Carver(char* b) : base(b) {}
  template <typename T>
  T* take(size_t n) {
    T* p = base ? (T*)(base + off) : nullptr;
    off += align256(n * sizeof(T));
    return p;
  }
};

void carve(mtad_ctx* c, char* base) {
  const mtad_model &t = c->tshape, &d = c->dshape;
  const size_t rows = (size_t)c->cfg.batch * c->Rmax;
  const int dmax = imax(t.d_model, d.d_model), fmax = imax(t.d_ffn, d.d_ffn);
  const int hhd = imax(t.n_heads * t.head_dim, d.n_heads * d.head_dim);
  const int qkv = imax((t.n_heads + 2 * t.n_kv_heads) * t.head_dim, (d.n_heads + 2 * d.n_kv_heads) * d.head_dim);
  const int hdmax = imax(t.head_dim, d.head_dim);
  Carver k(base);
  c->status = k.take<uint32_t>(64);
  c->h = k.take<float>(rows * dmax);
  const size_t rows8 = (rows + 7) / 8 * 8;  // operand-fragment order holds whole groups of 8 rows
  c->xn = k.take<float>(rows8 * imax(imax(dmax, hhd), fmax));
  c->xg = k.take<float>(rows8 * dmax);
  c->ssq = k.take<float>(rows * (size_t)(dmax / 16 + 1));
  c->lse_part = k.take<float>(rows * (size_t)(imax(t.vocab, d.vocab) / 16 + 1) * 2);
  c->attn_cnt_n = (size_t)c->cfg.batch * imax(t.n_heads, d.n_heads) * (size_t)((c->Rmax + 7) / 8);
  c->attn_cnt = k.take<int>(c->attn_cnt_n);
  {
    size_t pf = 0;
    int pc = 0;
    for (const mtad_model* m : {&t, &d}) {
      if (m->dtype != 1) continue;
      const int hh = m->n_heads * m->head_dim, qk = (m->n_heads + 2 * m->n_kv_heads) * m->head_dim;
      for (int N : {qk, m->d_model, 2 * m->d_ffn, m->vocab, hh}) {
        if (gemm_split_floats(N) > pf) pf = gemm_split_floats(N);
        if (gemm_split_counters(N) > pc) pc = gemm_split_counters(N);
      }
    }
    c->gemm_part_n = pf + 64;
    c->gemm_part = k.take<float>(c->gemm_part_n);
    c->gemm_cnt_n = pc + 1;
    c->gemm_cnt = k.take<int>((size_t)c->gemm_cnt_n);
    // widest reduction dimension of any product: the model widths and FFN widths
    c->gemm_xfrag_n = gemm_tiled_xfrag_elems((int)rows, imax(imax(dmax, fmax), hhd));
    c->gemm_xfrag = k.take<bf16_t>(c->gemm_xfrag_n);
  }
  {  // the one-launch pass: versions of what its steps hand on, sized for FLOW_MAX_ROWS rows of the larger need of the two models
    size_t xg = 0, ssq = 0, xa = 0, xf = 0, q = 0;
    int items = 0;
    for (const mtad_model* m : {&t, &d}) {
      if (m->dtype != 1 || m->n_layers > FLOW_MAX_LAYERS) continue;
      const size_t L = (size_t)m->n_layers, R8 = FLOW_MAX_ROWS, hh = (size_t)m->n_heads * m->head_dim;
      xg = imax64(xg, (2 * L + 1) * 2 * R8 * m->d_model);
      ssq = imax64(ssq, (2 * L + 1) * R8 * (m->d_model / 16 + 1));
      xa = imax64(xa, L * 2 * R8 * hh);
      xf = imax64(xf, L * 2 * R8 * m->d_ffn);
      q = imax64(q, L * R8 * hh);
      items = imax(items, 12 * m->n_heads + 64);
    }
    c->flow_xg = k.take<bf16_t>(xg);
    c->flow_ssq = k.take<float>(ssq);
    c->flow_xattn = k.take<bf16_t>(xa);
    c->flow_xffn = k.take<bf16_t>(xf);
    c->flow_q = k.take<float>(q);
    c->flow_sync_n = flow_sync_ints(items);
    c->flow_sync = k.take<int>((size_t)c->flow_sync_n);
    c->flow_args = k.take<FlowArgs>(1);
#ifdef MTAD_FLOW_PROFILE
    c->flow_prof = k.take<unsigned long long>((size_t)4 * 100000);
#endif
  }
  c->qkv = k.take<float>(rows * qkv);
  c->gu = k.take<float>(rows * 2 * fmax);
  c->dlogits = k.take<float>((size_t)c->cfg.batch * c->draft_rows * d.vocab);
  c->qrows = k.take<float>(c->cfg.beam == 1 ? (size_t)c->cfg.batch * c->cfg.gamma * d.vocab : 1);
  c->lse = k.take<float>(rows);
  const size_t pt = attention_partial_floats(c->cfg.batch, c->Rmax, t.n_heads, t.head_dim, 32);
  const size_t pd = attention_partial_floats(c->cfg.batch, c->Rmax, d.n_heads, d.head_dim, 32);
  c->partial = k.take<float>(pt > pd ? pt : pd);
  c->rope = k.take<float2>(rows * (hdmax / 2));
  c->rd.tok = k.take<int32_t>(rows);
  c->rd.pos = k.take<int32_t>(rows);
  c->rd.slot = k.take<int32_t>(rows);
  c->rd.mask = k.take<uint64_t>(rows);
  c->rd.nspec = k.take<int32_t>(c->cfg.batch);
  c->part_key = k.take<float>((size_t)c->cfg.batch * TOPB_BLOCKS * 8);
  c->part_idx = k.take<int>((size_t)c->cfg.batch * TOPB_BLOCKS * 8);
  c->ws_need = k.off;
}

int kv_ok(const mtad_kv* kv) {
  return kv && kv->k && kv->v && kv->page_table && kv->len && kv->page_size > 0 && kv->max_pages > 0 && kv->n_pages > 0;
}

KvView view_of(const mtad_kv* kv, const mtad_model* m) {
  KvView v;
  v.k = kv->k;
  v.v = kv->v;
  v.page_table = kv->page_table;
  v.len = kv->len;
  v.page_size = kv->page_size;
  v.max_pages = kv->max_pages;
  v.n_pages = kv->n_pages;
  v.n_kv_heads = m->n_kv_heads;
  v.head_dim = m->head_dim;
  v.layer_stride = (int64_t)kv->n_pages * kv->page_size * m->n_kv_heads * m->head_dim;
  return v;
}

int same_shape(const mtad_model* a, const mtad_model* b) {
  return a->n_layers == b->n_layers && a->d_model == b->d_model && a->n_heads == b->n_heads && a->n_kv_heads == b->n_kv_heads &&
         a->head_dim == b->head_dim && a->d_ffn == b->d_ffn && a->vocab == b->vocab && a->dtype == b->dtype;
}

#define HIP_TRY(ctx, expr)              \
  do {                                  \
    hipError_t e__ = (expr);            \
    if (e__ != hipSuccess) {            \
      (ctx)->last_hip = (int)e__;       \
      return MTAD_EHIP;                 \
    }                                   \
  } while (0)

int lm_head(mtad_ctx* c, const mtad_model* m, int rows, float* logits, float* lse, hipStream_t s);

// Row logsumexp from the per-strip partials the lm_head product left; inside mtad_verify_tree the same kernel also
// gathers the tree nodes' conditional log-likelihoods.
int finish_lse(mtad_ctx* c, const mtad_model* m, int rows, const float* logits, float* lse, hipStream_t s) {
  if (c->gather_out && c->gather_tree) {
    const mtad_tree* t = c->gather_tree;
    HIP_TRY(c, launch_lse_gather(c->lse_part, lse, rows / t->M, t->M, m->vocab / 16, logits, m->vocab, t->parent, t->tok, c->gather_out, s));
    c->gather_out = nullptr;  // done: the caller skips its separate gather
    return MTAD_OK;
  }
  HIP_TRY(c, launch_lse_finish(c->lse_part, lse, rows, m->vocab / 16, s));
  return MTAD_OK;
}

// The decoder pass over B*R rows described by ctx->rd.  float32 models: hidden states end in ctx->h.
// bf16 models: additionally ctx->xg holds the planes of h*g_final and ctx->ssq the per-strip sums of squares,
// ready for the lm_head product.
int decoder_pass_f32(mtad_ctx* c, const mtad_model* m, const mtad_kv* kv, int R, hipStream_t s) {
  const int B = c->cfg.batch, rows = B * R;
  const int d = m->d_model, f = m->d_ffn, H = m->n_heads, hd = m->head_dim;
  const int qkvw = (H + 2 * m->n_kv_heads) * hd;
  const KvView kvv = view_of(kv, m);
  const int n_splits = splits_for(c, m, R);
  const void* const* W = m->weights;
  HIP_TRY(c, launch_embed(0, W[0], c->rd.tok, c->h, rows, d, m->vocab, nullptr, nullptr, nullptr, c->rd.pos, c->rope, hd, m->rope_theta, 0, s));
  for (int l = 0; l < m->n_layers; ++l) {
    const void* const* L = W + 1 + 6 * l;
    HIP_TRY(c, launch_rmsnorm(0, c->h, (const float*)L[0], c->xn, rows, d, m->rms_eps, s));
    HIP_TRY(c, launch_gemm_f32(L[1], c->xn, c->qkv, rows, qkvw, d, qkvw, false, s));
    HIP_TRY(c, launch_rope_kv(0, c->qkv, c->rope, c->rd, kvv, l, B, R, H, c->status, s));
    HIP_TRY(c, launch_attention(0, c->qkv, qkvw, c->rd, kvv, l, B, R, H, c->partial, n_splits, c->attn_cnt, c->xn, 0, s));
    HIP_TRY(c, launch_gemm_f32(L[2], c->xn, c->h, rows, d, H * hd, d, true, s));
    HIP_TRY(c, launch_rmsnorm(0, c->h, (const float*)L[3], c->xn, rows, d, m->rms_eps, s));
    HIP_TRY(c, launch_gemm_f32(L[4], c->xn, c->gu, rows, 2 * f, d, 2 * f, false, s));
    HIP_TRY(c, launch_silu_mul(0, c->gu, c->xn, rows, f, s));
    HIP_TRY(c, launch_gemm_f32(L[5], c->xn, c->h, rows, d, f, d, true, s));
  }
  return MTAD_OK;
}

// bf16 passes of at most FLOW_MAX_ROWS rows: the row inputs (embedding, rotary table), then every product and the attention
// of every layer and the lm_head as work units of one launch (kernels_flow.hip), then the row logsumexps.  Passes whose
// attention items hold more than 16 (query head, row) pairs (grouped-query models at several rows) run the attention of
// each layer as its own kernels between launches that cover the steps from one attention to the next.
int flow_pass(mtad_ctx* c, const mtad_model* m, const mtad_kv* kv, int R, hipStream_t s, float* logits, float* lse) {
  const int B = c->cfg.batch, rows = B * R, L = m->n_layers;
  const int d = m->d_model, f = m->d_ffn, H = m->n_heads, KVH = m->n_kv_heads, hd = m->head_dim;
  const int hhd = H * hd, qkvw = (H + 2 * KVH) * hd;
  const KvView kvv = view_of(kv, m);
  const void* const* W = m->weights;
  const int ncg = rows < 2 ? 0 : 1;
  c->pass_ncg = ncg;
  FlowArgs fa;
  memset(&fa, 0, sizeof(fa));
  memcpy(fa.w, W, sizeof(void*) * (size_t)(3 + 6 * L));
  fa.n_layers = L; fa.d = d; fa.f = f; fa.H = H; fa.KVH = KVH; fa.hd = hd; fa.vocab = m->vocab;
  fa.eps = m->rms_eps;
  fa.rows = rows; fa.Rseq = R; fa.B = B; fa.ncg = ncg;
  fa.kv = kvv; fa.rd = c->rd;
  fa.h = c->h;
  fa.xg = c->flow_xg; fa.ssq = c->flow_ssq; fa.xattn = c->flow_xattn; fa.xffn = c->flow_xffn; fa.q = c->flow_q;
  const size_t R8 = FLOW_MAX_ROWS;
  fa.xg_stride = 2 * R8 * d; fa.ssq_stride = R8 * (size_t)(d / 16 + 1); fa.xattn_stride = 2 * R8 * hhd; fa.xffn_stride = 2 * R8 * f;
  fa.q_stride = R8 * hhd;
  fa.partial = c->partial; fa.rope = c->rope;
  fa.logits = logits; fa.lse_part = c->lse_part;
  fa.status = c->status; fa.sync = c->flow_sync;
#ifdef MTAD_FLOW_PROFILE
  fa.prof = same_shape(m, &c->tshape) ? c->flow_prof : nullptr;  // the target's passes
#endif
  const int n_cus = c->n_cus > 0 ? c->n_cus : 256;
  const int widths[6] = {qkvw, 0, d, 2 * f, d, m->vocab};
  for (int k = 0; k < 6; ++k) {
    if (k == FK_ATTN) continue;
    const int NT = widths[k] / 16;
    // three strips per unit share the activation fragments where the product has at least two strips per compute unit
    fa.strips[k] = (rows >= 4 && NT >= 2 * n_cus) ? 3 : 1;
    fa.units[k] = (NT + fa.strips[k] - 1) / fa.strips[k];
  }
  const int G = H / KVH;
  const bool attn_in = G * R <= 16;  // one row group per attention item
  fa.attn_chunks = (G * R + 15) / 16;
  fa.n_splits = imin(32, (c->cfg.max_context + 127) / 128);
  if (attn_in) {
    flow_attention_plan(KVH, fa.attn_chunks, B, fa.n_splits, &fa.attn_gx, &fa.attn_want);
    fa.units[FK_ATTN] = fa.attn_gx * KVH * fa.attn_chunks * B;
    if (B * KVH * fa.attn_chunks > c->flow_sync_n - flow_sync_ints(0)) return MTAD_ECAP;
  }
  const int s_last = 5 * L + (logits ? 1 : 0);
  HIP_TRY(c, launch_flow_setup(fa, c->flow_args, c->flow_sync, c->flow_sync_n, s));
  HIP_TRY(c, launch_embed(1, W[0], c->rd.tok, c->h, rows, d, m->vocab, (const float*)W[1], c->flow_xg, c->flow_ssq, c->rd.pos, c->rope, hd,
                          m->rope_theta, ncg, s));
  if (attn_in) {
    HIP_TRY(c, launch_flow(fa, c->flow_args, 0, s_last, s));
  } else {
    int s0 = 0;
    for (int l = 0; l < L; ++l) {
      HIP_TRY(c, launch_flow(fa, c->flow_args, s0, 5 * l + 1, s));  // up to this layer's QKV product
      HIP_TRY(c, launch_attention_mfma(c->flow_q + (size_t)l * fa.q_stride, hhd, c->rd, kvv, l, B, R, H, c->partial, fa.n_splits,
                                       c->flow_xattn + (size_t)l * fa.xattn_stride, ncg, s));
      s0 = 5 * l + 2;
    }
    HIP_TRY(c, launch_flow(fa, c->flow_args, s0, s_last, s));
  }
  return logits ? finish_lse(c, m, rows, logits, lse, s) : MTAD_OK;
}

// bf16 models: five kernels per layer.  Every element-wise step rides on a product's epilogue:
//   qkv product   (rows scaled by the fused RMSNorm factor) -> rotary, q to a buffer, k/v to the cache
//   attention     -> planes of the attention output
//   o product     -> h += ., planes of h*g_ffn, sums of squares
//   gate/up prod. (scaled) -> planes of silu(gate)*up
//   down product  -> h += ., planes of h*g_next, sums of squares
int decoder_pass_bf16(mtad_ctx* c, const mtad_model* m, const mtad_kv* kv, int R, hipStream_t s, float* logits, float* lse) {
  const int B = c->cfg.batch, rows = B * R;
  const int d = m->d_model, f = m->d_ffn, H = m->n_heads, hd = m->head_dim;
  const int qkvw = (H + 2 * m->n_kv_heads) * hd;
  const KvView kvv = view_of(kv, m);
  const int n_splits = splits_for(c, m, R);
  const int tag = same_shape(m, &c->tshape) ? 1 : 0;
  const void* const* W = m->weights;
  const int tail = 1 + 6 * m->n_layers;
  if (c->flow_on && rows <= FLOW_MAX_ROWS && m->n_layers <= FLOW_MAX_LAYERS) {
    // Steps hand over through counters and flags in memory, about as dear as a kernel boundary each; what the one launch
    // gains is the weights requested across those handovers, which counts where a layer streams tens of megabytes
    // (7B-shaped target, 405 MB per layer: pass 2.78 -> 2.61 ms) and not for small models (two 14 MB layers: 95 -> 106 us).
    const size_t layer_bytes = 2 * ((size_t)qkvw * d + (size_t)d * H * hd + (size_t)3 * d * f);
    if (c->flow_on >= 2 || layer_bytes >= ((size_t)64 << 20)) return flow_pass(c, m, kv, R, s, logits, lse);
  }
  // one kernel per step, 2 rows or more: activations in operand-fragment order (act_offset), whole cache lines per
  // fragment, without the unused row slots up to 24 rows (C3 verify, 5 rows: 3.20 ms on planes, 3.14 ms with 8-row
  // fragments, 2.98 ms with 5-row fragments on the three-strip product kernel; 2 to 4 rows 1 to 3 % faster than on
  // planes; one row, plain decoding, 1 % slower)
  const int ncg = rows < 2 ? 0 : (rows + 7) / 8;
  c->pass_ncg = ncg;
  HIP_TRY(c, launch_embed(1, W[0], c->rd.tok, c->h, rows, d, m->vocab, (const float*)W[1], c->xg, c->ssq, c->rd.pos, c->rope, hd, m->rope_theta,
                          ncg, s));
  int np = 1;  // partial sums of squares per row currently in ctx->ssq
  for (int l = 0; l < m->n_layers; ++l) {
    const void* const* L = W + 1 + 6 * l;
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.R = rows;
    a.ncg = ncg;
    a.eps = m->rms_eps;
    a.part = c->gemm_part;
    a.counters = c->gemm_cnt;
    a.part_floats = c->gemm_part_n;
    a.counters_n = c->gemm_cnt_n;
    a.xfrag = c->gemm_xfrag;
    a.xfrag_elems = c->gemm_xfrag_n;
    // qkv
    a.W = (const bf16_t*)L[1]; a.X = (const bf16_t*)c->xg; a.N = qkvw; a.K = d;
    a.ssq = c->ssq; a.NP = np;
    a.q_out = c->qkv; a.rope = c->rope; a.slot = c->rd.slot; a.kv = kvv; a.layer = l; a.Rseq = R; a.n_heads = H; a.status = c->status;
    HIP_TRY(c, launch_gemm_bf16(a, EPI_QKV, tag, s));
    HIP_TRY(c, launch_attention(1, c->qkv, H * hd, c->rd, kvv, l, B, R, H, c->partial, imin(32, (c->cfg.max_context + 127) / 128), c->attn_cnt,
                                c->xn, ncg, s));
    // o projection + residual; prepares the FFN's normalised input
    a.W = (const bf16_t*)L[2]; a.X = (const bf16_t*)c->xn; a.N = d; a.K = H * hd;
    a.ssq = nullptr; a.NP = 0;
    a.h = c->h; a.g_next = (const float*)L[3]; a.planes_out = (bf16_t*)c->xg; a.ssq_out = c->ssq;
    HIP_TRY(c, launch_gemm_bf16(a, EPI_RESID, tag, s));
    np = d / 16;
    // gate/up + SwiGLU
    a.W = (const bf16_t*)L[4]; a.X = (const bf16_t*)c->xg; a.N = 2 * f; a.K = d;
    a.ssq = c->ssq; a.NP = np;
    a.act_out = (bf16_t*)c->xn;
    HIP_TRY(c, launch_gemm_bf16(a, EPI_SWIGLU, tag, s));
    // down projection + residual; prepares the next layer's (or the final) normalised input
    a.W = (const bf16_t*)L[5]; a.X = (const bf16_t*)c->xn; a.N = d; a.K = f;
    a.ssq = nullptr; a.NP = 0;
    a.g_next = (const float*)(l + 1 < m->n_layers ? W[1 + 6 * (l + 1)] : W[tail]);
    HIP_TRY(c, launch_gemm_bf16(a, EPI_RESID, tag, s));
  }
  return logits ? lm_head(c, m, rows, logits, lse, s) : MTAD_OK;
}

// The pass, followed by final norm + lm_head + row logsumexp when `logits` is given.
int decoder_pass(mtad_ctx* c, const mtad_model* m, const mtad_kv* kv, int R, hipStream_t s, float* logits, float* lse) {
  if (m->dtype == 1) return decoder_pass_bf16(c, m, kv, R, s, logits, lse);
  int rc = decoder_pass_f32(c, m, kv, R, s);
  if (rc || !logits) return rc;
  return lm_head(c, m, c->cfg.batch * R, logits, lse, s);
}

int lm_head(mtad_ctx* c, const mtad_model* m, int rows, float* logits, float* lse, hipStream_t s) {
  const void* const* W = m->weights;
  const int tail = 1 + 6 * m->n_layers;
  if (m->dtype == 1) {
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.W = (const bf16_t*)W[tail + 1]; a.X = (const bf16_t*)c->xg; a.R = rows; a.N = m->vocab; a.K = m->d_model;
    a.ncg = c->pass_ncg;
    a.ssq = c->ssq; a.NP = m->d_model / 16; a.eps = m->rms_eps;
    a.Y = logits; a.ldy = m->vocab; a.lse_part = c->lse_part;
    a.part = c->gemm_part; a.counters = c->gemm_cnt; a.part_floats = c->gemm_part_n; a.counters_n = c->gemm_cnt_n;
    a.xfrag = c->gemm_xfrag; a.xfrag_elems = c->gemm_xfrag_n;
    HIP_TRY(c, launch_gemm_bf16(a, EPI_STORE, same_shape(m, &c->tshape) ? 1 : 0, s));
    return finish_lse(c, m, rows, logits, lse, s);
  }
  HIP_TRY(c, launch_rmsnorm(0, c->h, (const float*)W[tail], c->xn, rows, m->d_model, m->rms_eps, s));
  HIP_TRY(c, launch_gemm_f32(W[tail + 1], c->xn, logits, rows, m->vocab, m->d_model, m->vocab, false, s));
  HIP_TRY(c, launch_row_lse(logits, lse, rows, m->vocab, s));
  return MTAD_OK;
}

int weights_ok(const mtad_model* m) {
  if (!m || !m->weights) return 0;
  for (int i = 0; i < 3 + 6 * m->n_layers; ++i)
    if (!m->weights[i]) return 0;
  return 1;
}

TreeView tview(const mtad_tree* t) {
  TreeView v;
  v.M = t->M;
  v.tok = t->tok;
  v.parent = t->parent;
  v.depth = t->depth;
  v.src_beam = t->src_beam;
  v.anc_mask = t->anc_mask;
  v.qref = t->qref;
  return v;
}
int tree_ok(const mtad_tree* t) { return t && t->tok && t->parent && t->depth && t->src_beam && t->anc_mask && t->qref; }

}  // namespace

extern "C" {

int mtad_create(mtad_ctx** out, const mtad_config* cfg, const mtad_model* target, const mtad_model* draft) {
  if (!out || !cfg || !target || !draft) return MTAD_EINVAL;
  if (cfg->batch < 1 || cfg->gamma < 1 || cfg->beam < 1 || cfg->max_context < 1) return MTAD_EINVAL;
  if (cfg->mode != MTAD_MODE_MTAD && cfg->mode != MTAD_MODE_MMTAD) return MTAD_EINVAL;
  if (!shape_ok(target) || !shape_ok(draft)) return MTAD_ESHAPE;
  if (target->vocab != draft->vocab) return MTAD_ESHAPE;
  if (cfg->beam > MTAD_MAX_BEAM || cfg->beam > draft->vocab) return MTAD_ESHAPE;
  if (cfg->prefill_rows < 1 || cfg->prefill_rows > MTAD_MAX_ROWS) return MTAD_ESHAPE;
  const int M = 1 + (cfg->mode == MTAD_MODE_MTAD ? cfg->gamma : cfg->gamma * cfg->beam);
  if (M > MTAD_MAX_ROWS) return MTAD_ESHAPE;
  if ((cfg->gamma + 1) + (cfg->gamma - 1) * cfg->beam > MTAD_MAX_ROWS) return MTAD_ESHAPE;  // draft rows of one iteration
  mtad_ctx* c = new (std::nothrow) mtad_ctx();
  if (!c) return MTAD_ECAP;
  memset(c, 0, sizeof(*c));
  c->cfg = *cfg;
  c->tshape = *target;
  c->dshape = *draft;
  c->tshape.weights = nullptr;
  c->dshape.weights = nullptr;
  c->M = M;
  c->draft_rows = imax(cfg->gamma + 1, cfg->beam);
  c->Rmax = imax(imax(cfg->prefill_rows, M), c->draft_rows);
  if ((int64_t)cfg->batch * c->Rmax > 256) {  // the skinny product kernels hold at most 256 rows
    delete c;
    return MTAD_ESHAPE;
  }
  c->flow_on = 1;
  if (const char* e = getenv("MTAD_FUSED_PASS")) c->flow_on = atoi(e) < 0 ? 0 : (atoi(e) > 2 ? 2 : atoi(e));
  carve(c, nullptr);
  *out = c;
  return MTAD_OK;
}

void mtad_destroy(mtad_ctx* c) { delete c; }

size_t mtad_workspace_bytes(const mtad_ctx* c) { return c ? c->ws_need : 0; }

int mtad_bind_workspace(mtad_ctx* c, void* buf, size_t bytes) {
  if (!c || !buf) return MTAD_EINVAL;
  if (((uintptr_t)buf) & 255) return MTAD_EINVAL;
  if (bytes < c->ws_need) return MTAD_ECAP;
  c->ws = (char*)buf;
  carve(c, c->ws);
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
    c->n_cus = cus;
  }
  hipError_t e = hipMemset(c->status, 0, 256);
  if (e == hipSuccess) e = hipMemset(c->attn_cnt, 0, sizeof(int) * c->attn_cnt_n);
  if (e == hipSuccess) e = hipMemset(c->gemm_cnt, 0, sizeof(int) * (size_t)c->gemm_cnt_n);
  if (e != hipSuccess) {
    c->last_hip = (int)e;
    return MTAD_EHIP;
  }
  return MTAD_OK;
}

const char* mtad_strerror(int st) {
  switch (st) {
    case MTAD_OK: return "ok";
    case MTAD_EINVAL: return "invalid argument";
    case MTAD_ESHAPE: return "unsupported shape";
    case MTAD_ECAP: return "capacity exceeded";
    case MTAD_EHIP: return "HIP error";
    case MTAD_ENOSYS: return "not implemented";
    default: return "unknown status";
  }
}

int mtad_last_hip_error(const mtad_ctx* c) { return c ? c->last_hip : 0; }

int mtad_device_status(mtad_ctx* c, uint32_t* bits, void* stream) {
  if (!c || !bits || !c->ws) return MTAD_EINVAL;
  HIP_TRY(c, hipMemcpyAsync(bits, c->status, sizeof(uint32_t), hipMemcpyDeviceToHost, (hipStream_t)stream));
  HIP_TRY(c, hipStreamSynchronize((hipStream_t)stream));
  return MTAD_OK;
}

int mtad_prefill(mtad_ctx* c, const mtad_model* model, mtad_kv* kv, const int32_t* tokens, int32_t n_tokens, void* stream) {
  if (!c || !c->ws || !weights_ok(model) || !kv_ok(kv) || !tokens || n_tokens < 0) return MTAD_EINVAL;
  if (!same_shape(model, &c->tshape) && !same_shape(model, &c->dshape)) return MTAD_ESHAPE;
  if (n_tokens > kv->page_size * kv->max_pages) return MTAD_ECAP;
  hipStream_t s = (hipStream_t)stream;
  const int R = c->cfg.prefill_rows, B = c->cfg.batch, cap = kv->page_size * kv->max_pages;
  for (int c0 = 0; c0 < n_tokens; c0 += R) {
    const int r = imin(R, n_tokens - c0);
    HIP_TRY(c, launch_prefill_rows(c->rd, kv->len, tokens, n_tokens, c0, B, r, cap, c->status, s));
    int st = decoder_pass(c, model, kv, r, s, nullptr, nullptr);
    if (st) return st;
    HIP_TRY(c, launch_advance_len(kv->len, c->rd.nspec, B, cap, s));
  }
  return MTAD_OK;
}

int mtad_draft_beam_step(mtad_ctx* c, const mtad_model* draft, mtad_kv* dkv, mtad_beam* hist, int32_t step, const mtad_state* st,
                         int32_t sample_beam, uint64_t seed, void* stream) {
  if (!c || !c->ws || !weights_ok(draft) || !kv_ok(dkv) || !hist || !hist->tok || !hist->parent || !hist->cum_logq || !st ||
      !st->catchup_tok || !st->catchup_cnt)
    return MTAD_EINVAL;
  if (step < 0 || step >= c->cfg.gamma) return MTAD_EINVAL;
  if (!same_shape(draft, &c->dshape)) return MTAD_ESHAPE;
  hipStream_t s = (hipStream_t)stream;
  const int B = c->cfg.batch, gamma = c->cfg.gamma, beam = c->cfg.beam;
  const int R = (step == 0) ? gamma + 1 : beam;
  const BeamView hv{hist->tok, hist->parent, hist->cum_logq};
  HIP_TRY(c, launch_draft_rows(c->rd, dkv->len, hv, st->catchup_tok, st->catchup_cnt, step, B, R, gamma, beam,
                               dkv->page_size * dkv->max_pages, c->status, s));
  int rc = decoder_pass(c, draft, dkv, R, s, c->dlogits, c->lse);
  if (rc) return rc;
  if (c->warp_k > 0) HIP_TRY(c, launch_warp_rows(c->dlogits, c->lse, B * R, draft->vocab, c->warp_k, c->warp_p, s));
  if (beam == 1)  // a chain drawn token by token: keep log q of each step for token-wise acceptance (mtad_accept_spd)
    HIP_TRY(c, launch_save_logq_row(c->dlogits, c->lse, st->catchup_cnt, step, B, R, gamma, draft->vocab, c->qrows, s));
  HIP_TRY(c, launch_topb(c->dlogits, c->lse, hv, st->catchup_cnt, dkv->len, step, B, R, gamma, beam, draft->vocab, sample_beam ? 1 : 0,
                         seed, c->part_key, c->part_idx, TOPB_BLOCKS, s));
  return MTAD_OK;
}

int mtad_build_tree(mtad_ctx* c, const mtad_beam* hist, int32_t mode, mtad_tree* tree, void* stream) {
  if (!c || !hist || !hist->tok || !hist->parent || !hist->cum_logq || !tree_ok(tree)) return MTAD_EINVAL;
  if (mode != MTAD_MODE_MTAD && mode != MTAD_MODE_MMTAD) return MTAD_EINVAL;
  const int M = 1 + (mode == MTAD_MODE_MTAD ? c->cfg.gamma : c->cfg.gamma * c->cfg.beam);
  if (M > MTAD_MAX_ROWS) return MTAD_ESHAPE;
  tree->M = M;
  const BeamView hv{hist->tok, hist->parent, hist->cum_logq};
  HIP_TRY(c, launch_build_tree(hv, tview(tree), c->cfg.batch, c->cfg.gamma, c->cfg.beam, mode, (hipStream_t)stream));
  return MTAD_OK;
}

int mtad_verify_tree(mtad_ctx* c, const mtad_model* target, mtad_kv* tkv, const int32_t* root_tok, const mtad_tree* tree,
                     float* logp_cond, float* row_lse, float* logits, void* stream) {
  if (!c || !c->ws || !weights_ok(target) || !kv_ok(tkv) || !root_tok || !tree_ok(tree) || !logp_cond || !row_lse || !logits)
    return MTAD_EINVAL;
  if (!same_shape(target, &c->tshape)) return MTAD_ESHAPE;
  if (tree->M < 1 || tree->M > c->Rmax) return MTAD_ESHAPE;
  hipStream_t s = (hipStream_t)stream;
  const int B = c->cfg.batch, M = tree->M;
  HIP_TRY(c, launch_verify_rows(c->rd, tkv->len, root_tok, tview(tree), B, tkv->page_size * tkv->max_pages, c->status, s));
  c->gather_tree = c->warp_k > 0 ? nullptr : tree;  // warped rows are gathered after the warp
  c->gather_out = c->warp_k > 0 ? nullptr : logp_cond;
  int rc = decoder_pass(c, target, tkv, M, s, logits, row_lse);
  const bool gathered = c->gather_out == nullptr;
  c->gather_tree = nullptr;
  c->gather_out = nullptr;
  if (rc) return rc;
  if (c->warp_k > 0) HIP_TRY(c, launch_warp_rows(logits, row_lse, B * M, target->vocab, c->warp_k, c->warp_p, s));
  if (!gathered || c->warp_k > 0) HIP_TRY(c, launch_gather_logp(logits, row_lse, tview(tree), B, target->vocab, logp_cond, s));
  return MTAD_OK;
}

int mtad_accept(mtad_ctx* c, const mtad_tree* tree, const float* logp_cond, const float* logits, int32_t vocab, const mtad_kv* tkv,
                float tau, int32_t mode, int32_t sample_bonus, uint64_t seed, mtad_accept_out* out, void* stream) {
  if (!c || !tree_ok(tree) || !logp_cond || !logits || !tkv || !tkv->len || !out || !out->eta || !out->path || !out->bonus_row ||
      !out->bonus_tok || !out->out_tok || !out->out_cnt)
    return MTAD_EINVAL;
  if (!(tau >= 0.f && tau < 1.f) || vocab < 1) return MTAD_EINVAL;
  if (mode != MTAD_MODE_MTAD && mode != MTAD_MODE_MMTAD) return MTAD_EINVAL;
  if (tree->M < 1 || tree->M > MTAD_MAX_ROWS) return MTAD_ESHAPE;
  const float log_tau = (tau > 0.f) ? (float)log((double)tau) : -INFINITY;
  const AcceptView av{out->eta, out->path, out->bonus_row, out->bonus_tok, out->out_tok, out->out_cnt};
  HIP_TRY(c, launch_accept(tview(tree), logp_cond, logits, vocab, tkv->len, log_tau, mode, c->cfg.batch, c->cfg.gamma,
                           sample_bonus ? 1 : 0, seed, av, (hipStream_t)stream));
  return MTAD_OK;
}

int mtad_accept_chain(mtad_ctx* c, const mtad_tree* tree, mtad_accept_out* out, void* stream) {
  if (!c || !tree_ok(tree) || !out || !out->eta || !out->path || !out->bonus_row || !out->bonus_tok || !out->out_tok || !out->out_cnt)
    return MTAD_EINVAL;
  if (tree->M != c->cfg.gamma + 1) return MTAD_ESHAPE;
  const AcceptView av{out->eta, out->path, out->bonus_row, out->bonus_tok, out->out_tok, out->out_cnt};
  HIP_TRY(c, launch_accept_chain(tview(tree), c->cfg.batch, c->cfg.gamma, av, (hipStream_t)stream));
  return MTAD_OK;
}

int mtad_accept_spd(mtad_ctx* c, const mtad_tree* tree, const float* logits, const float* row_lse, int32_t vocab, const mtad_kv* tkv,
                    uint64_t seed, mtad_accept_out* out, void* stream) {
  if (!c || !c->ws || !tree_ok(tree) || !logits || !row_lse || !tkv || !tkv->len || !out || !out->eta || !out->path || !out->bonus_row ||
      !out->bonus_tok || !out->out_tok || !out->out_cnt)
    return MTAD_EINVAL;
  if (c->cfg.beam != 1 || tree->M != c->cfg.gamma + 1 || vocab != c->dshape.vocab || vocab != c->tshape.vocab) return MTAD_ESHAPE;
  const AcceptView av{out->eta, out->path, out->bonus_row, out->bonus_tok, out->out_tok, out->out_cnt};
  HIP_TRY(c, launch_accept_spd(tview(tree), logits, row_lse, c->qrows, vocab, tkv->len, c->cfg.batch, c->cfg.gamma, seed, av,
                               (hipStream_t)stream));
  return MTAD_OK;
}

int mtad_kv_commit(mtad_ctx* c, mtad_kv* tkv, mtad_kv* dkv, const mtad_tree* tree, const mtad_accept_out* acc, mtad_state* st,
                   void* stream) {
  if (!c || (!tkv && !dkv) || (tkv && !kv_ok(tkv)) || (dkv && !kv_ok(dkv)) || !tree_ok(tree) || !acc || !acc->eta || !acc->path ||
      !acc->bonus_tok || !st || !st->root_tok || !st->catchup_tok || !st->catchup_cnt)
    return MTAD_EINVAL;
  if (tree->M < 1 || tree->M > MTAD_MAX_ROWS) return MTAD_ESHAPE;
  hipStream_t s = (hipStream_t)stream;
  const int B = c->cfg.batch, gamma = c->cfg.gamma, beam = c->cfg.beam;
  if (tkv)
    HIP_TRY(c, launch_kv_gather(c->tshape.dtype, view_of(tkv, &c->tshape), c->tshape.n_layers, B, acc->eta, acc->path, tree->src_beam,
                                st->catchup_cnt, tree->M, gamma, beam, 0, s));
  if (dkv)
    HIP_TRY(c, launch_kv_gather(c->dshape.dtype, view_of(dkv, &c->dshape), c->dshape.n_layers, B, acc->eta, acc->path, tree->src_beam,
                                st->catchup_cnt, tree->M, gamma, beam, 1, s));
  const AcceptView av{acc->eta, acc->path, acc->bonus_row, acc->bonus_tok, acc->out_tok, acc->out_cnt};
  HIP_TRY(c, launch_commit_state(tkv ? tkv->len : nullptr, dkv ? dkv->len : nullptr, tview(tree), av, st->root_tok, st->catchup_tok,
                                 st->catchup_cnt, B, gamma, tkv ? tkv->page_size * tkv->max_pages : 0,
                                 dkv ? dkv->page_size * dkv->max_pages : 0, s));
  return MTAD_OK;
}

// ---- component entry points (include/mtad_kernels.h) ------------------------------------------------------------

#ifdef MTAD_FLOW_PROFILE
extern "C" void* mtad_flow_profile(mtad_ctx* c) { return c ? c->flow_prof : nullptr; }
#endif

int mtad_set_warp(mtad_ctx* c, int32_t top_k, float top_p) {
  if (!c) return MTAD_EINVAL;
  if (top_k < 0 || top_k > 16 || (top_k > 0 && !(top_p > 0.f))) return MTAD_EINVAL;
  c->warp_k = top_k;
  c->warp_p = top_p;
  return MTAD_OK;
}

int mtad_k_warp_rows(float* logits, float* lse, int32_t rows, int32_t vocab, int32_t top_k, float top_p, void* stream) {
  if (!logits || !lse || rows < 1 || vocab < 1 || top_k < 1 || top_k > 16 || !(top_p > 0.f)) return MTAD_EINVAL;
  return launch_warp_rows(logits, lse, rows, vocab, top_k, top_p, (hipStream_t)stream) == hipSuccess ? MTAD_OK : MTAD_EHIP;
}

int mtad_set_fused_pass(mtad_ctx* c, int32_t on) {
  if (!c || on < 0 || on > 2) return MTAD_EINVAL;
  c->flow_on = on;
  return MTAD_OK;
}

int mtad_k_gemm(mtad_ctx* c, int32_t dtype, const void* W, const void* X, float* Y, int32_t R, int32_t N, int32_t K, int32_t ldy, int32_t accumulate,
                void* stream) {
  return mtad_k_gemm_x(c, dtype, W, X, Y, R, N, K, ldy, accumulate, MTAD_X_PLANES, stream);
}

int mtad_k_gemm_x(mtad_ctx* c, int32_t dtype, const void* W, const void* X, float* Y, int32_t R, int32_t N, int32_t K, int32_t ldy,
                  int32_t accumulate, int32_t x_order, void* stream) {
  if (!W || !X || !Y || R < 1 || N < 1 || K < 1 || ldy < N) return MTAD_EINVAL;
  if (dtype != 0 && dtype != 1) return MTAD_EINVAL;
  if (x_order != MTAD_X_PLANES && x_order != MTAD_X_FRAGMENTS) return MTAD_EINVAL;
  if (dtype == 0 && x_order != MTAD_X_PLANES) return MTAD_EINVAL;
  if (dtype == 1 && ((N % 16) || (K % 32) || (ldy % 4) || R > 256)) return MTAD_ESHAPE;
  if (dtype == 0 && (K % 4)) return MTAD_ESHAPE;
  if (dtype == 0) return launch_gemm_f32(W, X, Y, R, N, K, ldy, accumulate != 0, (hipStream_t)stream) == hipSuccess ? MTAD_OK : MTAD_EHIP;
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  a.W = (const bf16_t*)W; a.X = (const bf16_t*)X; a.R = R; a.N = N; a.K = K;
  a.Y = Y; a.ldy = ldy; a.accumulate = accumulate != 0;
  a.ncg = x_order == MTAD_X_FRAGMENTS ? (R + 7) / 8 : 0;
  if (c && c->ws) {  // a cut of the reduction dimension needs the workspace; the launchers check that the product fits it
    a.part = c->gemm_part;
    a.counters = c->gemm_cnt;
    a.part_floats = c->gemm_part_n;
    a.counters_n = c->gemm_cnt_n;
  }
  if (c && c->ws && gemm_tiled_xfrag_elems(R, K) <= c->gemm_xfrag_n) {  // the many-row kernel needs its scratch
    a.xfrag = c->gemm_xfrag;
    a.xfrag_elems = c->gemm_xfrag_n;
  }
  return launch_gemm_bf16(a, EPI_STORE, 2, (hipStream_t)stream) == hipSuccess ? MTAD_OK : MTAD_EHIP;
}

int mtad_pack_matrix(int32_t kind, const void* src, void* dst, int32_t N, int32_t K, int32_t head_dim, void* stream) {
  if (!src || !dst || src == dst || N < 16 || K < 32) return MTAD_EINVAL;
  if (kind != MTAD_PACK_PLAIN && kind != MTAD_PACK_QKV && kind != MTAD_PACK_GATE_UP) return MTAD_EINVAL;
  if ((N % 16) || (K % 32)) return MTAD_ESHAPE;
  if (kind == MTAD_PACK_QKV && (head_dim < 16 || (head_dim % 16) || (N % head_dim))) return MTAD_ESHAPE;
  if (kind == MTAD_PACK_GATE_UP && (N % 32)) return MTAD_ESHAPE;
  return launch_pack_matrix(src, dst, N, K, kind, head_dim, (hipStream_t)stream) == hipSuccess ? MTAD_OK : MTAD_EHIP;
}

int mtad_k_rmsnorm(int32_t dtype, const float* h, const float* g, void* out, int32_t rows, int32_t d, float eps, void* stream) {
  if (!h || !g || !out || rows < 1 || d < 4 || (d % 4)) return MTAD_EINVAL;
  return launch_rmsnorm(dtype, h, g, out, rows, d, eps, (hipStream_t)stream) == hipSuccess ? MTAD_OK : MTAD_EHIP;
}

int mtad_k_row_lse(const float* logits, float* lse, int32_t rows, int32_t vocab, void* stream) {
  if (!logits || !lse || rows < 1 || vocab < 1) return MTAD_EINVAL;
  return launch_row_lse(logits, lse, rows, vocab, (hipStream_t)stream) == hipSuccess ? MTAD_OK : MTAD_EHIP;
}

int mtad_k_copy(const void* src, void* dst, int64_t bytes, void* stream) {
  if (!src || !dst || bytes < 16 || (bytes % 16) || (((uintptr_t)src | (uintptr_t)dst) & 15)) return MTAD_EINVAL;
  return launch_copy(src, dst, bytes, (hipStream_t)stream) == hipSuccess ? MTAD_OK : MTAD_EHIP;
}

int mtad_k_beam_topb(mtad_ctx* c, const float* logits, const float* lse, mtad_beam* hist, int32_t step, const int32_t* catchup_cnt,
                     const int32_t* len, int32_t rows_per_seq, int32_t vocab, int32_t sample_beam, uint64_t seed, void* stream) {
  if (!c || !c->ws || !logits || !lse || !hist || !hist->tok || !hist->parent || !hist->cum_logq || !catchup_cnt || !len)
    return MTAD_EINVAL;
  if (step < 0 || step >= c->cfg.gamma || vocab < c->cfg.beam) return MTAD_EINVAL;
  if (rows_per_seq < (step == 0 ? c->cfg.gamma + 1 : c->cfg.beam)) return MTAD_EINVAL;  // the rows the kernels may read
  const BeamView hv{hist->tok, hist->parent, hist->cum_logq};
  HIP_TRY(c, launch_topb(logits, lse, hv, catchup_cnt, len, step, c->cfg.batch, rows_per_seq, c->cfg.gamma, c->cfg.beam, vocab,
                         sample_beam ? 1 : 0, seed, c->part_key, c->part_idx, TOPB_BLOCKS, (hipStream_t)stream));
  return MTAD_OK;
}

// ---- the same selection for callers that cannot allocate --------------------------------------------------------
// The two-stage top-b keeps its stage-1 winners in a scratch buffer; here that buffer is a file-scope device array
// instead of a caller's workspace.  In host code the array's name is only a stand-in: its device address is looked up
// once per device (each device holds its own copy) and only that address is handed to kernels.
namespace {
constexpr size_t STATIC_TOPB_ENTRIES = (size_t)MTAD_STATIC_TOPB_MAX_BATCH * TOPB_BLOCKS * 8;  // stage-1 winners, MAXB per block
struct StaticTopbScratch {
  float key[STATIC_TOPB_ENTRIES];
  int idx[STATIC_TOPB_ENTRIES];
};
constexpr int STATIC_MAX_DEVICES = 64;
std::mutex scratch_mu;
void* scratch_ptr[STATIC_MAX_DEVICES];  // device address of `scratch` on each device, null until first used there
}  // namespace
static __device__ __align__(256) unsigned char scratch[sizeof(StaticTopbScratch)];  // 256 KiB per device, held until the process ends

int mtad_k_beam_topb_static(const float* logits, const float* lse, mtad_beam* hist, int32_t batch, int32_t gamma, int32_t beam, int32_t step,
                            const int32_t* catchup_cnt, const int32_t* len, int32_t rows_per_seq, int32_t vocab, int32_t sample_beam,
                            uint64_t seed, void* stream) {
  if (!logits || !lse || !hist || !hist->tok || !hist->parent || !hist->cum_logq || !catchup_cnt || !len) return MTAD_EINVAL;
  if (batch < 1 || gamma < 1 || beam < 1 || step < 0 || step >= gamma || vocab < beam) return MTAD_EINVAL;
  if (rows_per_seq < (step == 0 ? gamma + 1 : beam)) return MTAD_EINVAL;
  if (beam > MTAD_MAX_BEAM || gamma > MTAD_MAX_ROWS) return MTAD_ESHAPE;
  if (batch > MTAD_STATIC_TOPB_MAX_BATCH) return MTAD_ECAP;  // the static scratch array holds no more sequences
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return MTAD_EHIP;
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return MTAD_ECAP;
  void* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[dev]) {
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MTAD_EHIP;
      scratch_ptr[dev] = p;
    }
    base = scratch_ptr[dev];
  }
  StaticTopbScratch* sc = (StaticTopbScratch*)base;
  const BeamView hv{hist->tok, hist->parent, hist->cum_logq};
  // every entry stage 2 reads is written by stage 1 of the same call: nothing needs clearing between calls
  return launch_topb(logits, lse, hv, catchup_cnt, len, step, batch, rows_per_seq, gamma, beam, vocab, sample_beam ? 1 : 0, seed, sc->key,
                     sc->idx, TOPB_BLOCKS, (hipStream_t)stream) == hipSuccess
             ? MTAD_OK
             : MTAD_EHIP;
}

}  // extern "C"
