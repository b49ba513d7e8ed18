// Integer / decision side of one MTAD iteration: row descriptors of the draft and target passes, the
// beam top-b over beam x vocab candidates (Section 2.1, Eq. 2), the tree of the target pass (Section
// 3.3), the gather of the draft tokens' log-likelihoods, joint-likelihood acceptance with the bonus
// token (Algorithm 1; Eq. 9) and the KV commit / rollback.
#include "common.h"
#include "beam.h"

namespace mtad {

// ---- counter-based noise: SplitMix64 finaliser keyed by (seed, stream, position, index) ------------
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
constexpr uint64_t GOLDEN = 0x9E3779B97F4A7C15ull;
__device__ __forceinline__ uint64_t noise_key(uint64_t seed, int stream, int position) {
  return mix64(mix64(seed ^ (GOLDEN * (uint64_t)(stream + 1))) + (uint64_t)position);
}
// standard Gumbel from the top 23 hash bits: u = (k + 1/2) / 2^23 is exact in float32
__device__ __forceinline__ float gumbel(uint64_t key, uint64_t idx) {
  const uint64_t h = mix64(key ^ (GOLDEN * (idx + 1)));
  const float u = ((float)(uint32_t)(h >> 41) + 0.5f) * 1.1920928955078125e-07f;
  return -logf(-logf(u));
}
constexpr int STREAM_BONUS = 0, STREAM_BEAM = 1, STREAM_ACCEPT = 2, STREAMS_PER_SEQ = 4;
// the uniform number behind the noise: u = (k + 1/2) / 2^23, exact in float32
__device__ __forceinline__ float uniform01(uint64_t key, uint64_t idx) {
  const uint64_t h = mix64(key ^ (GOLDEN * (idx + 1)));
  return ((float)(uint32_t)(h >> 41) + 0.5f) * 1.1920928955078125e-07f;
}

// ---- row descriptors ------------------------------------------------------------------------------

// chain mask: bits 0..r
__device__ __forceinline__ uint64_t chain_bits(int r) { return (r >= 63) ? ~0ull : ((1ull << (r + 1)) - 1ull); }

__global__ void draft_rows_kernel(RowDesc rd, const int32_t* __restrict__ len, BeamView hist, const int32_t* __restrict__ cu_tok,
                                  const int32_t* __restrict__ cu_cnt, int step, int B, int R, int gamma, int beam, int cap,
                                  uint32_t* __restrict__ status) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= B * R) return;
  const int s = idx / R, r = idx % R;
  int cnt = cu_cnt[s];
  if (cnt < 1 || cnt > gamma + 1) {
    if (r == 0) atomicOr(status, (uint32_t)ST_BAD_CATCHUP);
    cnt = 1;
  }
  const int n = len[s];
  int tok = 0, pos = 0, slot = -1;
  uint64_t mask = 0;
  if (step == 0) {
    if (r < cnt) {
      tok = cu_tok[s * (gamma + 1) + r];
      pos = n + r;
      slot = n + r;
      mask = chain_bits(r);
    }
    if (r == 0) rd.nspec[s] = cnt;
  } else {
    const int rel = cnt + (step - 1) * beam + r;
    if (rel < 64) {
      tok = hist.tok[(s * gamma + step - 1) * beam + r];
      pos = n + cnt - 1 + step;
      slot = n + rel;
      mask = chain_bits(cnt - 1) | (1ull << rel);
      int jj = r;
      for (int ii = step - 1; ii >= 1; --ii) {  // ancestors fed at steps ii = step-1 .. 1
        jj = min(max(hist.parent[(s * gamma + ii) * beam + jj], 0), beam - 1);  // caller-owned memory: stay in range
        mask |= 1ull << (cnt + (ii - 1) * beam + jj);
      }
    } else if (r == 0) {
      atomicOr(status, (uint32_t)ST_SPEC_WINDOW);
    }
    if (r == 0) rd.nspec[s] = min(64, cnt + step * beam);
  }
  if (slot >= cap) {
    atomicOr(status, (uint32_t)ST_KV_CAP);
    slot = -1;
  }
  rd.tok[idx] = tok;
  rd.pos[idx] = pos;
  rd.slot[idx] = slot;
  rd.mask[idx] = mask;
}

hipError_t launch_draft_rows(const RowDesc& rd, const int32_t* len, BeamView hist, const int32_t* cu_tok, const int32_t* cu_cnt,
                             int step, int B, int R, int gamma, int beam, int cap, uint32_t* status, hipStream_t s) {
  hipLaunchKernelGGL(draft_rows_kernel, dim3((B * R + 63) / 64), dim3(64), 0, s, rd, len, hist, cu_tok, cu_cnt, step, B, R, gamma,
                     beam, cap, status);
  return hipGetLastError();
}

__global__ void verify_rows_kernel(RowDesc rd, const int32_t* __restrict__ len, const int32_t* __restrict__ root_tok, TreeView tree,
                                   int B, int cap, uint32_t* __restrict__ status) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int M = tree.M;
  if (idx >= B * M) return;
  const int s = idx / M, r = idx % M;
  const int n = len[s];
  int slot = n + r;
  if (slot >= cap) {
    atomicOr(status, (uint32_t)ST_KV_CAP);
    slot = -1;
  }
  rd.tok[idx] = (r == 0) ? root_tok[s] : tree.tok[idx];
  rd.pos[idx] = n + tree.depth[idx];
  rd.slot[idx] = slot;
  rd.mask[idx] = tree.anc_mask[idx];
  if (r == 0) rd.nspec[s] = M;
}

hipError_t launch_verify_rows(const RowDesc& rd, const int32_t* len, const int32_t* root_tok, TreeView tree, int B, int cap,
                              uint32_t* status, hipStream_t s) {
  hipLaunchKernelGGL(verify_rows_kernel, dim3((B * tree.M + 63) / 64), dim3(64), 0, s, rd, len, root_tok, tree, B, cap, status);
  return hipGetLastError();
}

// causal chunk of a prompt: rows c0 .. c0+R-1 of tokens[B][n]
__global__ void prefill_rows_kernel(RowDesc rd, const int32_t* __restrict__ len, const int32_t* __restrict__ tokens, int n, int c0,
                                    int B, int R, int cap, uint32_t* __restrict__ status) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= B * R) return;
  const int s = idx / R, r = idx % R;
  const int base = len[s];
  int tok = 0, pos = 0, slot = -1;
  uint64_t mask = 0;
  if (c0 + r < n) {
    tok = tokens[(int64_t)s * n + c0 + r];
    pos = base + r;
    slot = base + r;
    mask = chain_bits(r);
    if (slot >= cap) {
      atomicOr(status, (uint32_t)ST_KV_CAP);
      slot = -1;
    }
  }
  rd.tok[idx] = tok;
  rd.pos[idx] = pos;
  rd.slot[idx] = slot;
  rd.mask[idx] = mask;
  if (r == 0) rd.nspec[s] = min(R, n - c0);
}

__global__ void advance_len_kernel(int32_t* len, const int32_t* __restrict__ nspec, int B, int cap) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s < B) len[s] = min(cap, len[s] + nspec[s]);
}

hipError_t launch_prefill_rows(const RowDesc& rd, const int32_t* len, const int32_t* tokens, int n, int c0, int B, int R, int cap,
                               uint32_t* status, hipStream_t s) {
  hipLaunchKernelGGL(prefill_rows_kernel, dim3((B * R + 63) / 64), dim3(64), 0, s, rd, len, tokens, n, c0, B, R, cap, status);
  return hipGetLastError();
}
hipError_t launch_advance_len(int32_t* len, const int32_t* nspec, int B, int cap, hipStream_t s) {
  hipLaunchKernelGGL(advance_len_kernel, dim3((B + 63) / 64), dim3(64), 0, s, len, nspec, B, cap);
  return hipGetLastError();
}

// ---- beam top-b -----------------------------------------------------------------------------------

constexpr int MAXB = 8;

struct TopList {
  float key[MAXB];
  int idx[MAXB];
};
__device__ __forceinline__ bool better(float k1, int i1, float k2, int i2) { return k1 > k2 || (k1 == k2 && i1 < i2); }

__device__ __forceinline__ void list_init(TopList& L) {
#pragma unroll
  for (int p = 0; p < MAXB; ++p) { L.key[p] = -INFINITY; L.idx[p] = 0x7FFFFFFF; }
}
// keep the b best (sorted, best first); positions >= b stay empty
__device__ __forceinline__ void list_insert(TopList& L, int b, float k, int i) {
#pragma unroll
  for (int p = MAXB - 1; p >= 0; --p) {
    if (p == b - 1) {
      if (!better(k, i, L.key[p], L.idx[p])) return;
      L.key[p] = k;
      L.idx[p] = i;
    }
    if (p < b - 1) {
      if (better(L.key[p + 1], L.idx[p + 1], L.key[p], L.idx[p])) {
        const float tk = L.key[p]; const int ti = L.idx[p];
        L.key[p] = L.key[p + 1]; L.idx[p] = L.idx[p + 1];
        L.key[p + 1] = tk; L.idx[p + 1] = ti;
      }
    }
  }
}
__device__ __forceinline__ void list_pop(TopList& L) {
#pragma unroll
  for (int p = 0; p < MAXB - 1; ++p) { L.key[p] = L.key[p + 1]; L.idx[p] = L.idx[p + 1]; }
  L.key[MAXB - 1] = -INFINITY;
  L.idx[MAXB - 1] = 0x7FFFFFFF;
}

// block-wide argmax of (key, idx) over up to 1024 threads (shk, shi: 16 entries), ties to the lowest idx; result to every thread
__device__ __forceinline__ void block_best(float& k, int& i, float* shk, int* shi) {
  for (int off = 32; off > 0; off >>= 1) {
    const float ok = __shfl_xor(k, off, 64);
    const int oi = __shfl_xor(i, off, 64);
    if (better(ok, oi, k, i)) { k = ok; i = oi; }
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { shk[threadIdx.x >> 6] = k; shi[threadIdx.x >> 6] = i; }
  __syncthreads();
  k = shk[0]; i = shi[0];
  const int nw = (int)blockDim.x >> 6;
  for (int w = 1; w < nw; ++w)
    if (better(shk[w], shi[w], k, i)) { k = shk[w]; i = shi[w]; }
}

// The same for a workgroup of exactly 1024 threads with the second level on the shuffle network of wave 0 (16 entries):
// shorter than 15 serial comparisons in every thread when it runs many times in a row.  shk, shi: 17 entries.
__device__ __forceinline__ void block_best_1024(float& k, int& i, float* shk, int* shi) {
  for (int off = 32; off > 0; off >>= 1) {
    const float ok = __shfl_xor(k, off, 64);
    const int oi = __shfl_xor(i, off, 64);
    if (better(ok, oi, k, i)) { k = ok; i = oi; }
  }
  if ((threadIdx.x & 63) == 0) { shk[threadIdx.x >> 6] = k; shi[threadIdx.x >> 6] = i; }
  __syncthreads();
  if (threadIdx.x < 64) {
    float k2 = shk[threadIdx.x & 15];
    int i2 = shi[threadIdx.x & 15];
    for (int off = 8; off > 0; off >>= 1) {
      const float ok = __shfl_xor(k2, off, 64);
      const int oi = __shfl_xor(i2, off, 64);
      if (better(ok, oi, k2, i2)) { k2 = ok; i2 = oi; }
    }
    if (threadIdx.x == 0) { shk[16] = k2; shi[16] = i2; }
  }
  __syncthreads();
  k = shk[16];
  i = shi[16];
}

// b rounds of "best head wins and is popped"; thread 0 receives the winners in order
__device__ __forceinline__ void block_merge(TopList& L, int b, float* out_key, int* out_idx, float* shk, int* shi) {
  for (int j = 0; j < b; ++j) {
    float k = L.key[0];
    int i = L.idx[0];
    block_best(k, i, shk, shi);
    if (L.idx[0] == i && i != 0x7FFFFFFF) list_pop(L);  // candidate indices are unique, so exactly one owner
    if (threadIdx.x == 0) { out_key[j] = k; out_idx[j] = i; }
  }
}

// score of candidate (live beam r, token v): cum_logq[r] + (logit - lse), float32, in this order
__device__ __forceinline__ float cand_score(const float* logits, const float* lse, const float* cum, int row0, int r, int v, int V) {
  const int row = row0 + r;
  return cum[r] + (logits[(int64_t)row * V + v] - lse[row]);
}

// stage 1: grid (G, B); block g scans its slice of the n_live*V candidates
__global__ __launch_bounds__(256) void topb_stage1_kernel(const float* __restrict__ logits, const float* __restrict__ lse, BeamView hist,
                                                          const int32_t* __restrict__ cu_cnt, const int32_t* __restrict__ len, int step,
                                                          int R, int gamma, int beam, int V, int sample, uint64_t seed,
                                                          float* __restrict__ part_key, int* __restrict__ part_idx) {
  __shared__ float shk[4];
  __shared__ int shi[4];
  __shared__ float cum_s[MAXB];
  __shared__ float okey[MAXB];
  __shared__ int oidx[MAXB];
  const int s = blockIdx.y, G = gridDim.x;
  const int n_live = (step == 0) ? 1 : beam;
  int cnt = cu_cnt[s];
  if (cnt < 1 || cnt > gamma + 1) cnt = 1;
  const int row0 = s * R + ((step == 0) ? cnt - 1 : 0);  // step 0: the last catch-up row carries the context distribution
  if (threadIdx.x < MAXB)
    cum_s[threadIdx.x] = (step == 0 || (int)threadIdx.x >= beam) ? 0.f : hist.cum[(s * gamma + step - 1) * beam + threadIdx.x];
  __syncthreads();
  const int total = n_live * V;
  const int per = (total + G - 1) / G;
  const int c0 = blockIdx.x * per, c1 = min(total, c0 + per);
  const uint64_t nk = noise_key(seed, s * STREAMS_PER_SEQ + STREAM_BEAM, len[s] + cnt + step);
  TopList L;
  list_init(L);
  for (int c = c0 + threadIdx.x; c < c1; c += 256) {
    const int r = c / V, v = c % V;
    float k = cand_score(logits, lse, cum_s, row0, r, v, V);
    if (sample) k += gumbel(nk, (uint64_t)c);
    if (!(k == k)) k = -INFINITY;  // a NaN score never wins and never leaves an empty slot behind
    list_insert(L, beam, k, c);
  }
  block_merge(L, beam, okey, oidx, shk, shi);
  __syncthreads();
  if (threadIdx.x < beam) {
    part_key[(s * G + blockIdx.x) * MAXB + threadIdx.x] = okey[threadIdx.x];
    part_idx[(s * G + blockIdx.x) * MAXB + threadIdx.x] = oidx[threadIdx.x];
  }
}

// stage 2: grid (B); merge G*beam partial winners, write the survivors of this step, best first
__global__ __launch_bounds__(256) void topb_stage2_kernel(const float* __restrict__ logits, const float* __restrict__ lse, BeamView hist,
                                                          const int32_t* __restrict__ cu_cnt, int step, int R, int gamma, int beam,
                                                          int V, int G, const float* __restrict__ part_key,
                                                          const int* __restrict__ part_idx) {
  __shared__ float shk[4];
  __shared__ int shi[4];
  __shared__ float cum_s[MAXB];
  __shared__ float okey[MAXB];
  __shared__ int oidx[MAXB];
  const int s = blockIdx.x;
  int cnt = cu_cnt[s];
  if (cnt < 1 || cnt > gamma + 1) cnt = 1;
  const int row0 = s * R + ((step == 0) ? cnt - 1 : 0);
  if (threadIdx.x < MAXB)
    cum_s[threadIdx.x] = (step == 0 || (int)threadIdx.x >= beam) ? 0.f : hist.cum[(s * gamma + step - 1) * beam + threadIdx.x];
  TopList L;
  list_init(L);
  for (int e = threadIdx.x; e < G * beam; e += 256) {
    const int g = e / beam, j = e % beam;
    const int i = part_idx[(s * G + g) * MAXB + j];
    if (i != 0x7FFFFFFF) list_insert(L, beam, part_key[(s * G + g) * MAXB + j], i);
  }
  block_merge(L, beam, okey, oidx, shk, shi);
  __syncthreads();
  if (threadIdx.x < beam) {
    int c = oidx[threadIdx.x];
    if (c < 0 || c >= ((step == 0) ? 1 : beam) * V) c = 0;  // only reachable with non-finite logits: stay in bounds
    const int o = (s * gamma + step) * beam + threadIdx.x;
    const int r = c / V, v = c % V;
    hist.tok[o] = v;
    hist.parent[o] = r;
    hist.cum[o] = cand_score(logits, lse, cum_s, row0, r, v, V);  // the stored likelihood carries no noise
  }
}

hipError_t launch_topb(const float* logits, const float* lse, BeamView hist, const int32_t* cu_cnt, const int32_t* len, int step,
                       int B, int R, int gamma, int beam, int V, int sample, uint64_t seed, float* part_key, int* part_idx, int G,
                       hipStream_t s) {
  hipLaunchKernelGGL(topb_stage1_kernel, dim3(G, B), dim3(256), 0, s, logits, lse, hist, cu_cnt, len, step, R, gamma, beam, V, sample,
                     seed, part_key, part_idx);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(topb_stage2_kernel, dim3(B), dim3(256), 0, s, logits, lse, hist, cu_cnt, step, R, gamma, beam, V, G, part_key,
                     part_idx);
  return hipGetLastError();
}

// ---- tree of the target pass --------------------------------------------------------------------------

__global__ void build_tree_kernel(BeamView hist, TreeView tree, int B, int gamma, int beam, int mode) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= B) return;
  const int M = tree.M;
  const int32_t* htok = hist.tok + (int64_t)s * gamma * beam;
  const int32_t* hpar = hist.parent + (int64_t)s * gamma * beam;
  const float* hcum = hist.cum + (int64_t)s * gamma * beam;
  // x**: final beam with the largest stored likelihood (first maximum), traced back through the parents
  int j = 0;
  for (int k = 1; k < beam; ++k)
    if (hcum[(gamma - 1) * beam + k] > hcum[(gamma - 1) * beam + j]) j = k;
  int beams[MTAD_MAX_GAMMA];
  for (int i = gamma - 1; i >= 0; --i) {
    beams[i] = j;
    j = min(max(hpar[i * beam + j], 0), beam - 1);  // caller-owned memory: stay in range
  }
  int32_t* tok = tree.tok + (int64_t)s * M;
  int32_t* par = tree.parent + (int64_t)s * M;
  int32_t* dep = tree.depth + (int64_t)s * M;
  int32_t* src = tree.src_beam + (int64_t)s * M;
  uint64_t* am = tree.anc_mask + (int64_t)s * M;
  tok[0] = -1; par[0] = -1; dep[0] = 0; src[0] = -1; am[0] = 1ull;
  for (int i = 0; i < gamma; ++i) tree.qref[s * gamma + i] = hcum[i * beam + beams[i]];
  if (mode == 0) {
    for (int i = 0; i < gamma; ++i) {
      const int r = i + 1;
      tok[r] = htok[i * beam + beams[i]];
      par[r] = i;
      dep[r] = i + 1;
      src[r] = beams[i];
      am[r] = chain_bits(r);
    }
  } else {
    for (int i = 0; i < gamma; ++i)
      for (int k = 0; k < beam; ++k) {
        const int r = 1 + i * beam + k;
        const int p = (i == 0) ? 0 : 1 + (i - 1) * beam + min(max(hpar[i * beam + k], 0), beam - 1);
        tok[r] = htok[i * beam + k];
        par[r] = p;
        dep[r] = i + 1;
        src[r] = k;
        am[r] = am[p] | (1ull << r);
      }
  }
}

hipError_t launch_build_tree(BeamView hist, TreeView tree, int B, int gamma, int beam, int mode, hipStream_t s) {
  hipLaunchKernelGGL(build_tree_kernel, dim3((B + 63) / 64), dim3(64), 0, s, hist, tree, B, gamma, beam, mode);
  return hipGetLastError();
}

// ---- gather of the draft tokens' conditional log-likelihoods ----------------------------------------------

__global__ void gather_logp_kernel(const float* __restrict__ logits, const float* __restrict__ lse, TreeView tree, int B, int V,
                                   float* __restrict__ logp_cond) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int M = tree.M;
  if (idx >= B * M) return;
  const int s = idx / M, c = idx % M;
  float out = 0.f;
  if (c > 0) {
    const int p = tree.parent[idx], t = tree.tok[idx];
    if (p >= 0 && p < M && t >= 0 && t < V) out = logits[((int64_t)s * M + p) * V + t] - lse[s * M + p];
  }
  logp_cond[idx] = out;
}

hipError_t launch_gather_logp(const float* logits, const float* lse, TreeView tree, int B, int V, float* logp_cond, hipStream_t s) {
  hipLaunchKernelGGL(gather_logp_kernel, dim3((B * tree.M + 63) / 64), dim3(64), 0, s, logits, lse, tree, B, V, logp_cond);
  return hipGetLastError();
}

// ---- joint-likelihood acceptance and bonus token -----------------------------------------------------------

__global__ __launch_bounds__(1024) void accept_kernel(TreeView tree, const float* __restrict__ logp_cond, const float* __restrict__ logits,
                                                     int V, const int32_t* __restrict__ len, float log_tau, int mode, int gamma,
                                                     int sample, uint64_t seed, AcceptView out) {
  __shared__ float joint[MTAD_MAX_ROWS];
  __shared__ int sel[2];  // eta, node
  __shared__ float shk[16];
  __shared__ int shi[16];
  const int s = blockIdx.x, M = tree.M;
  const int32_t* par = tree.parent + (int64_t)s * M;
  const int32_t* dep = tree.depth + (int64_t)s * M;
  const int32_t* tok = tree.tok + (int64_t)s * M;
  if (threadIdx.x == 0) {
    // log p of every branch: conditionals summed from the first level down (parents precede children)
    joint[0] = 0.f;
    int eta = 0, node = 0;
    float best = -INFINITY;
    for (int c = 1; c < M; ++c) {
      const int p = par[c];
      const float jp = joint[(p >= 0 && p < c) ? p : 0] + logp_cond[(int64_t)s * M + c];
      joint[c] = jp;
      const int i = dep[c];
      if (i < 1 || i > gamma) continue;
      const float diff = jp - tree.qref[s * gamma + i - 1];
      if (mode == 0) {
        if (fminf(0.f, diff) > log_tau && i >= eta) { eta = i; node = c; }  // rows of a chain come in depth order
      } else {
        if (diff >= log_tau && (i > eta || (i == eta && jp > best))) { eta = i; node = c; best = jp; }
      }
    }
    sel[0] = eta;
    sel[1] = node;
    out.eta[s] = eta;
    out.bonus_row[s] = node;
    out.out_cnt[s] = eta + 1;
    for (int i = 0; i < gamma; ++i) out.path[s * gamma + i] = -1;
    int c = node;
    for (int i = eta; i >= 1 && c > 0; --i) {
      out.path[s * gamma + i - 1] = c;
      out.out_tok[s * (gamma + 1) + i - 1] = tok[c];
      c = par[c];
    }
  }
  __syncthreads();
  const int eta = sel[0], node = sel[1];
  const float* row = logits + ((int64_t)s * M + node) * V;
  const uint64_t nk = noise_key(seed, s * STREAMS_PER_SEQ + STREAM_BONUS, len[s] + 1 + eta);
  float bk = -INFINITY;
  int bi = 0x7FFFFFFF;
  for (int v = threadIdx.x; v < V; v += (int)blockDim.x) {
    float k = row[v];
    if (sample) k += gumbel(nk, (uint64_t)v);
    if (better(k, v, bk, bi)) { bk = k; bi = v; }
  }
  block_best(bk, bi, shk, shi);
  if (bi < 0 || bi >= V) bi = 0;  // only reachable with non-finite logits: stay in the vocabulary
  if (threadIdx.x == 0) {
    out.bonus_tok[s] = bi;
    out.out_tok[s * (gamma + 1) + eta] = bi;
  }
}

hipError_t launch_accept(TreeView tree, const float* logp_cond, const float* logits, int V, const int32_t* len, float log_tau, int mode,
                         int B, int gamma, int sample, uint64_t seed, AcceptView out, hipStream_t s) {
  hipLaunchKernelGGL(accept_kernel, dim3(B), dim3(1024), 0, s, tree, logp_cond, logits, V, len, log_tau, mode, gamma, sample, seed, out);
  return hipGetLastError();
}

// ---- vanilla speculative decoding (Section 2.2), the baseline: token-wise acceptance and the correction token ------------

// log q(. | prefix) of the one live beam of a draft step (beam width 1), kept for the accept step: row r of the step's
// logits (the last catch-up row at step 0, row 0 afterwards) minus its logsumexp.  grid (blocks, B).
__global__ __launch_bounds__(256) void save_logq_row_kernel(const float* __restrict__ logits, const float* __restrict__ lse,
                                                            const int32_t* __restrict__ cu_cnt, int step, int R, int gamma, int V,
                                                            float* __restrict__ qrows) {
  const int s = blockIdx.y;
  int r = 0;
  if (step == 0) {
    int cnt = cu_cnt[s];
    if (cnt < 1 || cnt > gamma + 1) cnt = 1;
    r = cnt - 1;
  }
  const float* row = logits + ((int64_t)s * R + r) * V;
  const float l = lse[s * R + r];
  float* out = qrows + ((int64_t)s * gamma + step) * V;
  for (int v = blockIdx.x * blockDim.x + threadIdx.x; v < V; v += gridDim.x * blockDim.x) out[v] = row[v] - l;
}

hipError_t launch_save_logq_row(const float* logits, const float* lse, const int32_t* cu_cnt, int step, int B, int R, int gamma, int V,
                                float* qrows, hipStream_t s) {
  hipLaunchKernelGGL(save_logq_row_kernel, dim3(8, B), dim3(256), 0, s, logits, lse, cu_cnt, step, R, gamma, V, qrows);
  return hipGetLastError();
}

// One workgroup per sequence.  Thread 0 walks the chain: x_t passes when log u_t < min(0, log p(x_t) - log q(x_t)), u_t
// keyed by the token's absolute position; the tokens before the first failure are kept.  Then the whole workgroup draws
// the next token: from the residual distribution norm(max(0, p - q)) of the failed position, or, when every token passed,
// from the target's row after the last one; both as argmax(log weight + Gumbel noise).
__global__ __launch_bounds__(1024) void accept_spd_kernel(TreeView tree, const float* __restrict__ logits, const float* __restrict__ lse,
                                                         const float* __restrict__ qrows, int V, const int32_t* __restrict__ len, int gamma,
                                                         uint64_t seed, AcceptView out) {
  __shared__ int eta_s;
  __shared__ float shk[16];
  __shared__ int shi[16];
  const int s = blockIdx.x, M = tree.M;
  const int32_t* tok = tree.tok + (int64_t)s * M;
  if (threadIdx.x == 0) {
    int eta = gamma;
    for (int t = 1; t <= gamma; ++t) {
      int x = tok[t];
      if (x < 0 || x >= V) x = 0;
      const float lp = logits[((int64_t)s * M + t - 1) * V + x] - lse[s * M + t - 1];
      const float lq = qrows[((int64_t)s * gamma + t - 1) * V + x];
      const float u = uniform01(noise_key(seed, s * STREAMS_PER_SEQ + STREAM_ACCEPT, len[s] + t), 0);
      if (!(logf(u) < fminf(0.f, lp - lq))) { eta = t - 1; break; }
    }
    eta_s = eta;
    out.eta[s] = eta;
    out.bonus_row[s] = eta;
    out.out_cnt[s] = eta + 1;
    for (int i = 0; i < gamma; ++i) out.path[s * gamma + i] = i < eta ? i + 1 : -1;
    for (int i = 0; i < eta; ++i) out.out_tok[s * (gamma + 1) + i] = tok[i + 1];
  }
  __syncthreads();
  const int eta = eta_s;
  const float* prow = logits + ((int64_t)s * M + eta) * V;
  const float pl = lse[s * M + eta];
  const float* qrow = qrows + ((int64_t)s * gamma + (eta < gamma ? eta : 0)) * V;
  const uint64_t nk = noise_key(seed, s * STREAMS_PER_SEQ + STREAM_BONUS, len[s] + 1 + eta);
  float bk = -INFINITY;
  int bi = 0x7FFFFFFF;
  for (int v = threadIdx.x; v < V; v += (int)blockDim.x) {
    const float lp = prow[v] - pl;
    float k;
    if (eta < gamma) {
      const float w = expf(lp) - expf(qrow[v]);
      k = w > 0.f ? logf(w) : -INFINITY;
    } else {
      k = lp;
    }
    k += gumbel(nk, (uint64_t)v);
    if (better(k, v, bk, bi)) { bk = k; bi = v; }
  }
  block_best(bk, bi, shk, shi);
  if (bi < 0 || bi >= V) bi = 0;  // only reachable with non-finite rows: stay in the vocabulary
  if (threadIdx.x == 0) {
    out.bonus_tok[s] = bi;
    out.out_tok[s * (gamma + 1) + eta] = bi;
  }
}

hipError_t launch_accept_spd(TreeView tree, const float* logits, const float* lse, const float* qrows, int V, const int32_t* len, int B,
                             int gamma, uint64_t seed, AcceptView out, hipStream_t s) {
  hipLaunchKernelGGL(accept_spd_kernel, dim3(B), dim3(1024), 0, s, tree, logits, lse, qrows, V, len, gamma, seed, out);
  return hipGetLastError();
}

// ---- warped distributions -------------------------------------------------------------------------------------

// One workgroup per logits row: the row becomes the row of log p~ of the warped distribution (appendix
// "Hyper-parameter Details": the top_k most likely tokens, normalised; of those, in descending order, the shortest
// prefix whose cumulative probability exceeds top_p; normalised again), minus infinity outside the support, and the
// row's logsumexp becomes 0, so that every consumer of (logits, lse) rows works on p~ unchanged.  The top_k tokens
// are found by top_k rounds of a workgroup-wide argmax over every thread's best remaining entry; after a round only the
// winner's owner looks for its next best, among its entries that rank after the winner (value descending, token id
// ascending): no bookkeeping of removed entries.  The ten-element arithmetic runs on one thread
// in a fixed order (float32, sums in descending order of probability).
constexpr int WARP_MAXK = 16;
__global__ __launch_bounds__(1024) void warp_rows_kernel(float* __restrict__ logits, float* __restrict__ lse, int V, int top_k, float top_p) {
  __shared__ float shk[17];
  __shared__ int shi[17];
  __shared__ float tv[WARP_MAXK];
  __shared__ int ti[WARP_MAXK];
  __shared__ int keep_s;
  float* row = logits + (int64_t)blockIdx.x * V;
  const int k = min(min(top_k, WARP_MAXK), V);
  // the first 32768 entries of the row live in registers for all rounds (entry tid + 1024*j in x[j]); longer rows read
  // the rest from memory in every round
  constexpr int PT = 32;
  float x[PT];
#pragma unroll
  for (int j = 0; j < PT; ++j) {
    const int v = (int)threadIdx.x + 1024 * j;
    float t = v < V ? row[v] : -INFINITY;
    x[j] = (t == t) ? t : -INFINITY;                                // a NaN logit ranks last
  }
  // this thread's best entry among those that rank after (pv, pi) (value descending, token id ascending)
  auto local_best = [&](float pv, int pi, float& bk, int& bi) {
    bk = -INFINITY;
    bi = 0x7FFFFFFF;
#pragma unroll
    for (int j = 0; j < PT; ++j) {
      const int v = (int)threadIdx.x + 1024 * j;
      const bool after = x[j] < pv || (x[j] == pv && v > pi);
      if (v < V && after && better(x[j], v, bk, bi)) { bk = x[j]; bi = v; }
    }
    for (int v = (int)threadIdx.x + 1024 * PT; v < V; v += 1024) {
      float t = row[v];
      if (!(t == t)) t = -INFINITY;
      const bool after = t < pv || (t == pv && v > pi);
      if (after && better(t, v, bk, bi)) { bk = t; bi = v; }
    }
  };
  float lk;
  int li;
  local_best(INFINITY, -1, lk, li);
  for (int r = 0; r < k; ++r) {
    float bk = lk;
    int bi = li;
    block_best_1024(bk, bi, shk, shi);  // its first barrier also orders this round after the previous round's reads
    if (threadIdx.x == 0) { tv[r] = bk; ti[r] = bi; }
    // only the winner's owner has lost its best entry: all its other entries rank after the winner
    if (li == bi && bi != 0x7FFFFFFF) local_best(bk, bi, lk, li);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float e[WARP_MAXK], p[WARP_MAXK];
    float S = 0.f;
    for (int i = 0; i < k; ++i) { e[i] = expf(tv[i] - tv[0]); S += e[i]; }
    float c = 0.f;
    int K = k;
    for (int i = 0; i < k; ++i) {
      p[i] = e[i] / S;
      c += p[i];
      if (K == k && c > top_p) K = i + 1;
    }
    float s2 = 0.f;
    for (int i = 0; i < K; ++i) s2 += p[i];
    for (int i = 0; i < K; ++i) tv[i] = logf(p[i] / s2);
    keep_s = K;
    lse[blockIdx.x] = 0.f;
  }
  __syncthreads();
  for (int v = threadIdx.x; v < V; v += (int)blockDim.x) row[v] = -INFINITY;
  __syncthreads();
  if ((int)threadIdx.x < keep_s && ti[threadIdx.x] >= 0 && ti[threadIdx.x] < V) row[ti[threadIdx.x]] = tv[threadIdx.x];
}

hipError_t launch_warp_rows(float* logits, float* lse, int rows, int V, int top_k, float top_p, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(warp_rows_kernel, dim3(rows), dim3(1024), 0, s, logits, lse, V, top_k, top_p);
  return hipGetLastError();
}

// ---- KV commit / rollback -------------------------------------------------------------------------------------

// grid (n_layers, B, 2): z = 0 keys, 1 values.  Every thread owns a fixed set of element offsets within a
// token's K (or V) and moves them for path depth 1, 2, ... in order; a destination slot is never the source
// of a later move, and earlier sources have been read already, so the in-place gather is race free.
template <typename T>
__global__ __launch_bounds__(256) void kv_gather_kernel(KvView kv, const int32_t* __restrict__ eta_p, const int32_t* __restrict__ path,
                                                        const int32_t* __restrict__ src_beam, const int32_t* __restrict__ cu_cnt,
                                                        int M, int gamma, int beam, int is_draft) {
  const int layer = blockIdx.x, s = blockIdx.y;
  T* base = (T*)(blockIdx.z ? kv.v : kv.k) + (int64_t)layer * kv.layer_stride;
  const int n = kv.len[s];
  const int eta = eta_p[s];
  const int row_elems = kv.n_kv_heads * kv.head_dim;
  const int cap = kv_capacity(kv);
  int cnt = 0, depth_max = eta;
  if (is_draft) {
    cnt = cu_cnt[s];
    if (cnt < 1 || cnt > gamma + 1) cnt = 1;
    depth_max = min(eta, gamma - 1);
  }
  for (int i = 1; i <= depth_max; ++i) {
    const int row = path[s * gamma + i - 1];
    if (row < 1 || row >= M) return;
    int src, dst;
    if (is_draft) {
      src = n + cnt + (i - 1) * beam + src_beam[s * M + row];
      dst = n + cnt - 1 + i;
    } else {
      src = n + row;
      dst = n + i;
    }
    if (src == dst) continue;
    if (src >= cap || dst >= cap) return;
    const T* sp = base + kv_token_offset(kv, s, src);
    T* dp = base + kv_token_offset(kv, s, dst);
    for (int e = threadIdx.x; e < row_elems; e += 256) dp[e] = sp[e];
  }
}

hipError_t launch_kv_gather(int dtype, KvView kv, int n_layers, int B, const int32_t* eta, const int32_t* path, const int32_t* src_beam,
                            const int32_t* cu_cnt, int M, int gamma, int beam, int is_draft, hipStream_t s) {
  dim3 grid(n_layers, B, 2);
  if (dtype == 1) hipLaunchKernelGGL((kv_gather_kernel<bf16_t>), grid, dim3(256), 0, s, kv, eta, path, src_beam, cu_cnt, M, gamma, beam, is_draft);
  else hipLaunchKernelGGL((kv_gather_kernel<float>), grid, dim3(256), 0, s, kv, eta, path, src_beam, cu_cnt, M, gamma, beam, is_draft);
  return hipGetLastError();
}

// Multi-token joint decoding (Section 3.1): the chain of the beam search is the output.  Written as an accept record
// whose last token plays the part of the bonus token: the first gamma - 1 tokens were run by the beam steps (their rows
// are gathered by the commit), the last one was not and becomes the pending token.
__global__ void accept_chain_kernel(TreeView tree, int B, int gamma, AcceptView out) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= B) return;
  const int32_t* tok = tree.tok + (int64_t)s * tree.M;
  out.eta[s] = gamma - 1;
  out.bonus_row[s] = gamma - 1;
  out.bonus_tok[s] = tok[gamma];
  out.out_cnt[s] = gamma;
  for (int i = 0; i < gamma; ++i) {
    out.path[s * gamma + i] = i < gamma - 1 ? i + 1 : -1;
    out.out_tok[s * (gamma + 1) + i] = tok[i + 1];
  }
}

hipError_t launch_accept_chain(TreeView tree, int B, int gamma, AcceptView out, hipStream_t s) {
  hipLaunchKernelGGL(accept_chain_kernel, dim3((B + 63) / 64), dim3(64), 0, s, tree, B, gamma, out);
  return hipGetLastError();
}

// lengths and the state of the next iteration
__global__ void commit_state_kernel(int32_t* tlen, int32_t* dlen, TreeView tree, AcceptView acc, int32_t* root_tok, int32_t* cu_tok,
                                    int32_t* cu_cnt, int B, int gamma, int tcap, int dcap) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= B) return;
  const int eta = acc.eta[s], t = acc.bonus_tok[s];
  if (tlen) tlen[s] = min(tcap, tlen[s] + eta + 1);
  if (dlen) {
    int cnt = cu_cnt[s];
    if (cnt < 1 || cnt > gamma + 1) cnt = 1;
    dlen[s] = min(dcap, dlen[s] + cnt + min(eta, gamma - 1));
  }
  root_tok[s] = t;
  if (eta == gamma) {
    const int row = acc.path[s * gamma + gamma - 1];
    cu_tok[s * (gamma + 1) + 0] = (row >= 0 && row < tree.M) ? tree.tok[(int64_t)s * tree.M + row] : 0;
    cu_tok[s * (gamma + 1) + 1] = t;
    cu_cnt[s] = 2;
  } else {
    cu_tok[s * (gamma + 1) + 0] = t;
    cu_cnt[s] = 1;
  }
}

hipError_t launch_commit_state(int32_t* tlen, int32_t* dlen, TreeView tree, AcceptView acc, int32_t* root_tok, int32_t* cu_tok,
                               int32_t* cu_cnt, int B, int gamma, int tcap, int dcap, hipStream_t s) {
  hipLaunchKernelGGL(commit_state_kernel, dim3((B + 63) / 64), dim3(64), 0, s, tlen, dlen, tree, acc, root_tok, cu_tok, cu_cnt, B, gamma,
                     tcap, dcap);
  return hipGetLastError();
}

}  // namespace mtad
