// Tree-masked paged attention for bf16 models (half-precision K/V cache), few query rows per sequence
// (Section 3.3: tree attention gives every tree token its conditional likelihood in one pass).
//
// Work item = (key split, head, chunk of 8 query rows, sequence) = one workgroup of 8 waves.  The keys of the item
// are cut into 32-key tiles dealt round-robin to the waves; every wave runs its own online softmax over its tiles
// and the 8 waves merge through LDS at the end.  A context of up to 256 keys is one workgroup, which writes the
// attention output itself; longer contexts use one split per 256 keys and the last-arriver merge of the generic
// kernel (same partial layout, same fixed merge order).
//
// Scores are computed transposed, S^T = K Q^T, on the matrix cores: the A operand of v_mfma_f32_16x16x32_f16 wants,
// per lane, 8 consecutive dims of one key = 16 contiguous bytes of a cache row, so K goes from global memory
// straight into the operand registers; Q^T (B operand) is the float32 query split into two half terms (hi + lo, two
// MFMAs), which keeps the product at float32 accuracy.  The result leaves lane (g, r) with the scores of row r for
// 8 of the tile's keys, which is what the per-row softmax needs (two cross-lane steps).  P V runs on the vector
// ALU: lane = (8-dim chunk of the head, key subgroup); probabilities reach it through a wave-private LDS tile.
// Loads are issued a tile ahead: K of the next tile is requested before the scores of this one are computed, and
// V of a tile before its scores, so that one memory latency is exposed per workgroup, not one per tile.
#include "common.h"

namespace mtad {

namespace {

constexpr int AW = 8;        // waves per workgroup
constexpr int ARB = 8;       // query rows per work item
constexpr int ATK = 32;      // keys per tile
constexpr int KEYS_PER_SPLIT = 256;  // keys per workgroup when splits are available: one 32-key tile per wave (measured best at 512 keys)

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

union KFrag {
  uint4 u;
  half8 h;
};

template <int HD>
struct MfmaAttnSmem {
  float p[AW][ATK][ARB];       // probabilities of the wave's current tile, [key][row]
  float alpha[AW][ARB];        // rescale factor of the running output, per row
  float o[AW][ARB][HD];        // per-wave outputs for the final merge
  float m[AW][ARB], l[AW][ARB];
  int last;
};

__device__ __forceinline__ float xmax(float v, int off) { return fmaxf(v, __shfl_xor(v, off, 64)); }
__device__ __forceinline__ float xsum(float v, int off) { return v + __shfl_xor(v, off, 64); }

// physical token index (page * page_size + offset) of logical position pos; pages outside the pool read page 0
__device__ __forceinline__ int token_index(const KvView& kv, int seq, int pos) {
  int page = kv.page_table[(int64_t)seq * kv.max_pages + pos / kv.page_size];
  page = (page < 0 || page >= kv.n_pages) ? 0 : page;
  return page * kv.page_size + pos % kv.page_size;
}

template <int HD>
__global__ __launch_bounds__(AW * 64) void tree_attn_mfma_kernel(const float* __restrict__ q, int q_stride, RowDesc rd, KvView kv, int layer,
                                                               int R, int n_heads, int n_chunks, float scale, float* __restrict__ partial,
                                                               int n_splits, int* __restrict__ counters, bf16_t* __restrict__ out) {
  constexpr int KS = HD / 32;      // k-steps of the score product
  constexpr int CH = HD / 8;       // 8-dim chunks of a head
  constexpr int SG = 64 / CH;      // key subgroups in the P V phase
  constexpr int KPS = ATK / SG;    // keys per subgroup and tile
  __shared__ MfmaAttnSmem<HD> sm;

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int split = blockIdx.x, head = blockIdx.y / n_chunks, chunk = blockIdx.y % n_chunks, seq = blockIdx.z;
  const int B = gridDim.z;
  const int row0 = chunk * ARB, nrows = min(ARB, R - row0);
  const int KVH = kv.n_kv_heads, g = head * KVH / n_heads;
  const int len = kv.len[seq];
  const int nspec = max(0, min(rd.nspec[seq], 64));
  const int ktot = min(len + nspec, kv_capacity(kv));

  // splits actually used for this sequence: short contexts stay in one workgroup (all workgroups agree on this)
  const int eff = max(1, min(n_splits, (ktot + KEYS_PER_SPLIT - 1) / KEYS_PER_SPLIT));
  if (split >= eff) return;
  int per = (ktot + eff - 1) / eff;
  per = ((per + ATK - 1) / ATK) * ATK;
  const int kbeg = split * per, kend = min(ktot, kbeg + per);
  const int n_tiles = kend > kbeg ? (kend - kbeg + ATK - 1) / ATK : 0;

  // score-phase role: query row and key group; output-phase role: dim chunk and key subgroup
  const int srow = lane & 15, sg4 = lane >> 4;
  const int dc = lane % CH, kq = lane / CH;
  const bool row_ok = srow < nrows;
  const unsigned long long rmask = row_ok ? rd.mask[seq * R + row0 + srow] : 0ull;

  // Q^T operand: row srow, dims ks*32 + sg4*8 .. +8, as hi + lo halves
  half8 qh[KS], ql[KS];
  {
    const float* qp = q + (int64_t)(seq * R + row0 + srow) * q_stride + (int64_t)head * HD + sg4 * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b2 = a;
      if (row_ok) {
        a = *(const float4*)(qp + ks * 32);
        b2 = *(const float4*)(qp + ks * 32 + 4);
      }
      const float v[8] = {a.x, a.y, a.z, a.w, b2.x, b2.y, b2.z, b2.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const _Float16 hi = (_Float16)v[e];
        qh[ks][e] = hi;
        ql[ks][e] = (_Float16)(v[e] - (float)hi);
      }
    }
  }

  const int64_t tok_stride = (int64_t)KVH * HD;  // elements per cached token
  const kv16_t* kbase = (const kv16_t*)kv.k + (int64_t)layer * kv.layer_stride + (int64_t)g * HD;
  const kv16_t* vbase = (const kv16_t*)kv.v + (int64_t)layer * kv.layer_stride + (int64_t)g * HD;

  float m_run = -INFINITY, l_run = 0.f;  // of row srow (replicated over the four key groups)
  float acc[ARB][8];
#pragma unroll
  for (int r = 0; r < ARB; ++r)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[r][e] = 0.f;

  // token index of key (tile start + lane % 32), looked up once per tile and handed round by shuffles
  auto lookup = [&](int ti) -> int {
    const int kj = kbeg + ti * ATK + (lane & 31);
    return (ti < n_tiles && kj < kend) ? token_index(kv, seq, kj) : -1;
  };
  auto load_k = [&](KFrag (&kf)[2][KS], int tok32) {
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int tk = __shfl(tok32, blk * 16 + srow, 64);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        kf[blk][ks].u = make_uint4(0, 0, 0, 0);
        if (tk >= 0) kf[blk][ks].u = *(const uint4*)(kbase + (int64_t)tk * tok_stride + ks * 32 + sg4 * 8);
      }
    }
  };

  KFrag kf[2][KS], kn[2][KS];
  int tok_cur = lookup(wave), tok_next = -1;
  if (wave < n_tiles) load_k(kf, tok_cur);

  for (int ti = wave; ti < n_tiles; ti += AW) {
    // V of this tile, then K of the next: both in flight while the scores are computed
    KFrag vf[KPS];
#pragma unroll
    for (int j = 0; j < KPS; ++j) {
      const int tk = __shfl(tok_cur, kq * KPS + j, 64);
      vf[j].u = make_uint4(0, 0, 0, 0);
      if (tk >= 0) vf[j].u = *(const uint4*)(vbase + (int64_t)tk * tok_stride + dc * 8);
    }
    const bool more = ti + AW < n_tiles;
    if (more) {
      tok_next = lookup(ti + AW);
      load_k(kn, tok_next);
    }

    // S^T = K Q^T: lane (sg4, srow) gets keys blk*16 + sg4*4 + i of row srow
    floatx4 s2[2];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      s2[blk] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s2[blk] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[blk][ks].h, qh[ks], s2[blk], 0, 0, 0);
        s2[blk] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[blk][ks].h, ql[ks], s2[blk], 0, 0, 0);
      }
    }
    // visibility, scale, running softmax of row srow
    float tmax = -INFINITY;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int kj = kbeg + ti * ATK + blk * 16 + sg4 * 4 + i;
        bool vis = kj < kend;
        if (vis && kj >= len) vis = (rmask >> (kj - len)) & 1ull;
        const float sv = vis ? s2[blk][i] * scale : -INFINITY;
        s2[blk][i] = sv;
        tmax = fmaxf(tmax, sv);
      }
    tmax = xmax(xmax(tmax, 16), 32);
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
    float psum = 0.f;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float pv = (s2[blk][i] == -INFINITY) ? 0.f : expf(s2[blk][i] - m_new);
        s2[blk][i] = pv;
        psum += pv;
      }
    psum = xsum(xsum(psum, 16), 32);
    l_run = l_run * alpha + psum;
    m_run = m_new;
    if (srow < ARB) {
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int i = 0; i < 4; ++i) sm.p[wave][blk * 16 + sg4 * 4 + i][srow] = s2[blk][i];
      if (sg4 == 0) sm.alpha[wave][srow] = alpha;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // O = alpha O + P V for this lane's 8 dims and KPS keys
    {
      float al[ARB];
#pragma unroll
      for (int r = 0; r < ARB; ++r) al[r] = sm.alpha[wave][r];
#pragma unroll
      for (int r = 0; r < ARB; ++r)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] *= al[r];
#pragma unroll
      for (int j = 0; j < KPS; ++j) {
        float pr[ARB];
        const float4 p0 = *(const float4*)&sm.p[wave][kq * KPS + j][0];
        const float4 p1 = *(const float4*)&sm.p[wave][kq * KPS + j][4];
        pr[0] = p0.x; pr[1] = p0.y; pr[2] = p0.z; pr[3] = p0.w; pr[4] = p1.x; pr[5] = p1.y; pr[6] = p1.z; pr[7] = p1.w;
        float vv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) vv[e] = (float)vf[j].h[e];
#pragma unroll
        for (int r = 0; r < ARB; ++r)
          if (r < nrows) {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r][e] = fmaf(pr[r], vv[e], acc[r][e]);
          }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // the tile's probabilities have been read before the next tile overwrites them
    if (more) {
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kf[blk][ks] = kn[blk][ks];
      tok_cur = tok_next;
    }
  }

  // the key subgroups of a wave add up (fixed order), then the waves meet in LDS
#pragma unroll
  for (int r = 0; r < ARB; ++r)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = acc[r][e];
      for (int off = CH; off < 64; off <<= 1) v += __shfl_xor(v, off, 64);
      acc[r][e] = v;
    }
  if (kq == 0) {
#pragma unroll
    for (int r = 0; r < ARB; ++r) {
      *(float4*)&sm.o[wave][r][dc * 8] = make_float4(acc[r][0], acc[r][1], acc[r][2], acc[r][3]);
      *(float4*)&sm.o[wave][r][dc * 8 + 4] = make_float4(acc[r][4], acc[r][5], acc[r][6], acc[r][7]);
    }
  }
  if (sg4 == 0 && srow < ARB) {
    sm.m[wave][srow] = m_run;
    sm.l[wave][srow] = l_run;
  }
  __syncthreads();

  // merge of the 8 waves in wave order: thread = (row, dim); HD = 128 takes two dims per thread
  const int mr = t >> 6;  // 0 .. 7 = row
  float M = -INFINITY;
#pragma unroll
  for (int w2 = 0; w2 < AW; ++w2) M = fmaxf(M, sm.m[w2][mr]);
  float L = 0.f, o[HD / 64];
#pragma unroll
  for (int x = 0; x < HD / 64; ++x) o[x] = 0.f;
#pragma unroll
  for (int w2 = 0; w2 < AW; ++w2) {
    const float mw = sm.m[w2][mr];
    const float e = (mw == -INFINITY) ? 0.f : expf(mw - M);
    L += sm.l[w2][mr] * e;
#pragma unroll
    for (int x = 0; x < HD / 64; ++x) o[x] += sm.o[w2][mr][lane + 64 * x] * e;
  }
  const int64_t lo_plane = (int64_t)B * R * n_heads * HD;
  if (eff == 1) {  // nothing to exchange: this workgroup saw every key
    if (mr < nrows) {
#pragma unroll
      for (int x = 0; x < HD / 64; ++x) {
        const float y = (L > 0.f) ? o[x] / L : 0.f;
        const int64_t idx = (int64_t)(seq * R + row0 + mr) * n_heads * HD + (int64_t)head * HD + lane + 64 * x;
        bf16_t hi, lo;
        split_bf16(y, hi, lo);
        out[idx] = hi;
        out[lo_plane + idx] = lo;
      }
    }
    return;
  }

  // partial[seq][head][row][split][HD+2] = (m, l, acc[HD]); device-scope write-through stores, cache-bypassing loads
  if (mr < nrows) {
    float* p = partial + ((((int64_t)seq * n_heads + head) * R + row0 + mr) * n_splits + split) * (HD + 2);
#pragma unroll
    for (int x = 0; x < HD / 64; ++x) __hip_atomic_store(p + 2 + lane + 64 * x, o[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (lane == 0) {
      __hip_atomic_store(p, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(p + 1, L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  __builtin_amdgcn_s_waitcnt(0);  // the stores have been acknowledged
  __syncthreads();
  if (t == 0) {
    int* c = counters + ((int64_t)seq * n_heads + head) * n_chunks + chunk;
    const int prev = __hip_atomic_fetch_add(c, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sm.last = (prev == eff - 1);
    if (sm.last) __hip_atomic_store(c, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // clean for the next launch
  }
  __syncthreads();
  if (!sm.last || mr >= nrows) return;
  {
    const float* p = partial + (((int64_t)seq * n_heads + head) * R + row0 + mr) * n_splits * (HD + 2);
    float M2 = -INFINITY, L2 = 0.f, o2[HD / 64];
#pragma unroll
    for (int x = 0; x < HD / 64; ++x) o2[x] = 0.f;
    for (int s2 = 0; s2 < eff; ++s2) {  // split order (deterministic)
      const float* ps = p + (int64_t)s2 * (HD + 2);
      const float mm = __hip_atomic_load(ps, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const float ll = __hip_atomic_load(ps + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      float oo[HD / 64];
#pragma unroll
      for (int x = 0; x < HD / 64; ++x) oo[x] = __hip_atomic_load(ps + 2 + lane + 64 * x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (mm == -INFINITY) continue;
      const float Mn = fmaxf(M2, mm);
      const float ws = (M2 == -INFINITY) ? 0.f : expf(M2 - Mn), wj = expf(mm - Mn);
      L2 = L2 * ws + ll * wj;
#pragma unroll
      for (int x = 0; x < HD / 64; ++x) o2[x] = o2[x] * ws + oo[x] * wj;
      M2 = Mn;
    }
#pragma unroll
    for (int x = 0; x < HD / 64; ++x) {
      const float y = (L2 > 0.f) ? o2[x] / L2 : 0.f;
      const int64_t idx = (int64_t)(seq * R + row0 + mr) * n_heads * HD + (int64_t)head * HD + lane + 64 * x;
      bf16_t hi, lo;
      split_bf16(y, hi, lo);
      out[idx] = hi;
      out[lo_plane + idx] = lo;
    }
  }
}

}  // namespace

// bf16 models: q float32 [B*R][q_stride], half-precision cache, output = bf16 hi / lo planes [2][B*R][n_heads*hd].
hipError_t launch_attention_mfma(const float* q, int q_stride, const RowDesc& rd, KvView kv, int layer, int B, int R, int n_heads,
                                 float* partial, int n_splits, int* counters, void* out, hipStream_t s) {
  const int n_chunks = (R + ARB - 1) / ARB;
  const float scale = 1.0f / sqrtf((float)kv.head_dim);
  const dim3 grid(n_splits, n_heads * n_chunks, B), block(AW * 64);
  if (kv.head_dim == 128)
    hipLaunchKernelGGL((tree_attn_mfma_kernel<128>), grid, block, 0, s, q, q_stride, rd, kv, layer, R, n_heads, n_chunks, scale, partial,
                       n_splits, counters, (bf16_t*)out);
  else if (kv.head_dim == 64)
    hipLaunchKernelGGL((tree_attn_mfma_kernel<64>), grid, block, 0, s, q, q_stride, rd, kv, layer, R, n_heads, n_chunks, scale, partial,
                       n_splits, counters, (bf16_t*)out);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace mtad
