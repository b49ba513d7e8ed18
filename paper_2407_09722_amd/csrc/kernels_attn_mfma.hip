// Tree-masked paged attention for bf16 models (half-precision K/V cache), few query rows per sequence
// (Section 3.3: tree attention gives every tree token its conditional likelihood in one pass).
//
// Work item = (key split, KV head, chunk of 16 or 32 (query head, row) pairs, sequence) = one workgroup of AW waves (4 in
// all configurations used; 8 measured no faster).  The query heads that share a KV head are rows of the same item, so a
// grouped-query model reads K and V once for all of them.  The keys of the item are cut into 32-key tiles dealt
// round-robin to the waves; every wave runs its own online softmax over its tiles, with the K and V of the next tile
// (the next two, where the registers allow a second set) in flight, and the waves merge through LDS at the end.  A context of fewer than 2 x waves x 32 keys is one workgroup,
// which writes the attention output itself: no exchange through global memory.  Longer contexts are cut into splits
// (at least one tile per wave each, at most as many as fill the machine once, or every resident slot where once is an
// uneven fill); every split leaves (max, sum, output)
// per row in global memory (same partial layout as the generic kernel) and a small second kernel, one wave per row,
// merges them in split order.
//
// Both products run on the matrix cores, transposed, so that every operand is cheap to fetch:
//   S^T = K Q^T   A operand = 8 consecutive dims of one key per lane = 16 contiguous bytes of a cache row, loaded from
//                 global memory straight into the operand registers; B operand = Q as two half terms (hi + lo, two
//                 MFMAs: float32 accuracy) from LDS.  Lane (g, r) ends up with the scores of row r for 8 keys of
//                 the tile: the per-row softmax needs two cross-lane steps and stays in that lane.
//   O^T = V^T P^T the probabilities a lane holds are exactly its B operand (the k index of the contraction is
//                 assigned to keys in the order the score product left them), again as hi + lo halves; V^T fragments
//                 are read transposed from a wave-private LDS copy of the V tile (padded rows: conflict free).
// The running output, maximum and sum of a row all live in the lanes of that row: no exchange inside the tile loop.
#include "common.h"

#include <type_traits>

namespace mtad {

namespace {


constexpr int ATK = 32;              // keys per tile

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

union KFrag {
  uint4 u;
  half8 h;
};

template <int HD, int NRG, int AW>
struct MfmaAttnSmem {
  static constexpr int VS = HD + 8;  // padded row of halves: 16-byte aligned, keys 4 apart land 16 banks apart
  union {
    struct {
      _Float16 v[AW][ATK][VS];         // V tile of each wave
      _Float16 q[2][NRG * 16][VS];     // query rows, hi and lo halves
    } a;
    // per-wave outputs for the final merge, MRG row groups at a time (padded rows: the 16 rows of a store land in different banks)
    float o[AW][(NRG <= 2 ? NRG : 1) * 16][HD + 4];
  };
  float m[AW][NRG * 16], l[AW][NRG * 16];
};

// Exchange with lane ^ 16 or lane ^ 32 through the row / half swap instructions of gfx950 (vector ALU, no LDS round trip:
// the softmax of a tile waits for four such exchanges per row group).  Swapping a register with its own copy leaves the
// even rows (lower half) in one result and the odd rows (upper half) in the other, each duplicated: every lane then
// holds its own value and its partner's.
template <int OFF>
__device__ __forceinline__ void lane_pair(float v, float& a, float& b) {
  static_assert(OFF == 16 || OFF == 32, "row or half swap");
  const unsigned u = __float_as_uint(v);
  if constexpr (OFF == 16) {
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
  } else {
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
  }
}
template <int OFF>
__device__ __forceinline__ float xmax(float v) {
  float a, b;
  lane_pair<OFF>(v, a, b);
  return fmaxf(a, b);
}
template <int OFF>
__device__ __forceinline__ float xsum(float v) {
  float a, b;
  lane_pair<OFF>(v, a, b);
  return a + b;
}

// physical token index (page * page_size + offset) of logical position pos; pages outside the pool read page 0
__device__ __forceinline__ int token_index(const KvView& kv, int seq, int pos) {
  int page = kv.page_table[(int64_t)seq * kv.max_pages + pos / kv.page_size];
  page = (page < 0 || page >= kv.n_pages) ? 0 : page;
  return page * kv.page_size + pos % kv.page_size;
}

// Keys of sequence seq (committed + speculative) and the key splits used for it.  Every workgroup of the attention
// kernel and of the merge kernel derives the same numbers: as many splits as the launch offers, but a split is worth its
// exchange only if it gives every wave a tile (measured at 512 and 2048 keys).  want_splits = fill_splits +
// (more_splits << 8): fill_splits give every compute unit a workgroup; more_splits, offered when that leaves some
// compute units with two workgroups and the rest with one, fill every resident slot and are taken only where every
// wave still gets four tiles.
constexpr int ATTN_WAVES = 4;
__device__ __forceinline__ int attn_keys(const KvView& kv, const RowDesc& rd, int seq) {
  const int nspec = max(0, min(rd.nspec[seq], 64));
  return min(kv.len[seq] + nspec, kv_capacity(kv));
}
__device__ __forceinline__ int attn_splits(int ktot, int n_splits, int want_splits) {
  // from two splits on, one more for a remainder: it keeps every wave at one tile (C3, 516 keys: 5 splits of 4 tiles
  // instead of 4 splits of 5, whose first wave runs a second tile after the first)
  constexpr int WK = ATTN_WAVES * ATK;
  const int fill = min(want_splits & 255, ktot < 2 * WK ? 1 : (ktot + WK - 1) / WK);
  const int more = min(want_splits >> 8, ktot / (4 * ATTN_WAVES * ATK));
  return max(1, min(n_splits, max(fill, more)));
}

template <int HD, int NRG, int AW>
__global__ __launch_bounds__(AW * 64) __attribute__((amdgpu_waves_per_eu(2))) void tree_attn_mfma_kernel(const float* __restrict__ q, int q_stride, RowDesc rd, KvView kv, int layer,
                                                               int R, int n_heads, int n_chunks, float scale, float* __restrict__ partial,
                                                               int n_splits, bf16_t* __restrict__ out, int want_splits, int ncg) {
  constexpr int KS = HD / 32;    // k-steps of the score product
  constexpr int DB = HD / 16;    // 16-dim blocks of the output
  constexpr int CH = HD / 8;     // 16-byte chunks of a cache row
  constexpr int KPL = 64 / CH;   // keys one V load instruction covers
  constexpr int NV = ATK / KPL;  // V load instructions per tile
  constexpr int RBK = NRG * 16;  // query rows per work item
  constexpr int TPR = AW * 4;    // threads per query row in the merge (16 rows per pass)
  constexpr int DPT = HD / TPR;  // output dims per thread in the merge
  using Smem = MfmaAttnSmem<HD, NRG, AW>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];  // dynamic: an 8-wave variant needs more than 64 KiB
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  // work item: key split, (KV head g, chunk of RBK (query head, row) pairs), sequence.  Pair p = hq * R + row of the G
  // query heads that share KV head g: grouped-query models read K and V once for all of them
  const int split = blockIdx.x, g = blockIdx.y / n_chunks, chunk = blockIdx.y % n_chunks, seq = blockIdx.z;
  const int B = gridDim.z;
  const int KVH = kv.n_kv_heads, G = n_heads / KVH;
  const int pair0 = chunk * RBK, nrows = min(RBK, G * R - pair0);
  auto pair_head = [&](int r) { return g * G + (pair0 + r) / R; };  // query head and tree row of pair r of this item
  auto pair_row = [&](int r) { return (pair0 + r) % R; };
  static_assert(AW == ATTN_WAVES, "attn_splits() assumes this many waves");
  const int len = kv.len[seq];
  const int ktot = attn_keys(kv, rd, seq);
  const int eff = attn_splits(ktot, n_splits, want_splits);  // splits actually used for this sequence
  if (split >= eff) return;
  int per = (ktot + eff - 1) / eff;
  per = ((per + ATK - 1) / ATK) * ATK;
  const int kbeg = split * per, kend = min(ktot, kbeg + per);
  const int n_tiles = kend > kbeg ? (kend - kbeg + ATK - 1) / ATK : 0;

  const int srow = lane & 15, sg4 = lane >> 4;  // this lane's query row (within a row group) and key group
  unsigned long long rmask[NRG];
#pragma unroll
  for (int rg = 0; rg < NRG; ++rg) rmask[rg] = (rg * 16 + srow < nrows) ? rd.mask[seq * R + pair_row(rg * 16 + srow)] : 0ull;

  // token index of key (tile start + lane % 32), looked up once per tile and handed round by shuffles
  auto lookup = [&](int ti) -> int {
    const int kj = kbeg + ti * ATK + (lane & 31);
    return (ti < n_tiles && kj < kend) ? token_index(kv, seq, kj) : -1;
  };
  const int64_t tok_stride = (int64_t)KVH * HD;  // elements per cached token
  const kv16_t* kbase = (const kv16_t*)kv.k + (int64_t)layer * kv.layer_stride + (int64_t)g * HD;
  const kv16_t* vbase = (const kv16_t*)kv.v + (int64_t)layer * kv.layer_stride + (int64_t)g * HD;

  // One register set for K and one for V: a tile's V registers are free once the tile is in LDS and its K registers once the
  // score product has been issued, and the next tile's requests go out at those points (V, needed first, first).  The
  // loads are unconditional (keys past the end read token 0 of page 0): their scores are masked, and their V rows are
  // zeroed so that they contribute exact zeros.  The first tile is requested before the queries are staged.
  // Where the registers allow it (DEEP) there are two such sets and a wave has two tiles in flight: with one set the
  // requests of a tile go out only when the tile before has arrived, so every tile of a wave pays a full memory latency.
  constexpr bool DEEP = HD == 64 || NRG == 1;
  constexpr int NSET = DEEP ? 2 : 1, AHEAD = NSET * AW;
  constexpr std::integral_constant<int, 0> SET0{};
  constexpr std::integral_constant<int, NSET - 1> SET1{};
  KFrag kf[NSET][2][KS], vf[NSET][NV];
  auto load_k = [&](auto set, int tok32) {
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int tk = max(0, __shfl(tok32, blk * 16 + srow, 64));
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kf[set()][blk][ks].u = *(const uint4*)(kbase + (int64_t)tk * tok_stride + ks * 32 + sg4 * 8);
    }
  };
  auto load_v = [&](auto set, int tok32) {
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int tk = __shfl(tok32, j * KPL + lane / CH, 64);
      const uint4 v = *(const uint4*)(vbase + (int64_t)max(0, tk) * tok_stride + (lane % CH) * 8);
      vf[set()][j].u = tk >= 0 ? v : make_uint4(0, 0, 0, 0);
    }
  };
  if (wave < n_tiles) {
    const int tok = lookup(wave);
    load_v(SET0, tok);
    load_k(SET0, tok);
  }
  if (DEEP && wave + AW < n_tiles) {
    const int tok = lookup(wave + AW);
    load_v(SET1, tok);
    load_k(SET1, tok);
  }

  // queries of the item as half hi / lo terms in LDS (rows beyond the item are zero)
  for (int i = t; i < RBK * (HD / 4); i += AW * 64) {
    const int r = i / (HD / 4), d = (i % (HD / 4)) * 4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (r < nrows) v = *(const float4*)(q + (int64_t)(seq * R + pair_row(r)) * q_stride + (int64_t)pair_head(r) * HD + d);
    const float x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const _Float16 hi = (_Float16)x[e];
      sm.a.q[0][r][d + e] = hi;
      sm.a.q[1][r][d + e] = (_Float16)(x[e] - (float)hi);
    }
  }
  __syncthreads();
  float m_run[NRG], l_run[NRG];  // of row rg*16 + srow (replicated over the four key groups)
  floatx4 acc[NRG][DB];          // O^T: dims db*16 + sg4*4 + i of row rg*16 + srow
#pragma unroll
  for (int rg = 0; rg < NRG; ++rg) {
    m_run[rg] = -INFINITY;
    l_run[rg] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[rg][db] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  auto process = [&](auto set, int ti) {                    // tile ti, whose K and V are in (or on the way to) register set `set`
    const bool more = ti + AHEAD < n_tiles;                 // uniform over the wave
    const int tok_next = more ? lookup(ti + AHEAD) : -1;    // the page-table read of the set's next tile starts here
    // V tile -> wave-private LDS copy
#pragma unroll
    for (int j = 0; j < NV; ++j) *(uint4*)&sm.a.v[wave][j * KPL + lane / CH][(lane % CH) * 8] = vf[set()][j].u;
    if (more) load_v(set, tok_next);

    // S^T = K Q^T: lane (sg4, srow) gets keys blk*16 + sg4*4 + i of row rg*16 + srow
    floatx4 s2[NRG][2];
#pragma unroll
    for (int rg = 0; rg < NRG; ++rg)
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) s2[rg][blk] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int rg = 0; rg < NRG; ++rg) {
        const half8 qh = *(const half8*)&sm.a.q[0][rg * 16 + srow][ks * 32 + sg4 * 8];
        const half8 ql = *(const half8*)&sm.a.q[1][rg * 16 + srow][ks * 32 + sg4 * 8];
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
          s2[rg][blk] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[set()][blk][ks].h, qh, s2[rg][blk], 0, 0, 0);
          s2[rg][blk] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[set()][blk][ks].h, ql, s2[rg][blk], 0, 0, 0);
        }
      }
    if (more) load_k(set, tok_next);  // the score product has read its K operands
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // the V tile is in LDS (the wave reads what other lanes wrote)
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // visibility, scale, running softmax per row; probabilities become the B operand of the second product
    half8 ph[NRG], pl[NRG];
    // a tile that lies inside the committed context (all but the last one or two) is visible to every row: no mask
    const bool plain = kbeg + (ti + 1) * ATK <= min(len, kend);  // uniform over the wave
#pragma unroll
    for (int rg = 0; rg < NRG; ++rg) {
      float tmax = -INFINITY;
      if (plain) {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float sv = s2[rg][blk][i] * scale;
            s2[rg][blk][i] = sv;
            tmax = fmaxf(tmax, sv);
          }
      } else {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int kj = kbeg + ti * ATK + blk * 16 + sg4 * 4 + i;
            bool vis = kj < kend;
            if (vis && kj >= len) vis = (rmask[rg] >> (kj - len)) & 1ull;
            const float sv = vis ? s2[rg][blk][i] * scale : -INFINITY;
            s2[rg][blk][i] = sv;
            tmax = fmaxf(tmax, sv);
          }
      }
      tmax = xmax<32>(xmax<16>(tmax));
      const float m_new = fmaxf(m_run[rg], tmax);
      const float alpha = (m_run[rg] == -INFINITY) ? 0.f : __expf(m_run[rg] - m_new);
      float psum = 0.f;
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float pv = (s2[rg][blk][i] == -INFINITY) ? 0.f : __expf(s2[rg][blk][i] - m_new);
          psum += pv;
          const _Float16 hi = (_Float16)pv;
          ph[rg][blk * 4 + i] = hi;
          pl[rg][blk * 4 + i] = (_Float16)(pv - (float)hi);
        }
      psum = xsum<32>(xsum<16>(psum));
      l_run[rg] = l_run[rg] * alpha + psum;
      m_run[rg] = m_new;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[rg][db][i] *= alpha;
    }

    // O^T += V^T P^T: contraction slot e of key group sg4 is key (e/4)*16 + sg4*4 + e%4, as the scores came out
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      half8 vt;
#pragma unroll
      for (int e = 0; e < 8; ++e) vt[e] = sm.a.v[wave][(e >> 2) * 16 + sg4 * 4 + (e & 3)][db * 16 + srow];
#pragma unroll
      for (int rg = 0; rg < NRG; ++rg) {
        acc[rg][db] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vt, ph[rg], acc[rg][db], 0, 0, 0);
        acc[rg][db] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vt, pl[rg], acc[rg][db], 0, 0, 0);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // the V tile has been read before the next one overwrites it
  };
#pragma unroll 1
  for (int ti = wave; ti < n_tiles; ti += AHEAD) {
    process(SET0, ti);
    if (DEEP && ti + AW < n_tiles) process(SET1, ti + AW);
  }
  // ---- the waves meet in LDS (the buffer aliases the V tiles and the queries)
  const int mrow = t / TPR, md = (t % TPR) * DPT;  // merge role: row within a row group, first of DPT dims
  typedef bf16_t bf16xd __attribute__((ext_vector_type(DPT)));
  auto store_out = [&](int r, const float (&o)[DPT], float L) {  // normalised row -> hi / lo planes, one vector store each
    const int arow = seq * R + pair_row(r), ak = pair_head(r) * HD + md;  // row of the pass, feature of the o product's input
    bf16xd hi, lo;
#pragma unroll
    for (int x = 0; x < DPT; ++x) {
      bf16_t h, l;
      split_bf16((L > 0.f) ? o[x] / L : 0.f, h, l);
      hi[x] = h;
      lo[x] = l;
    }
    *(bf16xd*)(out + act_offset(ncg, B * R, n_heads * HD, 0, arow, ak)) = hi;
    *(bf16xd*)(out + act_offset(ncg, B * R, n_heads * HD, 1, arow, ak)) = lo;
  };
#pragma unroll
  for (int rg = 0; rg < NRG; ++rg) {
    if (sg4 == 0) {
      sm.m[wave][rg * 16 + srow] = m_run[rg];
      sm.l[wave][rg * 16 + srow] = l_run[rg];
    }
  }
  constexpr int MRG = NRG <= 2 ? NRG : 1;  // row groups the merge buffer holds at a time
#pragma unroll
  for (int rg0 = 0; rg0 < NRG; rg0 += MRG) {
    __syncthreads();  // everyone is done with the tiles (first pass) / with the previous row groups' buffer
#pragma unroll
    for (int rm = 0; rm < MRG; ++rm)
#pragma unroll
      for (int db = 0; db < DB; ++db)
        *(float4*)&sm.o[wave][rm * 16 + srow][db * 16 + sg4 * 4] =
            make_float4(acc[rg0 + rm][db][0], acc[rg0 + rm][db][1], acc[rg0 + rm][db][2], acc[rg0 + rm][db][3]);
    __syncthreads();
#pragma unroll
    for (int rm = 0; rm < MRG; ++rm) {
      const int r = (rg0 + rm) * 16 + mrow;
      float M = -INFINITY;
#pragma unroll
      for (int w2 = 0; w2 < AW; ++w2) M = fmaxf(M, sm.m[w2][r]);
      float L = 0.f, o[DPT];
#pragma unroll
      for (int x = 0; x < DPT; ++x) o[x] = 0.f;
#pragma unroll
      for (int w2 = 0; w2 < AW; ++w2) {  // wave order (deterministic)
        const float mw = sm.m[w2][r];
        const float e = (mw == -INFINITY) ? 0.f : expf(mw - M);
        L += sm.l[w2][r] * e;
#pragma unroll
        for (int x4 = 0; x4 < DPT; x4 += 4) {
          const float4 v = *(const float4*)&sm.o[w2][rm * 16 + mrow][md + x4];
          o[x4] += v.x * e; o[x4 + 1] += v.y * e; o[x4 + 2] += v.z * e; o[x4 + 3] += v.w * e;
        }
      }
      if (r < nrows) {
        if (eff == 1) {  // nothing to exchange: this workgroup saw every key
          store_out(r, o, L);
        } else {  // partial[seq][head][row][split][HD+2] = (m, l, acc[HD]) for the merge kernel
          float* p = partial + ((((int64_t)seq * n_heads + pair_head(r)) * R + pair_row(r)) * n_splits + split) * (HD + 2);
#pragma unroll
          for (int x = 0; x < DPT; x += 2) st8<false>(p + 2 + md + x, make_uint2(__float_as_uint(o[x]), __float_as_uint(o[x + 1])));
          if (t % TPR == 0) st8<false>(p, make_uint2(__float_as_uint(M), __float_as_uint(L)));
        }
      }
    }
  }
}

// Merge of the key splits, a kernel of its own: one wave per (sequence, query head, row) adds the eff partial results in
// split order (deterministic) with all their loads in flight together, and writes the normalised row as bf16 hi / lo
// terms.  As a separate launch it is spread over the whole machine and costs about the same for any number of
// splits, where the last workgroup of an item merging inside the attention kernel (the first design: 3.3 us of 13.1 at
// 4 splits and 5 rows, 8 us of 28 at 8 splits and 17 rows) made more splits cost more than they gained.
template <int HD>
__global__ __launch_bounds__(256) void attn_merge_kernel(RowDesc rd, KvView kv, int B, int R, int n_heads, const float* __restrict__ partial,
                                                         int n_splits, int want_splits, bf16_t* __restrict__ out, int ncg) {
  constexpr int DPL = HD / 64;  // output dims per lane
  const int lane = threadIdx.x & 63;
  const int item = blockIdx.x * 4 + (threadIdx.x >> 6);  // (seq, head, row)
  if (item >= B * n_heads * R) return;
  const int row = item % R, head = (item / R) % n_heads, seq = item / (R * n_heads);
  const int eff = attn_splits(attn_keys(kv, rd, seq), n_splits, want_splits);
  if (eff == 1) return;  // the attention kernel wrote the output itself
  const float* pp = partial + (((int64_t)seq * n_heads + head) * R + row) * n_splits * (HD + 2);
  float M = -INFINITY, L = 0.f, o[DPL];
#pragma unroll
  for (int x = 0; x < DPL; ++x) o[x] = 0.f;
  constexpr int SB = 8;  // splits per batch
  for (int s0 = 0; s0 < eff; s0 += SB) {
    float2 ml[SB];
    float ov[SB][DPL];
#pragma unroll
    for (int j = 0; j < SB; ++j) {
      const float* ps = pp + (int64_t)min(s0 + j, eff - 1) * (HD + 2);
      ml[j] = *(const float2*)ps;
      if constexpr (DPL == 2) {
        const float2 v = *(const float2*)(ps + 2 + lane * 2);
        ov[j][0] = v.x;
        ov[j][1] = v.y;
      } else {
        ov[j][0] = ps[2 + lane];
      }
    }
#pragma unroll
    for (int j = 0; j < SB; ++j) {
      const float mj = ml[j].x, lj = ml[j].y;
      if (s0 + j >= eff || mj == -INFINITY) continue;
      const float Mn = fmaxf(M, mj);
      const float ws = (M == -INFINITY) ? 0.f : expf(M - Mn), wj = expf(mj - Mn);
      L = L * ws + lj * wj;
#pragma unroll
      for (int x = 0; x < DPL; ++x) o[x] = o[x] * ws + ov[j][x] * wj;
      M = Mn;
    }
  }
  typedef bf16_t bf16xd __attribute__((ext_vector_type(DPL)));
  bf16xd hi, lo;
#pragma unroll
  for (int x = 0; x < DPL; ++x) {
    bf16_t h, l;
    split_bf16((L > 0.f) ? o[x] / L : 0.f, h, l);
    hi[x] = h;
    lo[x] = l;
  }
  const int arow = seq * R + row, ak = head * HD + lane * DPL;
  *(bf16xd*)(out + act_offset(ncg, B * R, n_heads * HD, 0, arow, ak)) = hi;
  *(bf16xd*)(out + act_offset(ncg, B * R, n_heads * HD, 1, arow, ak)) = lo;
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
