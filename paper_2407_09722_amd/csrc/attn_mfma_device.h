// Device side of the tree-masked paged attention of bf16 models (half-precision K/V cache), shared by the stand-alone
// kernels (kernels_attn_mfma.hip) and the one-launch pass (kernels_flow.hip).  Section 3.3: tree attention gives every
// tree token its conditional likelihood in one pass.
//
// Work item = (key split, KV head, chunk of 16 or 32 (query head, row) pairs, sequence), run by AW waves of a workgroup
// of NTH threads (waves beyond AW only take part in the barriers).  The query heads that share a KV head are rows of the
// same item, so a grouped-query model reads K and V once for all of them.  The keys of the item are cut into 32-key tiles
// dealt round-robin to the waves; every wave runs its own online softmax over its tiles, with the K and V of the next
// tile (the next two with NSET = 2) in flight, and the waves merge through LDS at the end.
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
#pragma once
#include "common.h"

#include <type_traits>

namespace mtad {

constexpr int ATK = 32;  // keys per tile

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float attn_floatx4 __attribute__((ext_vector_type(4)));

union KFrag {
  uint4 u;
  half8 h;
};

template <int HD, int NRG, int AW, int DS = 1>
struct MfmaAttnSmem {
  static constexpr int VS = HD + 8;       // padded row of halves: 16-byte aligned, keys 4 apart land 16 banks apart
  static constexpr int VSV = HD / DS + 8;  // the same for the part of a V row one wave holds
  union {
    struct {
      _Float16 v[AW * DS][ATK][VSV];  // V tile of each wave (its share of the dims)
      _Float16 q[2][NRG * 16][VS];    // query rows, hi and lo halves
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

// Keys of sequence seq (committed + speculative) and the key splits used for it.  Every workgroup that works on the
// sequence derives the same numbers: as many splits as the launch offers, but a split is worth its
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
  // from two splits on, one more for a remainder: it keeps every wave at one tile (516 keys: 5 splits of 4 tiles
  // instead of 4 splits of 5, whose first wave runs a second tile after the first)
  constexpr int WK = ATTN_WAVES * ATK;
  const int fill = min(want_splits & 255, ktot < 2 * WK ? 1 : (ktot + WK - 1) / WK);
  const int more = min(want_splits >> 8, ktot / (4 * ATTN_WAVES * ATK));
  return max(1, min(n_splits, max(fill, more)));
}

// 2, 4, 8 or 16 bytes to global memory: plain (the consumer is a later kernel) or write-through (COH: the consumer is
// another workgroup of the same kernel)
template <bool COH, int BYTES>
__device__ __forceinline__ void attn_store(void* p, const void* v) {
  if constexpr (!COH) {
    __builtin_memcpy(p, v, BYTES);
  } else if constexpr (BYTES == 2) {
    unsigned short x;
    __builtin_memcpy(&x, v, 2);
    __hip_atomic_store((unsigned short*)p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else if constexpr (BYTES == 4) {
    unsigned x;
    __builtin_memcpy(&x, v, 4);
    __hip_atomic_store((unsigned*)p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else {
    static_assert(BYTES % 8 == 0, "whole 8-byte words");
#pragma unroll
    for (int i = 0; i < BYTES / 8; ++i) {
      unsigned long long x;
      __builtin_memcpy(&x, (const char*)v + 8 * i, 8);
      __hip_atomic_store((unsigned long long*)p + i, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// Merge of the key splits of one (sequence, query head, row) by one wave: the eff partial results are added in split
// order (deterministic) with all their loads in flight together, and the normalised row is written as bf16 hi / lo terms.
// COH: the partials were written by other workgroups of this kernel (cache-bypassing loads, write-through stores).
template <int HD, bool COH>
__device__ __forceinline__ void attn_merge_row(const float* __restrict__ pp, int eff, bf16_t* __restrict__ out, int ncg, int rows_all, int K,
                                               int arow, int head, int lane) {
  constexpr int DPL = HD / 64;  // output dims per lane
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
      if constexpr (COH) {
        const unsigned long long a = __hip_atomic_load((const unsigned long long*)ps, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ml[j] = make_float2(__uint_as_float((unsigned)a), __uint_as_float((unsigned)(a >> 32)));
        if constexpr (DPL == 2) {
          const unsigned long long b = __hip_atomic_load((const unsigned long long*)(ps + 2 + lane * 2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ov[j][0] = __uint_as_float((unsigned)b);
          ov[j][1] = __uint_as_float((unsigned)(b >> 32));
        } else {
          ov[j][0] = __hip_atomic_load(ps + 2 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      } else {
        ml[j] = *(const float2*)ps;
        if constexpr (DPL == 2) {
          const float2 v = *(const float2*)(ps + 2 + lane * 2);
          ov[j][0] = v.x;
          ov[j][1] = v.y;
        } else {
          ov[j][0] = ps[2 + lane];
        }
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
  const int ak = head * HD + lane * DPL;
  attn_store<COH, DPL * 2>(out + act_offset(ncg, rows_all, K, 0, arow, ak), &hi);
  attn_store<COH, DPL * 2>(out + act_offset(ncg, rows_all, K, 1, arow, ak), &lo);
}

// One work item.  All NTH threads of the workgroup call it with the same arguments (and their index t); threads of waves
// beyond the item's only pass the barriers.  NSET register sets for K and V (1 or 2).  Returns the splits in use for the sequence (eff): with eff == 1
// the item wrote the attention output itself, otherwise it left (max, sum, output) per row in
// partial[seq][head][row][split][HD+2] for a merge (attn_merge_row).  COH: outputs are write-through stores.
// DS = 2: every tile is worked on by two waves (w and w + AW), each with half of the output dims: both compute the tile's
// scores and softmax, each loads half of every V row and keeps half of the accumulators.  Two thirds of the tile registers
// per wave, for a kernel that must fit two workgroups of eight waves on a compute unit, and no wave of those eight idles.
// wait_for_rows: called once by all threads (it may hold a workgroup barrier) before anything is read that this pass's own
// rows produce, i.e. the queries and the K / V of speculative positions.  K and V tiles that lie inside the committed
// context are requested BEFORE it: a caller whose queries are still being computed has the cache reads of the context
// in flight meanwhile.  (Items without work return before the call.)
struct AttnNoWait {
  __device__ __forceinline__ void operator()() const {}
};
template <int HD, int NRG, int AW, int NSET, int NTH, bool COH, int DS = 1, typename WaitFn = AttnNoWait>
__device__ __forceinline__ int tree_attn_item(MfmaAttnSmem<HD, NRG, AW, DS>& sm, const float* __restrict__ q, int q_stride, const RowDesc& rd,
                                              const KvView& kv, int layer, int B, int R, int n_heads, int n_chunks, float scale,
                                              float* __restrict__ partial, int n_splits, bf16_t* __restrict__ out, int want_splits, int ncg,
                                              int split, int g, int chunk, int seq, int t, WaitFn wait_for_rows = WaitFn()) {
  constexpr int KS = HD / 32;    // k-steps of the score product
  constexpr int HV = HD / DS;    // output dims (= dims of every V row) this wave works on
  constexpr int DB = HV / 16;    // 16-dim blocks of the output
  constexpr int CH = HV / 8;     // 16-byte chunks of (this wave's part of) a cache row
  constexpr int KPL = 64 / CH;   // keys one V load instruction covers
  constexpr int NV = ATK / KPL;  // V load instructions per tile
  constexpr int RBK = NRG * 16;  // query rows per work item
  constexpr int TPR = AW * 4;    // threads per query row in the merge (16 rows per pass)
  constexpr int DPT = HD / TPR;  // output dims per thread in the merge
  static_assert(AW == ATTN_WAVES, "attn_splits() assumes this many waves");
  static_assert(NTH >= AW * DS * 64 && NSET >= 1 && NSET <= 2, "workgroup holds the waves of an item");
  static_assert(DS == 1 || DS == 2, "one or two waves per tile");

  const int lane = t & 63;  // t: index of the thread in the workgroup
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const bool active = wave < AW * DS;  // uniform over the wave
  const int wslot = active ? wave % AW : 0, dpart = active ? wave / AW : 0;  // tile slot and share of the dims
  // Pair p = hq * R + row of the G query heads that share KV head g: grouped-query models read K and V once for all of them
  const int KVH = kv.n_kv_heads, G = n_heads / KVH;
  const int pair0 = chunk * RBK, nrows = min(RBK, G * R - pair0);
  auto pair_head = [&](int r) { return g * G + (pair0 + r) / R; };  // query head and tree row of pair r of this item
  auto pair_row = [&](int r) { return (pair0 + r) % R; };
  const int len = kv.len[seq];
  const int ktot = attn_keys(kv, rd, seq);
  const int eff = attn_splits(ktot, n_splits, want_splits);  // splits actually used for this sequence
  if (split >= eff) return eff;
  int per = (ktot + eff - 1) / eff;
  per = ((per + ATK - 1) / ATK) * ATK;
  const int kbeg = split * per, kend = min(ktot, kbeg + per);
  const int n_tiles = (active && kend > kbeg) ? (kend - kbeg + ATK - 1) / ATK : 0;  // none for the waves that only pass barriers
  const int wv = active ? wave : 0;  // this wave's V tile in LDS

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
  const kv16_t* vbase = (const kv16_t*)kv.v + (int64_t)layer * kv.layer_stride + (int64_t)g * HD + dpart * HV;

  // One register set for K and one for V: a tile's V registers are free once the tile is in LDS and its K registers once the
  // score product has been issued, and the next tile's requests go out at those points (V, needed first, first).  The
  // loads are unconditional (keys past the end read token 0 of page 0): their scores are masked, and their V rows are
  // zeroed so that they contribute exact zeros.  The first tile is requested before the queries are staged.
  // With two sets a wave has two tiles in flight: with one set the requests of a tile go out only when the tile before
  // has arrived, so every tile of a wave pays a full memory latency.
  constexpr int AHEAD = NSET * AW;
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
  // The same for requests that go out before wait_for_rows: lanes without a committed key request nothing at all (token 0,
  // which the loads above fall back to, may be a slot that the caller's own pass is still writing, and a copy of its old
  // contents in a cache would be read again after the wait).
  auto load_k_committed = [&](auto set, int tok32) {
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int tk = __shfl(tok32, blk * 16 + srow, 64);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        kf[set()][blk][ks].u = make_uint4(0, 0, 0, 0);
        if (tk >= 0) kf[set()][blk][ks].u = *(const uint4*)(kbase + (int64_t)tk * tok_stride + ks * 32 + sg4 * 8);
      }
    }
  };
  auto load_v_committed = [&](auto set, int tok32) {
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int tk = __shfl(tok32, j * KPL + lane / CH, 64);
      vf[set()][j].u = make_uint4(0, 0, 0, 0);
      if (tk >= 0) vf[set()][j].u = *(const uint4*)(vbase + (int64_t)tk * tok_stride + (lane % CH) * 8);
    }
  };
  // The first tile(s) of a wave go out BEFORE wait_for_rows: the page-table lookups of all their keys, and K and V of the
  // keys inside the committed context.  Keys at speculative positions (their K and V are being written by the caller's
  // own pass) are marked -(token + 2) by the early lookup, read as absent for now, and fetched lane by lane after the wait.
  auto lookup_marked = [&](int ti) -> int {
    const int kj = kbeg + ti * ATK + (lane & 31);
    if (!(ti < n_tiles && kj < kend)) return -1;
    const int tk = token_index(kv, seq, kj);
    return kj < len ? tk : -(tk + 2);
  };
  auto patch_k = [&](auto set, int tokm) {
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int tm = __shfl(tokm, blk * 16 + srow, 64);
      if (tm <= -2) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kf[set()][blk][ks].u = *(const uint4*)(kbase + (int64_t)(-tm - 2) * tok_stride + ks * 32 + sg4 * 8);
      }
    }
  };
  auto patch_v = [&](auto set, int tokm) {
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int tm = __shfl(tokm, j * KPL + lane / CH, 64);
      if (tm <= -2) vf[set()][j].u = *(const uint4*)(vbase + (int64_t)(-tm - 2) * tok_stride + (lane % CH) * 8);
    }
  };
  int tokm0 = -1, tokm1 = -1;
  if (wslot < n_tiles) {
    tokm0 = lookup_marked(wslot);
    load_v_committed(SET0, tokm0);
    load_k_committed(SET0, tokm0);
  }
  if (NSET == 2 && wslot + AW < n_tiles) {
    tokm1 = lookup_marked(wslot + AW);
    load_v_committed(SET1, tokm1);
    load_k_committed(SET1, tokm1);
  }
  wait_for_rows();
  if (__any(tokm0 <= -2)) {  // uniform over the wave
    patch_v(SET0, tokm0);
    patch_k(SET0, tokm0);
  }
  if (NSET == 2 && __any(tokm1 <= -2)) {
    patch_v(SET1, tokm1);
    patch_k(SET1, tokm1);
  }

  // queries of the item as half hi / lo terms in LDS (rows beyond the item are zero)
  for (int i = t; i < RBK * (HD / 4); i += NTH) {
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
  attn_floatx4 acc[NRG][DB];     // O^T: dims db*16 + sg4*4 + i of row rg*16 + srow
#pragma unroll
  for (int rg = 0; rg < NRG; ++rg) {
    m_run[rg] = -INFINITY;
    l_run[rg] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[rg][db] = attn_floatx4{0.f, 0.f, 0.f, 0.f};
  }

  auto process = [&](auto set, int ti) {                    // tile ti, whose K and V are in (or on the way to) register set `set`
    const bool more = ti + AHEAD < n_tiles;                 // uniform over the wave
    const int tok_next = more ? lookup(ti + AHEAD) : -1;    // the page-table read of the set's next tile starts here
    // V tile -> wave-private LDS copy
#pragma unroll
    for (int j = 0; j < NV; ++j) *(uint4*)&sm.a.v[wv][j * KPL + lane / CH][(lane % CH) * 8] = vf[set()][j].u;
    if (more) load_v(set, tok_next);

    // S^T = K Q^T: lane (sg4, srow) gets keys blk*16 + sg4*4 + i of row rg*16 + srow
    attn_floatx4 s2[NRG][2];
#pragma unroll
    for (int rg = 0; rg < NRG; ++rg)
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) s2[rg][blk] = attn_floatx4{0.f, 0.f, 0.f, 0.f};
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
      for (int e = 0; e < 8; ++e) vt[e] = sm.a.v[wv][(e >> 2) * 16 + sg4 * 4 + (e & 3)][db * 16 + srow];
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
  for (int ti = wslot; ti < n_tiles; ti += AHEAD) {
    process(SET0, ti);
    if (NSET == 2 && ti + AW < n_tiles) process(SET1, ti + AW);
  }
  // ---- the waves meet in LDS (the buffer aliases the V tiles and the queries)
  const int mrow = t / TPR, md = (t % TPR) * DPT;  // merge role: row within a row group, first of DPT dims
  const bool merger = t < 16 * TPR;                 // the first AW waves
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
    attn_store<COH, DPT * 2>(out + act_offset(ncg, B * R, n_heads * HD, 0, arow, ak), &hi);
    attn_store<COH, DPT * 2>(out + act_offset(ncg, B * R, n_heads * HD, 1, arow, ak), &lo);
  };
  if (active && dpart == 0) {  // (the waves that share a tile hold the same statistics)
#pragma unroll
    for (int rg = 0; rg < NRG; ++rg) {
      if (sg4 == 0) {
        sm.m[wslot][rg * 16 + srow] = m_run[rg];
        sm.l[wslot][rg * 16 + srow] = l_run[rg];
      }
    }
  }
  constexpr int MRG = NRG <= 2 ? NRG : 1;  // row groups the merge buffer holds at a time
#pragma unroll
  for (int rg0 = 0; rg0 < NRG; rg0 += MRG) {
    __syncthreads();  // everyone is done with the tiles (first pass) / with the previous row groups' buffer
    if (active) {
#pragma unroll
      for (int rm = 0; rm < MRG; ++rm)
#pragma unroll
        for (int db = 0; db < DB; ++db)
          *(float4*)&sm.o[wslot][rm * 16 + srow][dpart * HV + db * 16 + sg4 * 4] =
              make_float4(acc[rg0 + rm][db][0], acc[rg0 + rm][db][1], acc[rg0 + rm][db][2], acc[rg0 + rm][db][3]);
    }
    __syncthreads();
    if (merger) {
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
          } else {  // partial[seq][head][row][split][HD+2] = (m, l, acc[HD]) for the merge
            float* p = partial + ((((int64_t)seq * n_heads + pair_head(r)) * R + pair_row(r)) * n_splits + split) * (HD + 2);
#pragma unroll
            for (int x = 0; x < DPT; x += 2) st8<COH>(p + 2 + md + x, make_uint2(__float_as_uint(o[x]), __float_as_uint(o[x + 1])));
            if (t % TPR == 0) st8<COH>(p, make_uint2(__float_as_uint(M), __float_as_uint(L)));
          }
        }
      }
    }
  }
  return eff;
}

}  // namespace mtad
