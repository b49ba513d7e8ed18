// The decoder pass of a bf16 model over a few rows (at most 8: the chain of a draft, a beam step, one token) as ONE kernel
// launch.  The paper's cost argument (Section 4: a run costs what it moves from global memory) makes the weight stream the
// floor of a verification pass (Algorithm 1: P <- M_p(input, X)); with one kernel per product, every kernel boundary
// drains that stream and ramps it up again, about 3 us each, six times per layer.  Here the products and the attention of
// all layers are work units of one grid:
//
//   * A unit is what a workgroup of the per-step kernels does: one or three strips of 16 output features of a product
//     (same loops, same tile-packed weights, same fused epilogues as kernels_gemm.hip) or one attention work item
//     (attn_mfma_device.h).  Units are numbered in dependency order: all units of step s before any unit of step s + 1.
//   * Workgroups are persistent: as many as the machine holds at once, workgroup b runs units b, b + G, b + 2G, ...
//     Every unit of a step needs the whole step before it (each product reduces over all features the previous one
//     wrote), so a unit waits until the previous step's flag is up (flow.h: sharded counters, one flag per step).  A
//     workgroup only ever waits for units with smaller numbers, which belong to workgroups that are resident and working
//     through their lists in order, so the pass cannot block itself; and every wait is bounded as well: a wall-clock limit
//     sets a status bit and an abort flag that ends all waiting (a launch that shares the machine with a foreign kernel
//     and does not get all its workgroups resident ends that way instead of hanging).
//   * Weights do not depend on activations: a unit requests its first two batches of weight tiles BEFORE it waits.  While
//     the last units of a step finish their epilogues, the waiting units of the next step already have 64 KiB per
//     workgroup in flight, so the memory system keeps streaming across what used to be a kernel boundary.
//   * What one step hands to the next crosses XCDs, whose L2 caches are not coherent with each other: it is written with
//     device-scope write-through stores, acknowledged before the unit counts as finished.  Buffers that every unit of the
//     next step reads in full (activation terms, sums of squares, queries) exist once per producing step, so a line is
//     written once per pass and read only afterwards through the ordinary caches, which start clean at every launch;
//     small exchanges (attention split partials, the residual stream, the counters) bypass the caches.
#include "attn_mfma_device.h"
#include "flow.h"
#include "gemm.h"
#include "gemm_device.h"

namespace mtad {

namespace {

constexpr int FT = 512;                                      // threads per workgroup (GW waves)
constexpr unsigned long long FLOW_SPIN_TICKS = 20000000ull;  // 0.2 s of the 100 MHz wall clock: far beyond any pass

#ifdef MTAD_FLOW_PROFILE
#define FLOW_STAMP(pr, k) do { if (tid == 0 && (pr)) (pr)[k] = wall_clock64(); } while (0)
#else
#define FLOW_STAMP(pr, k) do { } while (0)
#endif

template <int HD>
struct FlowSmem {
  union {
    floatx4 red[3 * GW * 64];  // partial sums of up to three strips, [strip][wave][lane]
    MfmaAttnSmem<HD, 1, ATTN_WAVES, HD == 128 ? 2 : 1> attn;
  };
  float inv_s[8];
  int flag;
};

// Waits until the flag is up (thread 0 polls past the caches, backing off; everyone meets at the barrier).  Gives up on the
// abort flag or after FLOW_SPIN_TICKS, then sets both the status bit and the flag: the pass runs on with whatever it finds
// and ends.
__device__ __forceinline__ void flow_wait(const int* flag, int* sync, uint32_t* status, int tid) {
  if (tid == 0 && __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
    const unsigned long long t0 = wall_clock64();
    for (int spins = 0;; ++spins) {
      if (spins < 8) __builtin_amdgcn_s_sleep(4);
      else __builtin_amdgcn_s_sleep(12);
      if (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
      if ((spins & 15) == 15) {
        if (__hip_atomic_load(sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
        if (wall_clock64() - t0 > FLOW_SPIN_TICKS) {
          atomicOr(status, (uint32_t)ST_TIMEOUT);
          __hip_atomic_store(sync, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
      }
    }
  }
  __syncthreads();
}

// Unit u of the n units of step `step` has finished (its stores are acknowledged): count it; the last unit of a shard counts
// the shard, the last shard raises the step's flags.  One thread.
__device__ __forceinline__ void flow_signal(int* sync, int step, int u, int n) {
  const int j = u % FLOW_SHARDS;
  const int in_shard = (n - j + FLOW_SHARDS - 1) / FLOW_SHARDS;  // units of this step that count in shard j
  const int prev = __hip_atomic_fetch_add(sync + FLOW_SHARD_BASE + (step * FLOW_SHARDS + j) * 32, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (prev != in_shard - 1) return;
  const int shards = n < FLOW_SHARDS ? n : FLOW_SHARDS;
  const int prev2 = __hip_atomic_fetch_add(sync + 8 + step, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (prev2 != shards - 1) return;
#pragma unroll
  for (int c = 0; c < FLOW_FLAGS; ++c)
    __hip_atomic_store(sync + FLOW_FLAG_BASE + (step * FLOW_FLAGS + c) * 32, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// What the streaming part of a product unit needs.  The epilogue's many pointers are loaded after it.
struct FlowStream {
  const bf16_t* W;
  const bf16_t* X;
  int R, N, K, ncg;
  int S;  // strips per unit: 3 (two weight tiles per batch and wave) or 1 (four)
};

// The streaming part of one product unit: S strips of 16 output features, U weight tiles per batch and wave, two batches
// in flight; one row group (at most 8 rows).  The loops are those of gemm_bf16_strips_kernel; the difference is the order
// at the start: the first two batches of weights (which depend on no activation) are requested first, then comes the wait
// for the step that produces the activations, then the activation fragments.  (Requesting the weights earlier still, while
// the workgroup's previous unit runs its epilogue, was measured and lost: the epilogue's few memory operations then queue
// behind 96 KiB of prefetch, and the step ends later.)
// With the first activation fragments go the few loads the epilogue will want (FlowEarly), so that the epilogue is not a
// chain of memory round trips queued behind whatever the compute unit's other workgroup is streaming; they must not go
// out before the wait: only then is everything earlier steps wrote final.
// Leaves the waves' partial sums in sm.red ([strip][wave][lane]); the caller synchronises and finishes the strips.
struct FlowEarly {
  const float* ssq_row;  // this wave's row of the producer's partial sums of squares (NP of them, at most 256), or null
  int NP;
  const float* h;        // finishing wave of an o / down product: this lane's residual values (4 floats) and next-norm gains, or null
  const float* gn;
  float sv[4];
  float4 pre_h, pre_gn;
};
template <int S, int U, int HD>
__device__ __forceinline__ void flow_stream(FlowSmem<HD>& sm, const FlowStream& p, int unit, const int* wait_flag, int* sync,
                                            uint32_t* status, FlowEarly& e, int tid, int lane, int wave, unsigned long long* pr) {
  const int KT = p.K >> 5, NT = p.N >> 4;
  const int c = lane & 15;
  const int nt0 = unit * S, ns = min(S, NT - nt0);
  const size_t strip_bytes = (size_t)KT << 10;
  const char* strip0 = (const char*)p.W + (size_t)nt0 * strip_bytes;
  const unsigned voff = (unsigned)lane * 16u;
  constexpr int span = U * GW;
  Frag w[2][U * S], b[2][U][1];
  auto load_w = [&](int h, int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int s2 = 0; s2 < S; ++s2)
        if (kt + u * GW < KT)
          w[h][u * S + s2].n = __builtin_nontemporal_load((const uintx4*)(strip0 + (size_t)min(s2, ns - 1) * strip_bytes + ((size_t)(kt + u * GW) << 10) + voff));
  };
  load_w(0, wave);
  load_w(1, wave + span);
  if (wait_flag) flow_wait(wait_flag, sync, status, tid);
  FLOW_STAMP(pr, 1);
  GemmArgs xa_args;  // act_addr reads the layout fields only
  xa_args.X = p.X;
  xa_args.R = p.R;
  xa_args.K = p.K;
  xa_args.ncg = p.ncg;
  xa_args.row0 = 0;
  const ActAddr xa = act_addr(xa_args, lane);
  gemm_load_b<1, U>(b[0], xa.X, xa.xoff, xa.kstride, xa.gstride, KT, wave, p.R, c);
  gemm_load_b<1, U>(b[1], xa.X, xa.xoff, xa.kstride, xa.gstride, KT, wave + span, p.R, c);
  if (e.ssq_row) {
#pragma unroll
    for (int i = 0; i < 4; ++i) e.sv[i] = e.ssq_row[min(lane + 64 * i, e.NP - 1)];
  }
  if (e.h) {  // written by a workgroup of this kernel (an earlier step's strip owner): past the caches
    const uint4 u4 = ld16<true>(e.h);
    e.pre_h = make_float4(__uint_as_float(u4.x), __uint_as_float(u4.y), __uint_as_float(u4.z), __uint_as_float(u4.w));
    e.pre_gn = *(const float4*)e.gn;
  }

  floatx4 acc[S];
#pragma unroll
  for (int s2 = 0; s2 < S; ++s2) acc[s2] = floatx4{0.f, 0.f, 0.f, 0.f};
  for (int kt = wave; kt < KT; kt += 2 * span) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int k0 = kt + h * span;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (k0 + u * GW < KT) {
#pragma unroll
          for (int s2 = 0; s2 < S; ++s2) acc[s2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[h][u * S + s2].v, b[h][u][0].v, acc[s2], 0, 0, 0);
        }
      if (k0 + 2 * span < KT) {
        gemm_load_b<1, U>(b[h], xa.X, xa.xoff, xa.kstride, xa.gstride, KT, k0 + 2 * span, p.R, c);
        load_w(h, k0 + 2 * span);
      }
    }
  }
#pragma unroll
  for (int s2 = 0; s2 < S; ++s2) sm.red[(s2 * GW + wave) * 64 + lane] = acc[s2];
  FLOW_STAMP(pr, 2);
}

// The arguments live in device memory and are read through a constant-address-space pointer: scalar loads issued where
// a value is needed, so that only one unit's parameters occupy registers at a time (as kernel arguments the whole
// record would be loaded at the start and spilled).
typedef const __attribute__((address_space(4))) FlowArgs* FlowPtr;
template <typename T>
__device__ __forceinline__ T ldc(const __attribute__((address_space(4))) T* p) {
  T v;
  __builtin_memcpy(&v, p, sizeof(T));
  return v;
}

struct FlowUnit {
  int kind, layer, idx, step;
};

template <int HD>
__global__ __launch_bounds__(FT) __attribute__((amdgpu_waves_per_eu(4, 4))) void flow_pass_kernel(const FlowArgs* args, int s_begin, int s_end) {
  __shared__ FlowSmem<HD> sm;
  const FlowPtr A = (FlowPtr)args;
  const int L = A->n_layers;
  const int u_qkv = A->units[FK_QKV], u_attn = A->units[FK_ATTN], u_o = A->units[FK_O], u_gu = A->units[FK_GU], u_down = A->units[FK_DOWN],
            u_head = A->units[FK_HEAD];
  const int UL = u_qkv + u_attn + u_o + u_gu + u_down;  // units of a layer
  auto units_of = [&](int k) { return k == FK_QKV ? u_qkv : k == FK_ATTN ? u_attn : k == FK_O ? u_o : k == FK_GU ? u_gu : k == FK_DOWN ? u_down : u_head; };
  auto first_unit = [&](int s) {  // global number of the first unit of step s (s = 5L + 1: one past the lm_head)
    if (s >= 5 * L) return L * UL + (s > 5 * L ? u_head : 0);
    int g = (s / 5) * UL;
    for (int k = 0; k < s % 5; ++k) g += units_of(k);
    return g;
  };
  const int g_begin = first_unit(s_begin), g_end = first_unit(s_end);
  int* const sync = A->sync;
  int* const item_cnt = sync + FLOW_ITEM_BASE;
  const int tail = 1 + 6 * L;

  auto decode = [&](int g) {
    FlowUnit u;
    if (g < L * UL) {
      u.layer = g / UL;
      u.idx = g % UL;
      u.kind = 0;
      while (u.idx >= units_of(u.kind)) {
        u.idx -= units_of(u.kind);
        ++u.kind;
      }
      u.step = 5 * u.layer + u.kind;
    } else {
      u.kind = FK_HEAD;
      u.layer = L;
      u.idx = g - L * UL;
      u.step = 5 * L;
    }
    return u;
  };
  // what the streaming part of product unit u reads (u.kind != FK_ATTN)
  auto stream_of = [&](const FlowUnit& u) {
    FlowStream p;
    const int d = A->d, f = A->f, hhd = A->H * HD;
    const int wl = 1 + 6 * (u.kind == FK_HEAD ? 0 : u.layer);
    p.R = A->rows;
    p.ncg = A->ncg;
    p.S = A->strips[u.kind];
    if (u.kind == FK_QKV) {
      p.W = (const bf16_t*)A->w[wl + 1];
      p.X = A->xg + (size_t)(2 * u.layer) * A->xg_stride;
      p.N = (A->H + 2 * A->KVH) * HD;
      p.K = d;
    } else if (u.kind == FK_O) {
      p.W = (const bf16_t*)A->w[wl + 2];
      p.X = A->xattn + (size_t)u.layer * A->xattn_stride;
      p.N = d;
      p.K = hhd;
    } else if (u.kind == FK_GU) {
      p.W = (const bf16_t*)A->w[wl + 4];
      p.X = A->xg + (size_t)(2 * u.layer + 1) * A->xg_stride;
      p.N = 2 * f;
      p.K = d;
    } else if (u.kind == FK_DOWN) {
      p.W = (const bf16_t*)A->w[wl + 5];
      p.X = A->xffn + (size_t)u.layer * A->xffn_stride;
      p.N = d;
      p.K = f;
    } else {
      p.W = (const bf16_t*)A->w[tail + 1];
      p.X = A->xg + (size_t)(2 * L) * A->xg_stride;
      p.N = A->vocab;
      p.K = d;
    }
    return p;
  };

#ifdef MTAD_FLOW_PROFILE
  if (threadIdx.x == 0 && A->prof)  // where this workgroup runs: (XCC id, hardware id word) behind the unit stamps
    A->prof[4 * 90000 + blockIdx.x] = ((unsigned long long)__builtin_amdgcn_s_getreg((3 << 11) | 20) << 32) | (unsigned)__builtin_amdgcn_s_getreg((31 << 11) | 4);
#endif
  int g = g_begin + (int)blockIdx.x;
  if (g >= g_end) return;
  FlowUnit cur = decode(g);
  for (;;) {
    // The thread index is made opaque once per unit: what a unit derives from it (lane offsets, LDS addresses) is then
    // computed inside the unit instead of being hoisted out of this loop and kept in registers across all unit kinds.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#ifdef MTAD_FLOW_PROFILE
    unsigned long long* const pr = A->prof ? A->prof + (size_t)g * 4 : nullptr;
#else
    unsigned long long* const pr = nullptr;
#endif
    FLOW_STAMP(pr, 0);
    const int kind = cur.kind, layer = cur.layer, idx = cur.idx, step = cur.step;
    const int g_next = g + (int)gridDim.x;
    const bool more = g_next < g_end;
    FlowUnit nxt = cur;
    if (more) nxt = decode(g_next);
    // the step before this one must be complete, unless an earlier launch ran it
    const int* wait_flag = step > s_begin ? sync + FLOW_FLAG_BASE + ((step - 1) * FLOW_FLAGS + ((int)blockIdx.x % FLOW_FLAGS)) * 32 : nullptr;
    uint32_t* const status = A->status;
    const int H = A->H, KVH = A->KVH, hhd = H * HD;
    if (kind == FK_ATTN) {
      const int gx = A->attn_gx, n_chunks = A->attn_chunks, per_seq = KVH * n_chunks;
      const int split = idx % gx, gc = (idx / gx) % per_seq, seq = idx / (gx * per_seq);
      const int kvh = gc / n_chunks, chunk = gc % n_chunks;
      const int Rseq = A->Rseq, B = A->B, ncg = A->ncg, n_splits = A->n_splits;
      bf16_t* const out = A->xattn + (size_t)layer * A->xattn_stride;
      float* const partial = A->partial;
      const KvView kv = ldc(&A->kv);
      const RowDesc rd = ldc(&A->rd);
      const int eff = tree_attn_item<HD, 1, ATTN_WAVES, 1, FT, true, HD == 128 ? 2 : 1>(sm.attn, A->q + (size_t)layer * A->q_stride, hhd, rd, kv, layer, B, Rseq, H,
                                                                      n_chunks, 1.0f / sqrtf((float)HD), partial, n_splits, out, A->attn_want, ncg,
                                                                      split, kvh, chunk, seq, tid, [&]() {
                                                                        // K and V of the committed context are on their way; the
                                                                        // queries and the new rows' K / V need this layer's QKV product
                                                                        if (wait_flag) flow_wait(wait_flag, sync, status, tid);
                                                                        FLOW_STAMP(pr, 1);
                                                                      });
      FLOW_STAMP(pr, 2);
      if (eff > 1 && split < eff) {  // uniform over the workgroup
        // the split that arrives last for its item merges the item's rows (split order: deterministic)
        __builtin_amdgcn_s_waitcnt(0);  // the partial results have been acknowledged
        __syncthreads();
        if (tid == 0) {
          int* cnt = item_cnt + seq * per_seq + gc;
          const int prev = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          sm.flag = prev == eff - 1;
          if (prev == eff - 1) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // clean for the next layer
        }
        __syncthreads();
        if (sm.flag) {
          const int G = H / KVH, pair0 = chunk * 16, nrows = min(16, G * Rseq - pair0);
          for (int r = wave; r < nrows; r += GW) {
            const int head = kvh * G + (pair0 + r) / Rseq, row = (pair0 + r) % Rseq;
            const float* pp = partial + (((int64_t)seq * H + head) * Rseq + row) * n_splits * (HD + 2);
            attn_merge_row<HD, true>(pp, eff, out, ncg, B * Rseq, hhd, seq * Rseq + row, head, lane);
          }
        }
      }
      // the unit's results must have been acknowledged by the memory system before it counts as finished
      __builtin_amdgcn_s_waitcnt(0);
    } else {
      const FlowStream p = stream_of(cur);
      const int d = A->d;
      const int wl = 1 + 6 * (kind == FK_HEAD ? 0 : layer);
      const int S = p.S;
      const int nt0 = idx * S, ns = min(S, (p.N >> 4) - nt0);
      const bool finisher = wave < ns;  // wave s2 finishes strip s2, the strips side by side
      // the producer's partial sums of squares, where the input is RMS-normalised
      const float* ssq = nullptr;
      int NP = 0;
      if (kind == FK_QKV || kind == FK_GU || kind == FK_HEAD) {
        const int v = kind == FK_QKV ? 2 * layer : kind == FK_GU ? 2 * layer + 1 : 2 * L;
        ssq = A->ssq + (size_t)v * A->ssq_stride;
        NP = v == 0 ? 1 : d / 16;
      }
      FlowEarly e;
      e.ssq_row = nullptr;
      e.NP = NP;
      e.h = nullptr;
      e.gn = nullptr;
      e.sv[0] = e.sv[1] = e.sv[2] = e.sv[3] = 0.f;
      e.pre_h = float4{0.f, 0.f, 0.f, 0.f};
      e.pre_gn = e.pre_h;
      const bool early_sums = ssq && NP <= 256;
      if (early_sums && wave < p.R) e.ssq_row = ssq + (size_t)wave * NP;  // wave m reduces row m (at most 8 rows)
      const bool resid = kind == FK_O || kind == FK_DOWN;
      if (resid && finisher) {
        const int c = lane & 15, kg = lane >> 4;
        if (c < 8 && (c & 7) < p.R) {
          const int n = (nt0 + wave) * 16 + kg * 4;
          e.h = A->h + (int64_t)(c & 7) * p.N + n;
          e.gn = (const float*)(kind == FK_O ? A->w[wl + 3] : (layer + 1 < L ? A->w[1 + 6 * (layer + 1)] : A->w[tail])) + n;
        }
      }
      if (S == 3) flow_stream<3, 2, HD>(sm, p, idx, wait_flag, sync, status, e, tid, lane, wave, pr);
      else flow_stream<1, 4, HD>(sm, p, idx, wait_flag, sync, status, e, tid, lane, wave, pr);
      // the epilogue's arguments, loaded now that the stream's registers are free
      GemmArgs ga;
      ga.R = p.R;
      ga.N = p.N;
      ga.K = p.K;
      ga.ncg = p.ncg;
      ga.row0 = 0;
      ga.eps = A->eps;
      ga.ssq = ssq;
      ga.NP = NP;
      ga.accumulate = 0;
      ga.lse_part = nullptr;
      ga.status = status;
      if (ssq) {
        if (early_sums) {
          if (wave < p.R) {
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (lane + 64 * i < NP) sum += e.sv[i];
            for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
            if (lane == 0) sm.inv_s[wave] = 1.0f / sqrtf(sum / (float)p.K + ga.eps);
          }
        } else {
          gemm_row_factors<false, 1>(ga, sm.inv_s, ga.R, wave, lane, GW);
        }
      }
      __syncthreads();  // partial sums and row factors are in LDS
      if (finisher) {
        const floatx4* r = sm.red + wave * GW * 64;
        const int nt = nt0 + wave;
        if (kind == FK_QKV) {
          ga.q_out = A->q + (size_t)layer * A->q_stride;
          ga.rope = A->rope;
          ga.slot = A->rd.slot;
          ga.kv = ldc(&A->kv);
          ga.layer = layer;
          ga.Rseq = A->Rseq;
          ga.n_heads = H;
          gemm_finish_group<1, EPI_QKV, true>(ga, nt, 0, r, sm.inv_s, ga.R, lane);
        } else if (kind == FK_GU) {
          ga.act_out = A->xffn + (size_t)layer * A->xffn_stride;
          gemm_finish_group<1, EPI_SWIGLU, true>(ga, nt, 0, r, sm.inv_s, ga.R, lane);
        } else if (kind == FK_HEAD) {
          ga.Y = A->logits;
          ga.ldy = A->vocab;
          ga.lse_part = A->lse_part;
          gemm_finish_group<1, EPI_STORE, true>(ga, nt, 0, r, sm.inv_s, ga.R, lane);
        } else {  // o and down products: residual add, then the next norm's input
          const int v = kind == FK_O ? 2 * layer + 1 : 2 * layer + 2;
          ga.h = A->h;
          ga.g_next = nullptr;  // (requested ahead)
          ga.planes_out = A->xg + (size_t)v * A->xg_stride;
          ga.ssq_out = A->ssq + (size_t)v * A->ssq_stride;
          gemm_finish_group<1, EPI_RESID, true, GW, true>(ga, nt, 0, r, sm.inv_s, ga.R, lane, e.pre_h, e.pre_gn);
        }
        // the strip's results must have been acknowledged by the memory system before the unit counts as finished
        __builtin_amdgcn_s_waitcnt(0);
      }
    }
    // The barrier also keeps the next unit's writes to the shared arrays behind this unit's reads; thread 0 signals while
    // the others go on.
    __syncthreads();
    FLOW_STAMP(pr, 3);
    if (tid == 0) flow_signal(sync, step, idx, units_of(kind));
    if (!more) break;
    cur = nxt;
    g = g_next;
  }
}

// Before the first launch of a pass: the argument record goes to device memory, the synchronisation words to zero (a
// kernel, not a memset: the pass must be recordable into a graph).
__global__ void flow_setup_kernel(FlowArgs a, FlowArgs* dev, int* sync, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  static_assert(sizeof(FlowArgs) % 4 == 0, "copied word by word");
  if (i < (int)(sizeof(FlowArgs) / 4)) ((uint32_t*)dev)[i] = ((const uint32_t*)&a)[i];
  if (i < n) sync[i] = 0;
}

int device_cus() {
  static const int n_cus = [] {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
    return cus > 0 ? cus : 256;
  }();
  return n_cus;
}

template <int HD>
hipError_t run_flow(const FlowArgs& a, const FlowArgs* dev, int s_begin, int s_end, hipStream_t s) {
  auto kern = flow_pass_kernel<HD>;
  static const int per_cu = [&] {  // resident workgroups per compute unit
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, (const void*)kern, FT, 0) != hipSuccess) n = 1;
    return n > 0 ? n : 1;
  }();
  const int L = a.n_layers;
  int total = 0;
  for (int st = s_begin; st < s_end; ++st) total += a.units[st >= 5 * L ? FK_HEAD : st % 5];
  if (total <= 0) return hipSuccess;
  const int slots = device_cus() * per_cu;
  hipLaunchKernelGGL(kern, dim3(total < slots ? total : slots), dim3(FT), 0, s, dev, s_begin, s_end);
  return hipGetLastError();
}

}  // namespace

void flow_attention_plan(int KVH, int n_chunks, int B, int n_splits, int* gx, int* want) {
  const int n_cus = device_cus();
  const int items = KVH * n_chunks * B;
  const int fill = items >= n_cus ? 1 : (n_cus + items - 1) / items;  // splits that give every compute unit a work item
  const int fill8 = fill < 255 ? fill : 255;
  *want = fill8;
  *gx = n_splits < fill8 ? n_splits : fill8;
}

hipError_t launch_flow_setup(const FlowArgs& a, FlowArgs* dev, int* sync, int n, hipStream_t s) {
  const int words = (int)(sizeof(FlowArgs) / 4), m = n > words ? n : words;
  hipLaunchKernelGGL(flow_setup_kernel, dim3((m + 255) / 256), dim3(256), 0, s, a, dev, sync, n);
  return hipGetLastError();
}

hipError_t launch_flow(const FlowArgs& a, const FlowArgs* dev, int s_begin, int s_end, hipStream_t s) {
  if (a.rows < 1 || a.rows > FLOW_MAX_ROWS || a.n_layers < 1 || a.n_layers > FLOW_MAX_LAYERS) return hipErrorInvalidValue;
  if (s_begin < 0 || s_end > 5 * a.n_layers + 1 || s_begin >= s_end) return hipErrorInvalidValue;
  if (a.hd == 128) return run_flow<128>(a, dev, s_begin, s_end, s);
  if (a.hd == 64) return run_flow<64>(a, dev, s_begin, s_end, s);
  return hipErrorInvalidValue;
}

}  // namespace mtad
