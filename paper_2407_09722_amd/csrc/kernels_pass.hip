// Persistent decoder pass for bf16 models with few rows: one workgroup per compute unit runs every step of
// every layer (QKV product, tree attention, o product, gate/up product, down product) and the lm_head, with a
// software grid barrier between steps.  What this buys over one kernel per step:
//   * no kernel boundary (drain, launch, ramp-up: about 5 us each, 160 of them per 32-layer pass);
//   * the weight stream never stops: before a workgroup finishes a strip, and before it waits at a barrier, it
//     has already issued the loads of its next strip's first tiles (weights do not depend on activations), so HBM
//     keeps delivering while the grid synchronises.
// The kernel is an interpreter of a step list (pass.h): ONE instance of the product loop serves all five products,
// only the epilogue is selected per step, and the per-step parameters are scalar loads that live for one step.
// Work split: strip nt of a matrix belongs to workgroup nt mod G, its k tiles are interleaved over the workgroup's 8
// waves (as in the stand-alone product kernel, whose epilogues are reused).  Data handed from one step to the next
// (activation planes, sums of squares, q, new K/V rows) crosses XCDs, whose L2s are not coherent with each
// other: it is written with device-scope write-through stores and read with cache-bypassing loads, so the
// barrier itself needs no cache flush.  The residual stream never leaves its workgroup (strip nt of both
// residual products belongs to the same workgroup) and stays in ordinary cached memory.
// Every wait is bounded: a workgroup that gives up sets a status bit and the abort flag, and all others leave.
#include "attn_device.h"
#include "gemm_device.h"
#include "pass.h"

namespace mtad {

constexpr int PT = 512;  // threads per workgroup
constexpr int PW = PT / 64;
constexpr long SPIN_LIMIT = 400000;

// The step list and the arguments are read through constant-address-space pointers: scalar loads, issued where the
// value is needed, so that only one step's parameters occupy scalar registers at a time.
typedef const __attribute__((address_space(4))) PassStep* StepPtr;
typedef const __attribute__((address_space(4))) PassArgs* ArgPtr;

template <typename T>
__device__ __forceinline__ T ldc(const __attribute__((address_space(4))) T* p) {
  T v;
  __builtin_memcpy(&v, p, sizeof(T));
  return v;
}
// Hides a pointer's origin from the optimiser, so that loads through it are not merged with (or hoisted to) earlier ones.
template <typename P>
__device__ __forceinline__ P fresh(P p) {
  asm volatile("" : "+s"(p));
  return p;
}

// Arrive at and wait for grid barrier number `epoch` (1, 2, ...).  Returns false if the wait was abandoned.
// wait_stores: this wave may still have write-through stores in flight (it then waits for everything it has issued).
__device__ __forceinline__ bool grid_sync(unsigned long long* bar, uint32_t* status, unsigned& epoch, int* abort_s, bool wait_stores) {
  ++epoch;
  if (wait_stores) __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(bar, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long target = (unsigned long long)epoch * gridDim.x;
    int ok = 1;
    long spins = 0;
    while (__hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      __builtin_amdgcn_s_sleep(1);
      if (++spins > SPIN_LIMIT || __hip_atomic_load(bar + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0ull) {
        ok = 0;
        break;
      }
    }
    if (!ok) {
      atomicOr(status, (uint32_t)ST_TIMEOUT);
      __hip_atomic_store(bar + 1, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // abort flag: everyone leaves
    }
    *abort_s = !ok;
  }
  __syncthreads();
  return *abort_s == 0;
}

// The attention work of one layer: (split, head, chunk, sequence) items round-robin over the workgroups.
template <int HD>
__device__ __forceinline__ void attn_phase(ArgPtr A, AttnSmem<kv16_t, HD, PT>& sm, int layer, bf16_t* out) {
  const int Rseq = A->Rseq, H = A->H, B = A->B, n_splits = A->n_splits;
  const int n_chunks = (Rseq + RB - 1) / RB;
  const float scale = 1.0f / sqrtf((float)HD);
  const int items = n_splits * H * n_chunks * B;
  const RowDesc rd = ldc(&A->rd);
  const KvView kv = ldc(&A->kv);
  for (int it = blockIdx.x; it < items; it += gridDim.x) {
    const int split = it % n_splits, hc = (it / n_splits) % (H * n_chunks), seq = it / (n_splits * H * n_chunks);
    __syncthreads();  // the previous item is done with the shared tiles
    attn_item<kv16_t, bf16_t, HD, PT, true>(sm, A->q, H * HD, rd, kv, layer, B, Rseq, H, n_chunks, scale, A->partial, n_splits,
                                              A->attn_cnt, out, split, hc / n_chunks, hc % n_chunks, seq);
  }
}

// Addresses are written as (wave-uniform base) + (32-bit unsigned lane offset), the form the scalar-base addressing
// mode of global loads takes: one offset register per wave instead of a 64-bit address per load.
template <int U>
__device__ __forceinline__ void load_batch(Frag (&w)[U], const void* W, int KT, int nt, int kt, int lane) {
  const char* base = (const char*)W + (((int64_t)nt * KT + kt) << 10);  // tile (nt, kt): 1 KiB each, k-major within the strip
  const unsigned voff = (unsigned)lane * 16u;
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (kt + u * PW < KT) w[u].n = __builtin_nontemporal_load((const uintx4*)(base + (size_t)u * (PW << 10) + voff));
}

// Activation fragments (B operands) of one batch: tiles kt, kt + PW, ... of the input planes; rows beyond the pass read as zero.
// xoff: this lane's byte offset within the planes (plane, row within the group, k group).
template <int NG, int U>
__device__ __forceinline__ void load_b(Frag (&b)[U][NG], const bf16_t* X, unsigned xoff, int K, int KT, int kt, int rows_here, int c) {
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      b[u][g].u = make_uint4(0, 0, 0, 0);
      const char* base = (const char*)X + ((size_t)g * 8 * K + (size_t)(kt + u * PW) * 32) * 2;
      if (kt + u * PW < KT && g * 8 + (c & 7) < rows_here) b[u][g].u = *(const uint4*)(base + xoff);
    }
}

// acc += (weight tiles of one batch) x (the matching activation fragments)
template <int NG, int U>
__device__ __forceinline__ void mma_batch(floatx4 (&acc)[NG], const Frag (&w)[U], const Frag (&b)[U][NG], int KT, int kt) {
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (kt + u * PW < KT) {
#pragma unroll
      for (int g = 0; g < NG; ++g) acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[u].v, b[u][g].v, acc[g], 0, 0, 0);
    }
}

template <int NG>
__global__ __launch_bounds__(PT) void pass_kernel(const PassArgs* args) {
  constexpr int U = (NG <= 1) ? 8 : 4;  // weight tiles per batch and wave; two batches in flight (128 KiB per CU at U = 8)
  __shared__ floatx4 red[PW * NG * 64];
  __shared__ float inv_s[NG * 8];
  __shared__ AttnSmem<kv16_t, 128, PT> attn128;  // the larger of the two head sizes; the 64-wide variant aliases it
  __shared__ int abort_s;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform by construction: keep it scalar
  const int G = gridDim.x, bid = blockIdx.x;
  const int c = lane & 15, kg = lane >> 4;
  const ArgPtr A0 = (ArgPtr)args;
  const int rows = A0->rows, rows_here = min(NG * 8, rows), n_steps = A0->n_steps;
  const StepPtr steps = (StepPtr)A0->steps;
  unsigned long long* const bar = A0->bar;
  unsigned epoch = 0;
  if (threadIdx.x == 0) abort_s = 0;

  // the weight tiles this wave has in flight: first two batches of strip pf_nt of step pf_step
  Frag w[2][U];
  int pf_step = -1, pf_nt = -1;
  if (bid < (steps[0].N >> 4)) {  // layer 0's QKV weights need nothing from anyone
    load_batch<U>(w[0], steps[0].W, steps[0].K >> 5, bid, wave, lane);
    load_batch<U>(w[1], steps[0].W, steps[0].K >> 5, bid, wave + U * PW, lane);
    pf_step = 0;
    pf_nt = bid;
  }

#ifdef MTAD_PASS_PROFILE
  // timestamps (100 MHz): [workgroup][step - first recorded step][start, products done, end]
  unsigned long long* const prof = A0->prof + bid * 3 * 32;  // steps 20 .. 51 of every workgroup
  const int prof0 = n_steps > 52 ? 20 : 0;
#define PROF(k) if (s >= prof0 && s < prof0 + 32 && threadIdx.x == 0) prof[(s - prof0) * 3 + (k)] = wall_clock64()
#else
#define PROF(k)
#endif
  for (int s = 0; s < n_steps; ++s) {
    PROF(0);
    const StepPtr st = fresh(steps + s);
    const ArgPtr A = fresh(A0);
    const int kind = st->kind;
    if (kind == STEP_ATTN) {
      if (A->hd == 128) attn_phase<128>(A, attn128, st->layer, st->out);
      else attn_phase<64>(A, *(AttnSmem<kv16_t, 64, PT>*)&attn128, st->layer, st->out);
    } else {
      GemmArgs a;
      a.W = (const bf16_t*)st->W; a.N = st->N; a.K = st->K; a.layer = st->layer;
      a.R = rows; a.row0 = 0; a.ncg = 0; a.eps = A->eps;  // activations as planes
      const bool normed = kind == STEP_QKV || kind == STEP_GATE_UP || kind == STEP_HEAD;  // input = planes of h*gain
      a.X = st->X;
      a.ssq = normed ? A->ssq : nullptr;
      a.NP = st->np;
      a.Y = nullptr; a.ldy = 0; a.accumulate = 0; a.lse_part = nullptr;
      a.h = nullptr; a.g_next = nullptr; a.planes_out = nullptr; a.ssq_out = nullptr; a.act_out = nullptr;
      a.q_out = nullptr; a.rope = nullptr; a.slot = nullptr; a.Rseq = 1; a.n_heads = 0; a.status = nullptr;
      const int K = a.K, KT = K >> 5, NT = a.N >> 4;
      const int next = st->next;
      const bf16_t* xp = a.X;
      const unsigned xoff = (unsigned)(((c >> 3) * rows * K + (c & 7) * K + kg * 8) * 2);  // < 2^31: rows <= 32, K < 2^20
      gemm_row_factors<true>(a, inv_s, rows_here, wave, lane, PW);  // visible after the first strip's barrier

      const int span = U * PW;                            // k tiles one batch of the whole workgroup covers
      const int nb2 = ((KT + span - 1) / span + 1) & ~1;  // batch slots per strip, padded to an even number
      // One flat loop over this workgroup's (strip, batch) stream, two batches per trip (register sets 0 and 1).  After a
      // batch is consumed its registers take the batch two places further down the stream: of this strip, of the next
      // strip, or of the first strip of the next product step.  Loads complete in issue order, so a wave that waits
      // for its newest load has waited for all of them: the activation fragments of a batch are issued BEFORE its
      // weight tiles (two batches ahead of their use), never between a batch's weight loads and its use.  Fragments
      // depend on the batch, not on the strip: with two batches per strip they are loaded once per step.
      int nt = bid;
      if (nt < NT) {
        Frag b[2][U][NG];
        if (pf_step != s || pf_nt != nt) {  // nothing usable was prefetched
          load_batch<U>(w[0], a.W, KT, nt, wave, lane);
          load_batch<U>(w[1], a.W, KT, nt, wave + span, lane);
        }
        load_b<NG, U>(b[0], xp, xoff, K, KT, wave, rows_here, c);
        load_b<NG, U>(b[1], xp, xoff, K, KT, wave + span, rows_here, c);
        const void* nW = nullptr;  // the next product step's weights, if this workgroup has a strip there
        int nKT = 0;
        if (next >= 0 && bid < (steps[next].N >> 4)) {
          nW = steps[next].W;
          nKT = steps[next].K >> 5;
        }
        floatx4 acc[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};
        int jb = 0;  // first batch of the current pair
        for (;;) {
          const bool more = nt + G < NT;
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            mma_batch<NG, U>(acc, w[h], b[h], KT, wave + (jb + h) * span);
            int jn = jb + h + 2;  // the stream element that takes over register set h
            const void* Wn = a.W;
            int KTn = KT, ntn = nt;
            bool need_b = true;
            if (jn >= nb2) {
              jn -= nb2;
              ntn = nt + G;
              need_b = nb2 > 2;
              if (!more) {
                // A wave that stores results waits for its stores before the grid barrier, and that wait would also cover
                // weight loads issued before it: such a wave fetches the next step's batches after its stores (below).
                Wn = wave < NG ? nullptr : nW;
                KTn = nKT;
                ntn = bid;
                need_b = false;
              }
            }
            if (need_b) load_b<NG, U>(b[h], xp, xoff, K, KT, wave + jn * span, rows_here, c);
            if (Wn) load_batch<U>(w[h], Wn, KTn, ntn, wave + jn * span, lane);
          }
          jb += 2;
          if (jb < nb2) continue;
          // ---- end of a strip: partial sums meet in LDS, waves 0 .. NG-1 run the epilogue of one row group each
#pragma unroll
          for (int g = 0; g < NG; ++g) red[(wave * NG + g) * 64 + lane] = acc[g];
          PROF(1);
          __syncthreads();
          if (wave < NG) {  // the epilogue's own parameters are loaded here, by the waves that need them
            const ArgPtr E = fresh(A0);
            if (kind == STEP_QKV) {
              a.q_out = E->q; a.rope = E->rope; a.slot = E->rd.slot; a.kv = ldc(&E->kv); a.Rseq = E->Rseq; a.n_heads = E->H; a.status = E->status;
              gemm_finish_group<NG, EPI_QKV, true, PW>(a, nt, wave, red, inv_s, rows_here, lane);
            } else if (kind == STEP_GATE_UP) {
              a.act_out = fresh(st)->out;
              gemm_finish_group<NG, EPI_SWIGLU, true, PW>(a, nt, wave, red, inv_s, rows_here, lane);
            } else if (kind == STEP_HEAD) {
              a.Y = E->logits; a.ldy = E->vocab; a.lse_part = E->lse_part;
              gemm_finish_group<NG, EPI_STORE, true, PW>(a, nt, wave, red, inv_s, rows_here, lane);
            } else {
              a.h = E->h; a.g_next = fresh(st)->g_next; a.planes_out = fresh(st)->out; a.ssq_out = E->ssq;
              gemm_finish_group<NG, EPI_RESID, true, PW>(a, nt, wave, red, inv_s, rows_here, lane);
            }
            if (!more) {
              __builtin_amdgcn_s_waitcnt(0);  // this wave's stores of this step have been acknowledged
              if (nW) {
                load_batch<U>(w[0], nW, nKT, bid, wave, lane);
                load_batch<U>(w[1], nW, nKT, bid, wave + span, lane);
              }
            }
          }
          __syncthreads();  // red is reused by the next strip
          if (!more) break;
          nt += G;
          jb = 0;
#pragma unroll
          for (int g = 0; g < NG; ++g) acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
        pf_step = nW ? next : -1;
        pf_nt = bid;
      }
    }
    PROF(2);
    if (s + 1 < n_steps && !grid_sync(bar, A0->status, epoch, &abort_s, kind == STEP_ATTN)) return;
  }
}

bool pass_supported(int rows, int n_layers) { return rows >= 1 && rows <= PASS_MAX_ROWS && n_layers <= PASS_MAX_LAYERS; }

void pass_build_steps(PassStep* steps, const void* const* W, int n_layers, int d, int f, int H, int KVH, int hd, int vocab,
                      const bf16_t* x0, bf16_t* act, int max_rows) {
  const int tail = 1 + 6 * n_layers, hhd = H * hd;
  int n = 0;
  auto add = [&](int kind, const void* w, const void* g, const bf16_t* X, bf16_t* out, int N, int K, int layer, int np) {
    PassStep& p = steps[n++];
    p = PassStep{};
    p.W = w; p.g_next = (const float*)g; p.X = X; p.out = out; p.kind = kind; p.N = N; p.K = K; p.layer = layer; p.np = np; p.next = -1;
  };
  const bf16_t* x_in = x0;  // planes of h*gain entering the layer
  for (int l = 0; l < n_layers; ++l) {
    const void* const* L = W + 1 + 6 * l;  // g_attn, w_qkv, w_o, g_ffn, w_gate_up, w_down
    bf16_t* xa = act + (size_t)l * pass_act_elems_per_layer(d, hhd, f, max_rows);
    bf16_t* xg2 = xa + (size_t)2 * max_rows * hhd;
    bf16_t* xf = xg2 + (size_t)2 * max_rows * d;
    bf16_t* xnext = xf + (size_t)2 * max_rows * f;
    add(STEP_QKV, L[1], nullptr, x_in, nullptr, (H + 2 * KVH) * hd, d, l, l == 0 ? 1 : d / 16);
    add(STEP_ATTN, nullptr, nullptr, nullptr, xa, 0, 0, l, 0);
    add(STEP_O, L[2], L[3], xa, xg2, d, hhd, l, 0);
    add(STEP_GATE_UP, L[4], nullptr, xg2, xf, 2 * f, d, l, d / 16);
    add(STEP_DOWN, L[5], l + 1 == n_layers ? W[tail] : W[1 + 6 * (l + 1)], xf, xnext, d, f, l, 0);
    x_in = xnext;
  }
  add(STEP_HEAD, W[tail + 1], nullptr, x_in, nullptr, vocab, d, n_layers, d / 16);
  for (int i = 0; i < n; ++i) {  // link every product step to the product step after it
    if (steps[i].kind == STEP_ATTN) continue;
    int j = i + 1;
    while (j < n && steps[j].kind == STEP_ATTN) ++j;
    steps[i].next = j < n ? j : -1;
  }
}

// Copies the arguments to device memory (stream-ordered, so a pass still running keeps its own) and zeroes the barrier.
__global__ void pass_setup_kernel(PassArgs a, PassArgs* dst, unsigned long long* bar) {
  if (threadIdx.x == 0) {
    *dst = a;
    bar[0] = 0ull;
    bar[1] = 0ull;
  }
}

hipError_t launch_pass(const PassArgs& a, PassArgs* dev_args, int n_cus, hipStream_t s) {
  if (a.n_steps < 1 || a.rows < 1 || a.rows > PASS_MAX_ROWS || n_cus < 1 || !dev_args) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pass_setup_kernel, dim3(1), dim3(64), 0, s, a, dev_args, a.bar);
  const int ng = (a.rows + 7) / 8;
  dim3 grid(n_cus), block(PT);
  const PassArgs* p = dev_args;
  if (ng <= 1) hipLaunchKernelGGL(pass_kernel<1>, grid, block, 0, s, p);
  else if (ng <= 2) hipLaunchKernelGGL(pass_kernel<2>, grid, block, 0, s, p);
  else if (ng <= 3) hipLaunchKernelGGL(pass_kernel<3>, grid, block, 0, s, p);
  else hipLaunchKernelGGL(pass_kernel<4>, grid, block, 0, s, p);
  return hipGetLastError();
}

}  // namespace mtad
