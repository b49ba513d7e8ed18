// Matrix products Y[R][N] = X[R][K] * W[N][K]^T for passes of many rows (a batch of token trees, Section 3.3, or a
// slab of prompt rows): the same operands, packing and epilogues as the skinny kernels (kernels_gemm.hip), but with
// both operands staged through LDS, because with 100+ rows the activation fragments a weight tile needs are 20x its
// own size and can no longer come from L2 per wave, and the product is as close to the matrix cores' bound as to the
// memory bound.
//
// One workgroup (8 waves) owns TN = 4*WS strips of 16 output features and all NCG = WCQ*C column groups of the pass
// (a column group = the hi and lo terms of 8 rows = the 16 columns of one MFMA).  The reduction dimension runs in
// stages of SK k tiles.  A stage's weight tiles (TN x SK KiB) and activation fragments (SK x NCG KiB, in B-operand
// order: a small kernel rewrites the pass's activation planes that way first, once per product, so that staging reads
// whole cache lines instead of gathering 64-byte pieces of 16 rows) are fetched by all waves together, every byte once,
// into registers and written to one of two LDS slabs
// while the other slab is being consumed: one barrier per stage.  Registers, not LDS, are the prefetch buffer: the
// weights (HBM latency) are requested DW = 4 stages ahead, the activations (L2) DX = 2 stages ahead, in rotating
// register sets, so that about 48 KiB of weights per compute unit are in flight.  A wave is (ws, wc, wk): strips
// ws*4 .. +3, column groups wc, wc + WCQ, ... (C of them: 4 x C accumulator tiles, every weight fragment read from
// LDS feeds C MFMAs and every activation fragment 4), k tiles wk, wk + KP, ... of each stage.  The KP waves that share
// an accumulator tile add their sums through LDS in wave order.
// A product with few strips also cuts the reduction dimension over workgroups (grid.y): partial sums go to global
// memory with device-scope write-through stores, and the workgroup that arrives last for a tile adds them in range
// order and runs the epilogues (deterministic; the same protocol as the skinny kernels).
#include "common.h"
#include "gemm.h"
#include "gemm_device.h"

#include <atomic>
#include <type_traits>

namespace mtad {

namespace {

constexpr int TW = 8;  // waves per workgroup

template <int WS, int WCQ, int KP, int C, int SK>
struct TiledShape {
  static_assert(WS * WCQ * KP == TW, "eight waves");
  static_assert(SK == KP, "every wave takes one k tile per stage");
  static constexpr int TN = 4 * WS;          // strips per workgroup
  static constexpr int NCG = WCQ * C;        // column groups per pass
  static constexpr int KW = SK / KP;         // k tiles per wave and stage
  static constexpr int FR = SK * NCG;        // activation fragments per stage
  static constexpr int FPW = FR / TW;        // staged per wave
  static_assert(FR % TW == 0, "the waves share the staging evenly");
  static constexpr int WF = TN * SK;         // weight tiles per stage
  static constexpr int WPW = WF / TW;        // staged per wave
  static_assert(WF % TW == 0, "the waves share the staging evenly");
  static constexpr int SLAB = WF + FR;       // fragments (KiB) per slab: weight tiles, then activation fragments
  static constexpr int OWN = TW / KP;        // waves that end up holding sums
  static constexpr int SLAB_KIB = 2 * SLAB;
  static constexpr int RED_KIB = KP > 1 ? OWN * 4 * C : 0;
  static constexpr int LDS_BYTES = (SLAB_KIB > RED_KIB ? SLAB_KIB : RED_KIB) * 1024;
};

// Activation planes [2][R][K] -> fragments [k tile][column group][64 lanes][8]: lane l of fragment (kt, cg) holds row
// cg*8 + l%8 of plane (l/8)%2, k = kt*32 + (l/16)*8 .. +8 (the B operand of one MFMA); rows beyond the pass are zeros.
// One wave per fragment.
__global__ __launch_bounds__(256) void xfrag_kernel(const bf16_t* __restrict__ X, bf16_t* __restrict__ out, int R, int K, int row0, int rows_here,
                                                    int ncg) {
  const int lane = threadIdx.x & 63;
  const int64_t f = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int KT = K >> 5;
  if (f >= (int64_t)KT * ncg) return;
  const int kt = (int)(f / ncg), cg = (int)(f % ncg);
  const int row = cg * 8 + (lane & 7), plane = (lane >> 3) & 1;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (row < rows_here) v = *(const uint4*)(X + ((size_t)plane * R + row0 + row) * K + kt * 32 + (lane >> 4) * 8);
  *(uint4*)(out + (f * 64 + lane) * 8) = v;
}

template <int WS, int WCQ, int KP, int C, int SK, int EPI>
__global__ __launch_bounds__(TW * 64) void gemm_bf16_tiled_kernel(GemmArgs a) {
  using Sh = TiledShape<WS, WCQ, KP, C, SK>;
  constexpr int TN = Sh::TN, NCG = Sh::NCG, FR = Sh::FR, FPW = Sh::FPW, WF = Sh::WF, WPW = Sh::WPW, SLAB = Sh::SLAB, OWN = Sh::OWN;
  // stages ahead the weights / the activations are requested = register sets of each (powers of two; about 32 and 48
  // registers): the weights come from HBM and need the longer flight
  constexpr int DW0 = 8 / (WPW * SK), DW = DW0 >= 8 ? 8 : (DW0 >= 4 ? 4 : 2);
  constexpr int DX0 = 12 / (FPW * SK), DX = DX0 >= 4 ? 4 : 2;
  constexpr int CYC = DW > DX ? DW : DX;  // stages after which both rotations and the slab parity repeat
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  uintx4* const slab = reinterpret_cast<uintx4*>(lds_raw);  // [2][SLAB][64]
  __shared__ float inv_s[NCG * 8];
  __shared__ int last_s;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wk = wave % KP, wc = (wave / KP) % WCQ, ws = wave / (KP * WCQ);
  const int K = a.K, KT_all = K >> 5, NT = a.N >> 4;
  const int R = a.R, row0 = a.row0;
  const int rows_here = min(NCG * 8, R - row0);
  const int ncg_here = (rows_here + 7) >> 3;
  const int tile = blockIdx.x, nt0 = tile * TN + ws * 4;
  const int KS = gridDim.y, ks = blockIdx.y;
  const int stages_all = (KT_all + SK - 1) / SK;
  const int per = (stages_all + KS - 1) / KS;
  const int st_lo = ks * per, n_st = max(0, min(stages_all, st_lo + per) - st_lo);

  // staging roles.  Activation fragment f = i*TW + wave of a stage is (column group f / SK, k tile f % SK); weight tile
  // g = i*TW + wave of a stage is (strip g / SK, k tile g % SK).  Both land in LDS in operand order.
  // The stage loop is free of branches (the compiler's wait counts stay exact, so the requests really stay in flight
  // across stages): every load is unconditional from an address clamped into the operand.  Requests for stages beyond the range and k tiles beyond K read the
  // last valid ones (finite activations), and such weights are replaced by zeros on their way to LDS.
  const unsigned voff = (unsigned)lane * 16u;
  static_assert(TW % SK == 0, "a wave stages the same k tile of every fragment it takes");
  const int xkk = wave % SK;  // (i*TW + wave) % SK for every i
  // activations in operand-fragment order: the pass's own buffer when its producer wrote that order (a.ncg row groups per
  // k tile, this launch's first one at row0 / 8), else the scratch copy xfrag_kernel made of this launch's rows (NCG per
  // k tile).  Column groups beyond the pass's last one read that last one: their columns are never stored.
  const char* const XF = a.ncg ? (const char*)a.X + (size_t)(row0 >> 3) * 1024 : (const char*)a.xfrag;
  const int xncg = a.ncg ? a.ncg : NCG;
  const int cg_last = a.ncg ? a.ncg - (row0 >> 3) - 1 : NCG - 1;
  unsigned xsrc[FPW];
#pragma unroll
  for (int i = 0; i < FPW; ++i) xsrc[i] = (unsigned)min((i * TW + wave) / SK, cg_last) * 1024u + voff;
  auto load_x = [&](uintx4 (&xr)[FPW], int t) {  // stage t of this workgroup's range
    const int kt = min((st_lo + t) * SK + xkk, KT_all - 1);
    const char* base = XF + (size_t)kt * xncg * 1024;
#pragma unroll
    for (int i = 0; i < FPW; ++i) xr[i] = *(const uintx4*)(base + xsrc[i]);
  };
  const char* const W = (const char*)a.W;
  auto load_w = [&](Frag (&wr)[WPW], int t) {
    const int st = st_lo + t;
#pragma unroll
    for (int i = 0; i < WPW; ++i) {
      const int g = i * TW + wave, nt = tile * TN + g / SK, kt = st * SK + g % SK;
      wr[i].n = __builtin_nontemporal_load((const uintx4*)(W + ((((size_t)min(nt, NT - 1)) * KT_all + min(kt, KT_all - 1)) << 10) + voff));
    }
  };
  // stage t's registers go to slab buf; weight tiles that do not exist become zeros here, where the value is first used
  // (a mask at the load would make the wave wait for it at once)
  auto store_stage = [&](const Frag (&wr)[WPW], const uintx4 (&xr)[FPW], int t, int buf) {
    const int st = st_lo + t;
#pragma unroll
    for (int i = 0; i < WPW; ++i) {
      const int g = i * TW + wave, nt = tile * TN + g / SK, kt = st * SK + g % SK;
      const unsigned keep = (t < n_st && nt < NT && kt < KT_all) ? ~0u : 0u;
      slab[(buf * SLAB + i * TW + wave) * 64 + lane] = uintx4{wr[i].n[0] & keep, wr[i].n[1] & keep, wr[i].n[2] & keep, wr[i].n[3] & keep};
    }
#pragma unroll
    for (int i = 0; i < FPW; ++i) slab[(buf * SLAB + WF + i * TW + wave) * 64 + lane] = xr[i];
  };

  floatx4 acc[4][C];
#pragma unroll
  for (int si = 0; si < 4; ++si)
#pragma unroll
    for (int j = 0; j < C; ++j) acc[si][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  const int cv = max(0, min(C, (ncg_here - wc + WCQ - 1) / WCQ));  // column groups of this wave that hold rows
  // The two waves of a SIMD (waves w and w + 4) work half a stage apart: a stage is a memory phase (this stage's operand
  // fragments LDS -> registers, requests for later stages, the next stage's registers -> LDS) and a compute phase (the
  // MFMAs, operands all in registers), each ended by a workgroup barrier; waves 4..7 pass one extra barrier at the start
  // and waves 0..3 one at the end, so that on every SIMD one wave computes while the other moves data.  Slab (t+1)&1 is
  // written in the memory phases of stage t (two consecutive barrier intervals) and read in those of stage t+1 (the two
  // after), and was last read two intervals before the first write.
  Frag fw[4], fb[C];
  auto fetch = [&](int buf) {
#pragma unroll
    for (int si = 0; si < 4; ++si) fw[si].n = slab[(buf * SLAB + (ws * 4 + si) * SK + wk) * 64 + lane];
#pragma unroll
    for (int j = 0; j < C; ++j) fb[j].n = slab[(buf * SLAB + WF + (j * WCQ + wc) * SK + wk) * 64 + lane];
  };
  auto compute = [&]() {
#pragma unroll
    for (int j = 0; j < C; ++j)
#pragma unroll
      for (int si = 0; si < 4; ++si) acc[si][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[si].v, fb[j].v, acc[si][j], 0, 0, 0);
  };

  Frag wr[DW][WPW];
  uintx4 xr[DX][FPW];
  // stage 0 goes to slab 0; the next stages' requests are issued, activations before weights within a stage (loads
  // complete in issue order: a wait for stage t's activations must not include later weight requests)
  load_x(xr[0], 0);
  load_w(wr[0], 0);
#pragma unroll
  for (int u = 1; u < CYC; ++u) {
    if (u < DX) load_x(xr[u], u);
    if (u < DW) load_w(wr[u], u);
  }
  store_stage(wr[0], xr[0], 0, 0);
  __syncthreads();
  const bool late = wave >= TW / 2;
  if (late) __syncthreads();
  auto stage = [&](auto U, int t) {  // U: position in the register rotations, a compile-time constant
    constexpr int u = decltype(U)::value;
    fetch(u & 1);
    load_x(xr[u % DX], t + DX);  // these registers went to LDS during the previous stage
    load_w(wr[u % DW], t + DW);
    store_stage(wr[(u + 1) % DW], xr[(u + 1) % DX], t + 1, (u + 1) & 1);
    __builtin_amdgcn_sched_barrier(0);  // the MFMAs below use registers only: without this they drift above the barrier
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    compute();
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
  };
  // whole trips of the rotation, then the first stages of one more trip
  static_assert(CYC == 2 || CYC == 4 || CYC == 8, "the stages below are written out for these");
  int t0 = 0;
  for (; t0 + CYC <= n_st; t0 += CYC) {
    stage(std::integral_constant<int, 0>{}, t0);
    stage(std::integral_constant<int, 1>{}, t0 + 1);
    if constexpr (CYC > 2) {
      stage(std::integral_constant<int, 2>{}, t0 + 2);
      stage(std::integral_constant<int, 3>{}, t0 + 3);
    }
    if constexpr (CYC > 4) {
      stage(std::integral_constant<int, 4>{}, t0 + 4);
      stage(std::integral_constant<int, 5>{}, t0 + 5);
      stage(std::integral_constant<int, 6>{}, t0 + 6);
      stage(std::integral_constant<int, 7>{}, t0 + 7);
    }
  }
  const int rem = n_st - t0;  // uniform over the workgroup
  if (rem > 0) stage(std::integral_constant<int, 0>{}, t0);
  if constexpr (CYC > 2) {
    if (rem > 1) stage(std::integral_constant<int, 1>{}, t0 + 1);
    if (rem > 2) stage(std::integral_constant<int, 2>{}, t0 + 2);
  }
  if constexpr (CYC > 4) {
    if (rem > 3) stage(std::integral_constant<int, 3>{}, t0 + 3);
    if (rem > 4) stage(std::integral_constant<int, 4>{}, t0 + 4);
    if (rem > 5) stage(std::integral_constant<int, 5>{}, t0 + 5);
    if (rem > 6) stage(std::integral_constant<int, 6>{}, t0 + 6);
  }
  if (!late) __syncthreads();

  gemm_row_factors<false, 8>(a, inv_s, rows_here, wave, lane, TW);
  if constexpr (KP > 1) {  // the waves of one accumulator tile add their sums in wave order
    floatx4* const red = reinterpret_cast<floatx4*>(lds_raw);  // [OWN][4*C][64], over the slabs (all consumed)
    const int own = ws * WCQ + wc;
#pragma unroll
    for (int p = 1; p < KP; ++p) {
      if (p > 1) __syncthreads();
      if (wk == p) {
#pragma unroll
        for (int si = 0; si < 4; ++si)
#pragma unroll
          for (int j = 0; j < C; ++j) red[((own * 4 + si) * C + j) * 64 + lane] = acc[si][j];
      }
      __syncthreads();
      if (wk == 0) {
#pragma unroll
        for (int si = 0; si < 4; ++si)
#pragma unroll
          for (int j = 0; j < C; ++j) {
            const floatx4 t2 = red[((own * 4 + si) * C + j) * 64 + lane];
            acc[si][j][0] += t2[0]; acc[si][j][1] += t2[1]; acc[si][j][2] += t2[2]; acc[si][j][3] += t2[3];
          }
      }
    }
  }
  __syncthreads();  // the row factors are in place
  const bool owner = wk == 0;
  const int own = ws * WCQ + wc;
  // The epilogues of a tile's 4 strips x C column groups are shared between its KP waves: strip si goes to wave si % KP.
  // One wave running all of them queued up to 24 chains of dependent loads (rotary table, cache slots, residual rows)
  // behind each other while its partner waves had already left.
  if (KS == 1) {
    if constexpr (KP > 1) {
      floatx4* const red = reinterpret_cast<floatx4*>(lds_raw);  // free again: the sums were read before the barrier above
      if (owner) {
#pragma unroll
        for (int si = 0; si < 4; ++si)
          if (si % KP != 0) {
#pragma unroll
            for (int j = 0; j < C; ++j) red[((own * 4 + si) * C + j) * 64 + lane] = acc[si][j];
          }
      }
      __syncthreads();
      if (!owner) {
#pragma unroll
        for (int si = 0; si < 4; ++si)
          if (si % KP == wk) {
#pragma unroll
            for (int j = 0; j < C; ++j) acc[si][j] = red[((own * 4 + si) * C + j) * 64 + lane];
          }
      }
    }
#pragma unroll
    for (int si = 0; si < 4; ++si)
      if (si % KP == wk && nt0 + si < NT) {
        if constexpr (EPI == EPI_RESID) {  // the strip's residual inputs for all column groups first: one latency, not C
          float4 ph[C], pg[C];
#pragma unroll
          for (int j = 0; j < C; ++j) gemm_resid_inputs(a, nt0 + si, j * WCQ + wc, j < cv ? rows_here : 0, lane, ph[j], pg[j]);
#pragma unroll
          for (int j = 0; j < C; ++j)
            if (j < cv) gemm_finish_sum<EPI, false, true>(a, nt0 + si, j * WCQ + wc, acc[si][j], inv_s, rows_here, lane, ph[j], pg[j]);
        } else {
#pragma unroll
          for (int j = 0; j < C; ++j)
            if (j < cv) gemm_finish_sum<EPI>(a, nt0 + si, j * WCQ + wc, acc[si][j], inv_s, rows_here, lane);
        }
      }
    return;
  }
  // partial sums of (tile, range ks, owner wave, strip, column group): 64 lanes x 4 floats
  float* const mine = a.part + ((((size_t)tile * KS) * OWN + own) * (4 * C)) * 256 + (size_t)lane * 4;
  constexpr size_t range_stride = (size_t)OWN * 4 * C * 256;
  if (owner) {
#pragma unroll
    for (int si = 0; si < 4; ++si)
#pragma unroll
      for (int j = 0; j < C; ++j)
        if (j < cv) {
          float* p = mine + (size_t)ks * range_stride + (size_t)(si * C + j) * 256;
          st8<true>(p, make_uint2(__float_as_uint(acc[si][j][0]), __float_as_uint(acc[si][j][1])));
          st8<true>(p + 2, make_uint2(__float_as_uint(acc[si][j][2]), __float_as_uint(acc[si][j][3])));
        }
  }
  __builtin_amdgcn_s_waitcnt(0);  // the stores have been acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    const int prev = __hip_atomic_fetch_add(a.counters + tile, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    last_s = (prev == KS - 1);
    if (last_s) __hip_atomic_store(a.counters + tile, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // clean for the next launch
  }
  __syncthreads();
  if (!last_s) return;
#pragma unroll
  for (int si = 0; si < 4; ++si)
    if (si % KP == wk && nt0 + si < NT) {  // the tile's KP waves share its strips
      float4 ph[C], pg[C];
      if constexpr (EPI == EPI_RESID) {  // the residual inputs of all column groups are requested with the partial sums
#pragma unroll
        for (int j = 0; j < C; ++j) gemm_resid_inputs(a, nt0 + si, j * WCQ + wc, j < cv ? rows_here : 0, lane, ph[j], pg[j]);
      }
#pragma unroll
      for (int j = 0; j < C; ++j)
        if (j < cv) {
          const float* p = mine + (size_t)(si * C + j) * 256;
          floatx4 sum = floatx4{0.f, 0.f, 0.f, 0.f};
          for (int k2 = 0; k2 < KS; ++k2) {
            const uint4 v = ld16<true>(p + (size_t)k2 * range_stride);
            sum[0] += __uint_as_float(v.x); sum[1] += __uint_as_float(v.y); sum[2] += __uint_as_float(v.z); sum[3] += __uint_as_float(v.w);
          }
          if constexpr (EPI == EPI_RESID) gemm_finish_sum<EPI, false, true>(a, nt0 + si, j * WCQ + wc, sum, inv_s, rows_here, lane, ph[j], pg[j]);
          else gemm_finish_sum<EPI>(a, nt0 + si, j * WCQ + wc, sum, inv_s, rows_here, lane);
        }
    }
}

int device_cus() {
  static const int n_cus = [] {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
    return cus > 0 ? cus : 256;
  }();
  return n_cus;
}

constexpr int KS_MAX = 8;        // most ranges of the reduction dimension
constexpr int MIN_STAGES = 8;    // fewest stages a range is worth

// strips per workgroup: 8 when that still gives at least half the compute units a workgroup (activations are
// re-staged once per workgroup, so wider tiles halve that traffic), else 4
int tiled_tn(int NT) { return (NT + 7) / 8 * 2 >= device_cus() ? 8 : 4; }
// ranges of the reduction dimension for a product with `tiles` workgroups per range and `stages` stages
int tiled_ks(int tiles, int stages) {
  int ks = device_cus() / tiles;
  if (ks > KS_MAX) ks = KS_MAX;
  if (ks > stages / MIN_STAGES) ks = stages / MIN_STAGES;
  return ks < 1 ? 1 : ks;
}

// LDS of one compute unit (the most a workgroup can be given); 160 KiB on gfx950 if the query fails
size_t device_lds_bytes() {
  static const size_t n = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess) v = 0;
    return v > 0 ? (size_t)v : (size_t)160 * 1024;
  }();
  return n;
}

template <int WS, int WCQ, int KP, int C, int SK, int EPI>
hipError_t run_shape(const GemmArgs& a, hipStream_t s) {
  using Sh = TiledShape<WS, WCQ, KP, C, SK>;
  static_assert(Sh::LDS_BYTES <= 160 * 1024, "more LDS than a gfx950 compute unit has");
  auto kern = gemm_bf16_tiled_kernel<WS, WCQ, KP, C, SK, EPI>;
  if ((size_t)Sh::LDS_BYTES + 1024 > device_lds_bytes()) return hipErrorInvalidValue;  // + the kernel's static arrays
  // more than 64 KiB of dynamic LDS needs the attribute; a success is remembered, a failure is reported and tried again
  static std::atomic<bool> attr_set{false};
  if (!attr_set.load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, Sh::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set.store(true, std::memory_order_release);
  }
  const int NT = a.N >> 4, tiles = (NT + Sh::TN - 1) / Sh::TN;
  if (!a.ncg) {  // this launch's activations in fragment order (a pass that already holds them that way needs no copy)
    const int64_t frags = (int64_t)(a.K >> 5) * Sh::NCG;
    if ((size_t)frags * 512 > a.xfrag_elems) return hipErrorInvalidValue;
    const int rows = a.R - a.row0 < Sh::NCG * 8 ? a.R - a.row0 : Sh::NCG * 8;
    hipLaunchKernelGGL(xfrag_kernel, dim3((unsigned)((frags + 3) / 4)), dim3(256), 0, s, a.X, a.xfrag, a.R, a.K, a.row0, rows, Sh::NCG);
  }
  int ks = 1;
  if (a.part && a.counters) ks = tiled_ks(tiles, ((a.K >> 5) + SK - 1) / SK);
  // the exchange of a cut reduction must fit what the caller offers: (tile, range, owner wave, strip, column group) x 256 floats
  // and one counter per tile; a product that does not fit runs uncut
  if (ks > 1 && ((size_t)tiles * ks * Sh::OWN * 4 * C * 256 > a.part_floats || tiles > a.counters_n)) ks = 1;
  hipLaunchKernelGGL(kern, dim3(tiles, ks), dim3(TW * 64), Sh::LDS_BYTES, s, a);
  return hipGetLastError();
}

template <int EPI>
hipError_t run_tiled(GemmArgs a, hipStream_t s) {
  // passes of at most 192 rows, of equal size
  const int n_pass = (a.R + 191) / 192;
  const int rows_pass = (((a.R + n_pass - 1) / n_pass) + 7) / 8 * 8;
  const bool wide = tiled_tn(a.N >> 4) == 8;
  for (int r0 = 0; r0 < a.R; r0 += rows_pass) {
    a.row0 = r0;
    const int rows = a.R - r0 < rows_pass ? a.R - r0 : rows_pass;
    hipError_t e;
    if (rows <= 32) e = run_shape<2, 1, 4, 4, 4, EPI>(a, s);
    else if (rows <= 64) e = wide ? run_shape<2, 2, 2, 4, 2, EPI>(a, s) : run_shape<1, 2, 4, 4, 4, EPI>(a, s);
    else if (rows <= 128) e = wide ? run_shape<2, 4, 1, 4, 1, EPI>(a, s) : run_shape<1, 4, 2, 4, 2, EPI>(a, s);
    else e = wide ? run_shape<2, 4, 1, 6, 1, EPI>(a, s) : run_shape<1, 4, 2, 6, 2, EPI>(a, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace


size_t gemm_tiled_xfrag_elems(int R, int K) { (void)R; return (size_t)(K >> 5) * 24 * 512; }  // up to 24 column groups per pass

bool gemm_tiled_wide(int N) { return tiled_tn(N >> 4) == 8; }

// floats of workspace the k split of a product with N outputs may use (0: never split): the larger of the needs of the
// two tile widths the shapes above use (4 or 8 strips per workgroup; passes of 32 rows or fewer always take 8), each
// with the most ranges tiled_ks can return for it and all 24 column groups
size_t gemm_tiled_split_floats(int N) {
  const int NT = N >> 4;
  if (NT < 1) return 0;
  size_t need = 0;
  for (int TN : {4, 8}) {
    const int tiles = (NT + TN - 1) / TN;
    int ks = device_cus() / tiles;
    if (ks > KS_MAX) ks = KS_MAX;
    if (ks < 2) continue;
    const size_t n = (size_t)tiles * ks * TN * 24 * 256;  // TN strips x up to 24 column groups x 64 lanes x 4 floats per range
    if (n > need) need = n;
  }
  return need;
}
int gemm_tiled_split_counters(int N) { return gemm_tiled_split_floats(N) ? ((N >> 4) + 3) / 4 : 0; }

hipError_t launch_gemm_bf16_tiled(const GemmArgs& a, int epi, hipStream_t s) {
  switch (epi) {
    case EPI_STORE: return run_tiled<EPI_STORE>(a, s);
    case EPI_RESID: return run_tiled<EPI_RESID>(a, s);
    case EPI_SWIGLU: return run_tiled<EPI_SWIGLU>(a, s);
    case EPI_QKV: return run_tiled<EPI_QKV>(a, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace mtad
