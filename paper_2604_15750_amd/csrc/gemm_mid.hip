// Mid-size GEMM of a bf16 model (65 .. 160 rows: a block plus its look-ahead window, a few packed blocks; fewer rows where its wide
// column groups pay, see choose_kernel in gemm_bf16.hip):
// Y[M,N] = X[M,K] * W[N,K]^T, fp32 accumulation, epilogue fused.
//
// At these row counts W is still the larger operand, but every column group re-reads X, so the groups
// have to be wide.  A workgroup of four wavefronts owns ALL the rows (MT row tiles) of CT adjacent
// column tiles (32 .. 128 columns) and a range of K; its wavefronts split that range among themselves,
// and each multiplies its k-tiles of the CT W fragments against all MT X fragments (CT MT products
// per CT + MT fragments fetched), everything in registers:
//   * W goes HBM -> registers, the step in use and the two to four after it, as many as the registers hold (a step is one
//     k-tile, two for the narrowest groups; a wavefront keeps 8 .. 24 KiB of W in flight, a workgroup 32 .. 96 KiB: what it takes to keep HBM busy with 128 .. 256 workgroups);
//     X goes L2 -> registers one step ahead, issued BEFORE the W loads of the same step, so that
//     waiting for it never waits for younger W loads (the memory counter retires in order);
//   * no barrier, no LDS inside the loop: a wavefront never waits for another.  (X through
//     direct-to-LDS loads would save a third of the registers, but the compiler then no longer counts
//     the register loads beside them and waits for every load in flight once per trip.)
//   * at the end the four partial accumulators meet in LDS (32 fragments per round), are added in
//     wavefront order, and each wavefront finishes every fourth output fragment.
// When the column groups are fewer than the compute units, K is split across workgroups as well:
// partial tiles go to an fp32 workspace written through to device scope, and the workgroup that takes
// the last ticket adds them in split order (the protocol of gemm_tiled.hip; a wavefront fetches the
// same split of all its output fragments in a single trip to memory).
#include "gemm_epilogue.h"
#include <type_traits>

namespace {

constexpr int TPB = 256, NWV = 4;
constexpr int MID_STEPS_MAX_MT = 4;  // row tiles up to which a launch may read the step-major copy of W
#ifndef MID_WD_MAX
#define MID_WD_MAX 4
#endif

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int SC1 = 16;  // cache-policy bit of the raw-buffer builtins: device scope

__device__ inline __amdgpu_buffer_rsrc_t part_rsrc(const float* base) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, 0x7fffffff, 0x00020000);
}

template <int MT, int CT>
struct MidShape {
  static constexpr int KB = CT <= 3 ? 2 : 1;  // k-tiles per step: narrow column groups take two, so that a step's loads are still 6 KiB of W
  // steps of W per register ring (one in use, the others in flight): as many as fit beside the accumulators and two steps of
  // X in about 370 registers, and whose loads the memory counter can count; 3 .. MID_WD_MAX
  static constexpr int WD_FIT = (92 - CT * MT - 2 * KB * MT) / (KB * CT);
  static constexpr int WD_CNT = (63 / KB - MT) / CT + 1;
  static constexpr int WD_ = WD_FIT < WD_CNT ? WD_FIT : WD_CNT;
  static constexpr int WD = WD_ < 3 ? 3 : WD_ > MID_WD_MAX ? MID_WD_MAX : WD_;
  static constexpr int TRIP = WD % 2 ? 2 * WD : WD;  // steps after which both the W ring and the two X sets are back where they started
  static constexpr int F = CT * MT;                 // output fragments of a workgroup
  static constexpr int FW = (F + NWV - 1) / NWV;    // ... finished by one wavefront
  static constexpr int FR = F < 32 ? (F + 3) / 4 * 4 : 32;  // fragments per reduction round (a multiple of 4: fragment f stays with wavefront f % 4)
  static constexpr int ROUNDS = (F + FR - 1) / FR;
  static constexpr int BODY = NWV * FR * 1024;
  static constexpr int LDS_BYTES = BODY + MT * 16 * 4 + CT * MT * 16 * 4;  // + 1/rms of the rows + every column tile's sum of squares per row
};

// grid.x = groups * splits; MT >= ceil(M / 16), and X has MT row tiles (the activation buffers are padded to 16 rows).
// STEPS: W is read from the step-major copy (e.w_steps) instead of wt.
template <int MT, int CT, int PR, int EPI, bool STEPS = false>
__global__ __launch_bounds__(TPB) void gemm_mid_kernel(const op8* __restrict__ xt, const op8* __restrict__ wt, int M, int N, int K,
                                                       int kt_per_split, int splits, GemmEpi e) {
  typedef MidShape<MT, CT> SH;
  constexpr int F = SH::F, FW = SH::FW, FR = SH::FR, ROUNDS = SH::ROUNDS;
  constexpr int KB = SH::KB, WD = SH::WD, TRIP = SH::TRIP;
  static_assert(KB * (MT + (WD - 1) * CT) < 64, "the loads in flight must fit the memory counter");
  extern __shared__ __align__(16) unsigned char lds[];
  __shared__ int s_last;
  float* s_rinv = (float*)(lds + SH::BODY);  // [MT * 16]
  float* s_ssq = s_rinv + MT * 16;           // [CT][MT * 16]

  const int group = blockIdx.x / splits, split = blockIdx.x - group * splits, groups = gridDim.x / splits;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int KT = K >> 5, NT = N >> 4;
  const int nt0 = group * CT;
  const int tb = split * kt_per_split, te = min(KT, tb + kt_per_split);
  const int per = (te - tb + NWV - 1) / NWV;
  const int t0 = tb + wave * per, t1 = min(te, t0 + per);  // this wavefront's k-tiles (possibly none)

  // fragment (nt0 + r, k-tile t) = wptr[r][(t - tsub) * wstep]; column tiles past the end repeat the last one.  With the step-major
  // copy (no K split, whole groups, KT a multiple of 4: the host checks) the wavefront's step s is at wptr[r][s * wstep]
  static_assert(!STEPS || MT <= MID_STEPS_MAX_MT, "the larger variants have no register to spare for a run-time stride");
  constexpr bool steps = STEPS;
  const size_t wstep = steps ? (size_t)groups * NWV * CT * 64 : (PR == 2 ? 128 : 64);
  const int tsub = steps ? t0 : 0;
  const op8* wptr[CT];
#pragma unroll
  for (int r = 0; r < CT; ++r) {
    const int nt = min(nt0 + r, NT - 1);
    wptr[r] = steps ? (const op8*)e.w_steps + ((size_t)(group * NWV + wave) * CT + r) * 64 + lane
                    : PR == 2 ? wt + ((size_t)(nt >> 1) * KT * 2 + (nt & 1)) * 64 + lane : wt + (size_t)nt * KT * 64 + lane;
  }
  const op8* xptr = xt + lane;  // fragment (j, t) = xptr[(j * KT + t) * 64]
  // In the last row tile, lanes whose row does not exist re-read row 0 of their k-group instead of fetching lines of their
  // own (a fragment's 128-byte lines hold 8 rows each: a block of 8 rows reads half of them); what they get is never stored.
  const op8* xptr_last = xt + ((MT - 1) * 16 + (lane & 15) < M ? lane : (lane & ~15));

  f32x4 acc[CT][MT];
#pragma unroll
  for (int r = 0; r < CT; ++r)
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  op8 w[WD][KB][CT], x[2][KB][MT];
  const int nsteps = (t1 - t0 + KB - 1) / KB;
  const op8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  // step st of the wavefront (its k-tiles clamped to the wavefront's last one) -> register set `slot`
  auto load_x = [&](const int slot, int st) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < KB; ++i) {
      const int tc = min(t0 + st * KB + i, t1 - 1);
#pragma unroll
      for (int j = 0; j < MT; ++j) x[slot][i][j] = (j == MT - 1 ? xptr_last : xptr)[((size_t)j * KT + tc) * 64];
    }
  };
  auto load_w = [&](const int slot, int st) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < KB; ++i) {
      const int tc = min(t0 + st * KB + i, t1 - 1);
#pragma unroll
      for (int r = 0; r < CT; ++r) w[slot][i][r] = wptr[r][(size_t)(tc - tsub) * wstep];
    }
  };
  auto compute = [&](const int ws, const int xs, int st) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < KB; ++i) {
      const bool past = KB > 1 && t0 + st * KB + i >= t1;  // the surplus k-tile of a ragged last step multiplies zeros
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        const op8 xv = past ? zero8 : x[xs][i][j];
#pragma unroll
        for (int r = 0; r < CT; ++r) acc[r][j] = mfma_op(w[ws][i][r], xv, acc[r][j]);
      }
    }
  };
  // step S of a trip: X of the next step first, then W of the step WD - 1 ahead, so that the wait for this step's operands
  // (the oldest loads) leaves W WD - 1 steps deep and X one step deep in flight; the scheduling barriers keep the compiler
  // from sinking the loads down to their uses (which it does under register pressure, undoing the prefetch)
  auto step = [&](auto Sc, int st) __attribute__((always_inline)) {
    constexpr int S = decltype(Sc)::value;
    load_x((S + 1) & 1, st + 1);
    load_w((S + WD - 1) % WD, st + WD - 1);
    __builtin_amdgcn_sched_barrier(0);
    compute(S % WD, S & 1, st);
    __builtin_amdgcn_sched_barrier(0);
  };
  // (every lambda here is forced inline: left to its own judgement the compiler keeps the largest variants' steps as
  // functions, and the operand rings, passed by reference, then live in scratch memory)
  // whole trips: TRIP steps in a row; the steps left over: nested, not skippable one by one (a path around a step's loads is
  // one the compiler's count of outstanding loads cannot follow: it would wait for all of them)
  auto trip = [&](auto self, auto Ic, int st) __attribute__((always_inline)) {
    constexpr int I = decltype(Ic)::value;
    if constexpr (I < TRIP) {
      step(Ic, st + I);
      self(self, std::integral_constant<int, I + 1>{}, st);
    }
  };
  auto rest = [&](auto self, auto Ic, int st) __attribute__((always_inline)) {
    constexpr int I = decltype(Ic)::value;
    if constexpr (I < TRIP - 1) {
      if (st + I < nsteps) {
        step(Ic, st + I);
        self(self, std::integral_constant<int, I + 1>{}, st);
      }
    }
  };
  if (nsteps > 0) {
    load_x(0, 0);
#pragma unroll
    for (int i = 0; i < WD - 1; ++i) load_w(i, i);
  }
  // 1/rms of the input rows, needed only by the epilogue: fetched while the first k-tiles are in flight (published by the
  // barriers of the reduction)
  if (EPI != EPI_RESID) block_rinv<TPB>(e.rs, 0, min(M, MT * 16), s_rinv);
  // ... and so is what the epilogue of the fragment this wavefront finishes first (fragment `wave`) reads from memory, in the
  // variants of narrow passes, which are short enough for that round trip to show
  EpiAhead ahead = epi_none();
  if constexpr (MT <= 2 && (EPI == EPI_RESID || EPI == EPI_QKV)) {
    if (splits == 1 && wave < F && nt0 + wave / MT < NT)
      ahead = epi_ahead<EPI>(e, M, N, (wave % MT) * 16 + (lane & 15), (nt0 + wave / MT) * 16, lane >> 4);
  }
  if (nsteps > 0) {
    int st = 0;
    for (; st + TRIP <= nsteps; st += TRIP) trip(trip, std::integral_constant<int, 0>{}, st);
    rest(rest, std::integral_constant<int, 0>{}, st);
  }

  // ---- the four partial accumulators -> one finished (or, with a K split, one partial) value per output fragment
  const int g = lane >> 4, ml = lane & 15;
  f32x4* red = (f32x4*)lds;  // [NWV][FR][64]
  const size_t stride = (size_t)M * N;
  float* mine = e.part + split * stride;
  // fragment f = r * MT + j (column tile r, row tile j) in the accumulator layout -> its epilogue
  auto finish = [&](int f, f32x4 v) {
    const int r = f / MT, j = f - r * MT;
    const int nt = nt0 + r, m = j * 16 + ml;
    float ss = 0.f;
    if (nt < NT) ss = finish_frag<EPI>(e, M, N, m, nt * 16, g, v, EPI == EPI_RESID ? 1.f : s_rinv[m], f == wave ? ahead : epi_none());  // uniform in the wavefront
    if (EPI == EPI_RESID && g == 0) s_ssq[r * MT * 16 + m] = ss;
  };
#pragma unroll
  for (int rd = 0; rd < ROUNDS; ++rd) {
    if (rd) __syncthreads();  // the previous round has been read
#pragma unroll
    for (int i = 0; i < FR; ++i)
      if (rd * FR + i < F) red[(wave * FR + i) * 64 + lane] = acc[min(rd * FR + i, F - 1) / MT][min(rd * FR + i, F - 1) % MT];
    __syncthreads();
    for (int i = wave; i < FR && rd * FR + i < F; i += NWV) {
      const f32x4 v = ((red[i * 64 + lane] + red[(FR + i) * 64 + lane]) + red[(2 * FR + i) * 64 + lane]) + red[(3 * FR + i) * 64 + lane];
      const int f = rd * FR + i;
      if (splits == 1) {
        finish(f, v);
      } else {  // partial tile -> workspace, written through to device scope
        const int r = f / MT, j = f - r * MT;
        const int nt = nt0 + r, m = j * 16 + ml;
        if (nt < NT && m < M)
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), part_rsrc(mine), ((unsigned)m * N + nt * 16 + 4 * g) * 4u, 0, SC1);
      }
    }
  }
  if (splits > 1) {
    // Hand-off across workgroups (possibly across XCDs, whose L2s are separate): every wavefront waits until its own partial
    // stores, written through to device scope, have been acknowledged; then the workgroup takes its ticket with release order
    // at device scope, and the last arriver reads the partial tiles (device-scope loads) behind an acquire.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
      int* ticket = e.counters + group;
      const int last = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT) == splits - 1;
      if (last) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next launch
      s_last = last;
    }
    __syncthreads();
    if (!s_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    // the finished tile = the partial tiles added in split order; a wavefront fetches one split of all its fragments per trip
    f32x4 v[FW];
    unsigned off[FW];
#pragma unroll
    for (int i = 0; i < FW; ++i) {
      const int f = wave + NWV * i, r = f / MT, j = f - r * MT;
      const int nt = nt0 + r, m = j * 16 + ml;
      off[i] = (f < F && nt < NT && m < M) ? ((unsigned)m * N + nt * 16 + 4 * g) * 4u : 0u;  // fragments that do not exist re-read element 0
      v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    for (int s = 0; s < splits; s += 2) {  // two splits per trip to memory
      const int s1 = min(s + 1, splits - 1);
      u32x4 ta[FW], tb[FW];
#pragma unroll
      for (int i = 0; i < FW; ++i) ta[i] = __builtin_amdgcn_raw_buffer_load_b128(part_rsrc(e.part + s * stride), off[i], 0, SC1);
#pragma unroll
      for (int i = 0; i < FW; ++i) tb[i] = __builtin_amdgcn_raw_buffer_load_b128(part_rsrc(e.part + s1 * stride), off[i], 0, SC1);
#pragma unroll
      for (int i = 0; i < FW; ++i) v[i] += __builtin_bit_cast(f32x4, ta[i]);
      if (s + 1 < splits)
#pragma unroll
        for (int i = 0; i < FW; ++i) v[i] += __builtin_bit_cast(f32x4, tb[i]);
    }
#pragma unroll
    for (int i = 0; i < FW; ++i)
      if (wave + NWV * i < F) finish(wave + NWV * i, v[i]);
  }
  if (EPI == EPI_RESID) {  // the workgroup's share of sum h^2 per row: its column tiles in order
    __syncthreads();
    if (tid < MT * 16 && tid < M) {
      float ss = 0.f;
#pragma unroll
      for (int r = 0; r < CT; ++r) ss += s_ssq[r * MT * 16 + tid];
      e.ssq_out[(size_t)tid * groups + group] = ss;
    }
  }
}

int g_mid_wgs = 256;  // workgroups the K split of a narrow matrix aims at

struct MidPlan {
  int ct, pr, mt, groups, splits, kps;
};

// What the compute units can load through their L2s (W once, X once per column group; about 45 GB/s each, 10 .. 12 TB/s
// together) bounds these shapes before HBM does, and a K split costs a round trip of partial tiles through memory plus a
// serial tail.  Wide matrices: of the group widths 128 (to 112 rows), 96 and 48 columns, the one that fills the chip's 256
// compute units best, without a K split if it can (QKV of an 8B model: 256 groups of 48; gate/up: 256 groups of 96).
// Narrow ones (O, down; at most 256 column tiles): 64-column groups and a four-way K split when K is long (down), 32-column
// groups and a two-way split when it is short (O); all measured against their alternatives.
MidPlan mid_plan(int M, int N, int K, bool may_split) {
  MidPlan best;
  double best_fill = -1.;
  const int pr = weight_pack_rows(N), mt = (M + 15) >> 4, KT = K >> 5;
  // accumulators (4 CT MT registers) + three k-tiles of W + two of X within the register file: 128-column groups up to 112 rows
  // short K: the partial tiles of a four-way split cost more than X re-read by twice the groups; beyond 13 row tiles the
  // 32-column variant's two k-tiles of X per step no longer fit the registers
  const int narrow = (K >= 8192 && mt > 1) || mt > 13 ? 4 : 2;
  const int cts[3] = {pr == 2 ? (mt <= 7 ? 8 : 6) : narrow, pr == 2 ? 6 : narrow, pr == 2 ? (mt <= 10 ? 3 : 6) : narrow};
  for (int c = 0; c < 3; ++c) {
    MidPlan p;
    p.pr = pr; p.mt = mt; p.ct = cts[c];
    p.groups = (N + 16 * p.ct - 1) / (16 * p.ct);
    int s = pr == 2 ? 256 / p.groups : (g_mid_wgs + p.groups / 2) / p.groups;
    if (pr == 1 && mt == 1) s = 1;  // one row tile of a narrow matrix comes here only to avoid a second round of 16-column workgroups
    if (s > (pr == 2 ? 2 : 4)) s = pr == 2 ? 2 : 4;  // a short serial tail for the last arriver, and little traffic of partial tiles
    if (s > KT / 16) s = KT / 16;     // at least four k-tiles per wavefront
    if (s < 1 || !may_split) s = 1;
    p.kps = (KT + s - 1) / s;
    p.splits = (KT + p.kps - 1) / p.kps;  // no empty split
    // more groups of the widest kind than compute units (the LM head): several rounds anyway, the widest re-reads X least
    if (c == 0 && p.groups >= 256) return p;
    // otherwise, of the group widths, the one whose workgroups fill the chip's 256 compute units best; on a near tie the
    // one without a K split, then the wider
    const int wgs = p.groups * p.splits;
    const double fill = (double)wgs / ((wgs + 255) / 256 * 256) + (p.splits == 1 ? 0.01 : 0.);
    if (fill > best_fill + 0.005) { best_fill = fill; best = p; }
  }
  return best;
}

template <int MT, int CT, int PR, int EPI>
void launch_one(const op_t* xt, const op_t* wt, int M, int N, int K, const MidPlan& p, const GemmEpi& e, hipStream_t st) {
  typedef MidShape<MT, CT> SH;
  static bool configured = false;  // raise the dynamic LDS limit of this instantiation once
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)gemm_mid_kernel<MT, CT, PR, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, SH::LDS_BYTES);
    configured = true;
  }
  if constexpr (MT <= MID_STEPS_MAX_MT) {
    if (e.w_steps) {
      static bool configured_steps = false;
      if (!configured_steps) {
        (void)hipFuncSetAttribute((const void*)gemm_mid_kernel<MT, CT, PR, EPI, true>, hipFuncAttributeMaxDynamicSharedMemorySize, SH::LDS_BYTES);
        configured_steps = true;
      }
      DLM_LAUNCH((gemm_mid_kernel<MT, CT, PR, EPI, true>), p.groups * p.splits, TPB, SH::LDS_BYTES, st, (const op8*)xt, (const op8*)wt, M, N, K, p.kps, p.splits, e);
      return;
    }
  }
  DLM_LAUNCH((gemm_mid_kernel<MT, CT, PR, EPI>), p.groups * p.splits, TPB, SH::LDS_BYTES, st, (const op8*)xt, (const op8*)wt, M, N, K, p.kps, p.splits, e);
}

template <int MT, int EPI>
void launch_mt(const op_t* xt, const op_t* wt, int M, int N, int K, const MidPlan& p, const GemmEpi& e, hipStream_t st) {
  if (p.pr == 1) {
    if (p.ct == 2) { if constexpr (MT <= 13) launch_one<MT, 2, 1, EPI>(xt, wt, M, N, K, p, e, st); }
    else if constexpr (MT >= 2) launch_one<MT, 4, 1, EPI>(xt, wt, M, N, K, p, e, st);
  } else if (p.ct == 8) {
    if constexpr (MT <= 7) launch_one<MT, 8, 2, EPI>(xt, wt, M, N, K, p, e, st);
  } else if (p.ct == 3) {
    if constexpr (MT <= 10) launch_one<MT, 3, 2, EPI>(xt, wt, M, N, K, p, e, st);
  } else {
    if constexpr (MT <= 10) launch_one<MT, 6, 2, EPI>(xt, wt, M, N, K, p, e, st);
  }
}

template <int EPI>
void launch_epi(const op_t* xt, const op_t* wt, int M, int N, int K, const MidPlan& p, const GemmEpi& e, hipStream_t st) {
  switch (p.mt) {  // the dispatcher sends only row counts that have an instantiation
    case 1: launch_mt<1, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 2: launch_mt<2, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 3: launch_mt<3, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 4: launch_mt<4, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 5: launch_mt<5, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 6: launch_mt<6, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 7: launch_mt<7, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 8: launch_mt<8, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 9: launch_mt<9, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 10: launch_mt<10, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 11: launch_mt<11, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 12: launch_mt<12, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 13: launch_mt<13, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 14: launch_mt<14, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 15: launch_mt<15, EPI>(xt, wt, M, N, K, p, e, st); break;
    default: launch_mt<16, EPI>(xt, wt, M, N, K, p, e, st); break;
  }
}

}  // namespace

// one compute unit's worth of workgroups per 96-column group, no K split: the shapes the mid kernel takes even below 17 rows
bool gemm_mid_fills_chip(int M, int N, int K) {
  const MidPlan p = mid_plan(M, N, K, true);
  return p.splits == 1 && p.groups % 256 == 0;
}
int gemm_mid_splits(int M, int N, int K) { return mid_plan(M, N, K, true).splits; }
int gemm_mid_ssq_chunks(int M, int N, int K) { return mid_plan(M, N, K, true).groups; }
int gemm_mid_counters(int max_n) { return (max_n + 31) / 32; }  // 32-column groups are the narrowest
void gemm_mid_set_target(int wgs) { g_mid_wgs = wgs; }


int gemm_mid_steps_ct(int N, int K) {
  const MidPlan p = mid_plan(16, N, K, true);
  return (p.splits == 1 && N % (16 * p.ct) == 0 && (K >> 5) % NWV == 0) ? p.ct : 0;
}

void launch_gemm_mid(const op_t* xt, const op_t* wt, int M, int N, int K, const GemmEpi& e_in, hipStream_t st) {
  const MidPlan p = mid_plan(M, N, K, e_in.kind != EPI_DIRECT);  // EPI_DIRECT has no workspace
  GemmEpi e = e_in;
  // the step-major copy serves exactly the launches it was laid out for
  if (!(e.w_steps && p.mt <= MID_STEPS_MAX_MT && e.w_steps_ct == p.ct && p.splits == 1 && N % (16 * p.ct) == 0 && (K >> 5) % NWV == 0)) e.w_steps = nullptr;
  switch (e.kind) {
    case EPI_QKV: launch_epi<EPI_QKV>(xt, wt, M, N, K, p, e, st); break;
    case EPI_SWIGLU: launch_epi<EPI_SWIGLU>(xt, wt, M, N, K, p, e, st); break;
    case EPI_RESID: launch_epi<EPI_RESID>(xt, wt, M, N, K, p, e, st); break;
    default: launch_epi<EPI_SUM>(xt, wt, M, N, K, p, e, st); break;
  }
}
