// Macro-tile GEMM of a bf16 model for wide passes (M > 256 rows: batched decoding, prefill): Y[M,N] = X[M,K] * W[N,K]^T,
// fp32 accumulation, epilogue fused.
//
// Beyond a few hundred rows the GEMMs leave the weight-streaming regime and are bound by the matrix
// cores and by how often operands are re-read.  A workgroup of NW wavefronts (NW / 2 x 2) owns a tile of
// 8 NW WM rows x 32 WN columns: 256 x 256 with eight wavefronts (two per SIMD, 128 accumulator registers
// each: what a compute unit fetches per product is half of what a 128 x 256 tile needs, and that fetch rate,
// L2 / memory-side cache -> LDS, is what bounds the smaller tiles), or 192 x 256, 128 x 256 with four
// wavefronts and 192 x 192, 128 x 128 with eight where the larger tile would leave compute units idle; it walks
// K one k-tile (32) at a time (two for 128 x 128):
//   * both operands are already stored as 1 KiB matrix-core fragments (16 rows x 32 k), so a stage of
//     the pipeline is just 2 WM + 2 WN fragments copied HBM/L2 -> LDS by direct-to-LDS loads (no
//     registers, no LDS writes): 4 to 8 stages of 16 .. 32 KiB rotate through up to 128 KiB of LDS
//     (3 stages in 74 KiB where two four-wavefront workgroups share a compute unit: macro_plan);
//   * a wavefront owns WM x WN fragments of the output (fp32 accumulators, up to 256 registers), reads
//     its WM + WN operand fragments of the NEXT k-tile from LDS into a second register set while the
//     matrix cores work on the current one (WM WN products per WM + WN fragment reads); the order in
//     which products, copies and reads are issued is fixed by hand (see step);
//   * the accumulators reach the epilogue through LDS, half of a wavefront's column tiles at a time;
//   * one barrier per k-tile; the waits on the direct-to-LDS loads are counted by hand (every stage is
//     the same number of loads per wavefront; indices past the end are clamped, so the count never
//     varies), and so are the waits on the LDS reads (once per step, behind the products).
// Workgroups that share columns (and so W) get ids congruent mod 8: they run on the same XCD and find
// W in its L2 after the first reader; X is shared by every column block through the L2s and the
// memory-side cache.  The product is computed transposed (W fragment = A operand) like the other
// kernels, so the epilogues of gemm_epilogue.h apply unchanged.
#include "gemm_epilogue.h"

namespace {


typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int SC1 = 16;  // cache-policy bit of the raw-buffer builtins: device scope
__device__ inline __amdgpu_buffer_rsrc_t part_rsrc(const float* base) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, 0x7fffffff, 0x00020000);
}

#define GLOBAL_PTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define LDS_PTR(p) ((void __attribute__((address_space(3)))*)(p))

// KB: k-tiles per pipeline stage (and barrier).  A 128 x 128 tile has few products per k-tile to set against what a step
// costs besides them (barrier, copy issue, waits): when it has a compute unit to itself it is run by eight wavefronts of
// 32 x 64 outputs (two per SIMD, which hide each other's waits) and takes two k-tiles per step (four stages of 32 KiB):
// -10 % for the two k-tiles and another -10 % for the eight wavefronts at 256 .. 1024 rows of the layer matrices.  (For
// 128 x 256 the stages would be 48 KiB, three deep: measured slower than one k-tile per step, five deep.)
template <int WM, int WN, int NW = 4, bool TWO = false, int KB = 1>
struct MacroShape {
  static constexpr int TPB = NW * 64;
  static constexpr int AT = (NW / 2) * WM;         // row tiles of the workgroup
  static constexpr int AF = AT, BF = 2 * WN;       // X (row) and W (column) fragments of a k-tile
  static constexpr int NFR = AF + BF;
  static constexpr int LPT = (NFR + NW - 1) / NW;  // direct-to-LDS loads per wavefront and k-tile (surplus ones repeat the last fragment)
  static constexpr int LPS = KB * LPT;             // ... and stage
  static constexpr int STAGE = KB * NFR * 1024;
  // TWO: two workgroups share a compute unit (three stages each; see macro_plan)
  static constexpr int LDSB = TWO ? 75776 : 131072;
  static constexpr int S = LDSB / STAGE > 8 ? 8 : LDSB / STAGE;  // stages: at most 128 KiB (of the 160 KiB of a compute unit)
  static constexpr int LDS_BYTES = S * STAGE + AT * 16 * 4 * 3;      // + 1/rms of the rows, two partial sums of squares per row
};

template <int WM, int WN, int PR, int EPI, int NW = 4, bool TWO = false, int KB = 1>
__global__ __launch_bounds__(NW * 64, TWO ? 2 : 1) void gemm_macro_kernel(const op8* __restrict__ xt, const op8* __restrict__ wt, int M, int N,
                                                                          int K, int nblocks, int mblocks, int splits, int kt_per_split, GemmEpi e) {
  typedef MacroShape<WM, WN, NW, TWO, KB> SH;
  constexpr int TPB = SH::TPB, AT = SH::AT, AF = SH::AF, BF = SH::BF, NFR = SH::NFR, LPT = SH::LPT, LPS = SH::LPS, STAGE = SH::STAGE, S = SH::S;
  static_assert(S >= 3 && (S - 2) * LPS < 64, "pipeline shape");
  extern __shared__ __align__(16) unsigned char lds[];
  float* s_rinv = (float*)(lds + S * STAGE);  // [AT * 16]
  float* s_ssq = s_rinv + AT * 16;            // [2][AT * 16]

  // workgroup id -> (column block, K split, row block): ids congruent mod 8 share an XCD
  int q = blockIdx.x >> 3;
  const int rb = q % mblocks;
  q /= mblocks;
  const int split = q % splits;
  const int cb = (q / splits) * 8 + (blockIdx.x & 7);
  if (cb >= nblocks) return;
  __shared__ int s_last;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int KT = K >> 5, MTILES = (M + 15) >> 4, NT = N >> 4;
  const int mt0 = rb * AT, nt0 = cb * BF;

  // stage kt % S <- k-tiles kt KB .. kt KB + KB - 1 (the host gives every workgroup a whole number of stages): fragment f of a
  // k-tile (f < AF: X row tile mt0 + f, else W column tile nt0 + f - AF) is moved by wavefront f % NW
  const int kb = split * kt_per_split, nk = (min(KT, kb + kt_per_split) - kb) / KB;  // this workgroup's stages: k-tiles kb .. kb + nk KB - 1
  auto issue = [&](int kt) {
#pragma unroll
    for (int sub = 0; sub < KB; ++sub) {
    const int t = kb + min(kt, nk - 1) * KB + sub;
    unsigned char* base = lds + (kt % S) * STAGE + sub * NFR * 1024;
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int f = i * NW + wave;
      const op8* src;
      if (AF % NW == 0 ? i < AF / NW : f < AF) {  // (uniform in the wavefront)
        const int mt = min(mt0 + f, MTILES - 1);
        src = xt + ((size_t)mt * KT + t) * 64 + lane;
      } else {
        const int fw = min(f - AF, BF - 1);  // a wavefront without a fragment of its own in the last round moves the last one again
        const int nt = min(nt0 + fw, NT - 1);
        src = PR == 2 ? wt + (((size_t)(nt >> 1) * KT + t) * 2 + (nt & 1)) * 64 + lane : wt + ((size_t)nt * KT + t) * 64 + lane;
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(src), LDS_PTR(base + (AF + fw) * 1024), 16, 0, 0);
        continue;
      }
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(src), LDS_PTR(base + f * 1024), 16, 0, 0);
    }
    }
  };

  f32x4 acc[WN][WM];
#pragma unroll
  for (int j = 0; j < WN; ++j)
#pragma unroll
    for (int i = 0; i < WM; ++i) acc[j][i] = f32x4{0.f, 0.f, 0.f, 0.f};
  op8 xf[2][KB][WM], wf[2][KB][WN];
  auto read_frags = [&](int buf, int kt) {
#pragma unroll
    for (int sub = 0; sub < KB; ++sub) {
      const op8* st = (const op8*)(lds + (kt % S) * STAGE + sub * NFR * 1024) + lane;
#pragma unroll
      for (int i = 0; i < WM; ++i) xf[buf][sub][i] = st[(wm * WM + i) * 64];
#pragma unroll
      for (int j = 0; j < WN; ++j) wf[buf][sub][j] = st[(AF + wn * WN + j) * 64];
    }
  };
  auto multiply = [&](int buf) {
#pragma unroll
    for (int sub = 0; sub < KB; ++sub)
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int i = 0; i < WM; ++i) acc[j][i] = mfma_op(wf[buf][sub][j], xf[buf][sub][i], acc[j][i]);
  };

  // 1/rms of the workgroup's input rows, needed only by the epilogue: fetched before the pipeline starts (its loads are counted
  // by the compiler, the pipeline's by hand: the two must not be in flight together), all of a thread's loads in one trip;
  // published to the other wavefronts by the loop's barriers
  const int m_lo = mt0 * 16;
  if (EPI != EPI_RESID) block_rinv_batched<TPB, AT * 16>(e.rs, m_lo, max(0, min(M, m_lo + AT * 16) - m_lo), s_rinv);

#pragma unroll
  for (int s = 0; s < S - 1; ++s) issue(s);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * LPS) : "memory");  // stage 0 has landed (this wavefront's share)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  read_frags(0, 0);
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): as at the end of every step below
  // iteration kt: registers kt & 1 hold stage kt; stages kt + 1 .. kt + S - 2 are in flight
  auto step = [&](int buf, int kt) {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 3) * LPS) : "memory");  // stage kt + 1 has landed
    __builtin_amdgcn_s_barrier();  // ... for every wavefront, and every wavefront has finished with the buffer of stage kt - 1
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    issue(kt + S - 1);
    read_frags(buf ^ 1, kt + 1);
    multiply(buf);
    // Issue order, fixed by hand: the products (which depend on registers only) start right behind the barrier, and the copies
    // and the LDS reads of the next k-tile go out between them.  Left alone, the scheduler puts the reads next to their uses,
    // and all wavefronts of a SIMD, which leave the barrier together, would issue their loads while its matrix core idles.
    constexpr int NM = KB * WN * WM, RF = KB * (WM + WN);
    constexpr int OPS = 2 * (LPS + RF) <= NM ? 1 : 2;  // copies / reads per product: all of them go out in the first half of the products,
                                                        // so that the last read has the second half's time to return
#pragma unroll
    for (int i = 0; i < LPS; i += OPS) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one product
      __builtin_amdgcn_sched_group_barrier(0x010, OPS, 0);  // copies to LDS
    }
#pragma unroll
    for (int i = 0; i < RF; i += OPS) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, OPS, 0);  // LDS reads
    }
    __builtin_amdgcn_sched_group_barrier(0x008, NM, 0);  // what is left of the products
    __builtin_amdgcn_sched_barrier(0);
    // The reads have had the products' time to complete.  Waiting here, not at their first use behind the next step's reads:
    // the compiler counts the copies to LDS as possibly out of order on this counter and can only wait for everything.
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
  };
  // two k-tiles per trip, unconditionally: a fragment read that is used only behind a branch would be moved behind it, next to
  // its use, and the matrix cores would wait for LDS
  int kt = 0;
  for (; kt + 1 < nk; kt += 2) {
    step(0, kt);
    step(1, kt + 1);
  }
  if (kt < nk) step(0, kt);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the surplus loads of the last stages: LDS must be quiet before it is reused

  const int g = lane >> 4, ml = lane & 15;
  if (splits > 1) {
    // K split (narrow matrices at a few hundred rows, whose tiles alone cover half of the chip): partial tiles go to the fp32
    // workspace in the accumulator layout, written through to device scope; the workgroup that takes the tile's last ticket
    // re-reads them all, one split per trip to memory, adds them in split order and runs the epilogue (gemm_tiled.hip's protocol)
    const size_t stride = (size_t)M * N;
    auto offset = [&](int j, int i) { return ((unsigned)((wm * WM + i) * 16 + ml) * N + (nt0 + wn * WN + j) * 16 + 4 * g) * 4u; };
    auto exists = [&](int j, int i) { return nt0 + wn * WN + j < NT && m_lo + (wm * WM + i) * 16 + ml < M; };
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int i = 0; i < WM; ++i)
        if (exists(j, i))
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[j][i]), part_rsrc(e.part + split * stride + (size_t)m_lo * N), offset(j, i), 0, SC1);
    // Hand-off across workgroups (possibly across XCDs, whose L2s are separate): every wavefront waits until its own partial
    // stores, written through to device scope, have been acknowledged; then the workgroup takes its ticket with release order
    // at device scope, and the last arriver reads the partial tiles (device-scope loads) behind an acquire.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
      int* ticket = e.counters + cb * mblocks + rb;
      const int last = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT) == splits - 1;
      if (last) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next launch
      s_last = last;
    }
    __syncthreads();
    if (!s_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int i = 0; i < WM; ++i) acc[j][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < splits; ++s0) {
      u32x4 t[WN][WM];
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int i = 0; i < WM; ++i)
          t[j][i] = __builtin_amdgcn_raw_buffer_load_b128(part_rsrc(e.part + s0 * stride + (size_t)m_lo * N), exists(j, i) ? offset(j, i) : 0u, 0, SC1);
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int i = 0; i < WM; ++i) acc[j][i] += __builtin_bit_cast(f32x4, t[j][i]);
    }
  }

  // ---- epilogue
  __syncthreads();
  // The accumulators leave the registers through LDS (each wavefront its own region, half of its column tiles at a time), so
  // that the epilogue runs as a loop over fragments instead of 64 unrolled copies with every accumulator live.
  constexpr int HJ = WN / 2;
  f32x4* mine = (f32x4*)lds + wave * (HJ * WM * 64) + lane;
  float ssq[WM];
#pragma unroll
  for (int i = 0; i < WM; ++i) ssq[i] = 0.f;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    // what the fragments' epilogues read from memory (residual and gain; rotary cosines and sines) is fetched for up to twelve
    // fragments per trip instead of one trip per fragment
#pragma unroll
    for (int jj = 0; jj < HJ; ++jj)
#pragma unroll
      for (int i = 0; i < WM; ++i) mine[(jj * WM + i) * 64] = acc[h * HJ + jj][i];
    constexpr int IB = WM * HJ > 12 ? WM / 2 : WM;  // row tiles per trip: at most 12 fragments' worth of registers
#pragma unroll
    for (int i0 = 0; i0 < WM; i0 += IB) {
      EpiAhead ah[IB][HJ];
#pragma unroll
      for (int i = 0; i < IB; ++i)
#pragma unroll
        for (int jj = 0; jj < HJ; ++jj) {
          const int nt = nt0 + wn * WN + h * HJ + jj;
          ah[i][jj] = (EPI == EPI_RESID || EPI == EPI_QKV) && nt < NT ? epi_ahead<EPI>(e, M, N, m_lo + (wm * WM + i0 + i) * 16 + ml, nt * 16, g) : epi_none();
        }
#pragma unroll
      for (int i = 0; i < IB; ++i) {
        const int rl = (wm * WM + i0 + i) * 16 + ml;
        const float rinv = EPI == EPI_RESID ? 1.f : s_rinv[rl];
#pragma unroll
        for (int jj = 0; jj < HJ; ++jj) {
          const int nt = nt0 + wn * WN + h * HJ + jj;
          if (nt < NT) ssq[i0 + i] += finish_frag<EPI>(e, M, N, m_lo + rl, nt * 16, g, mine[(jj * WM + i0 + i) * 64], rinv, ah[i][jj]);  // uniform in the wavefront
        }
      }
    }
  }
  if (EPI == EPI_RESID) {  // the workgroup's share of sum h^2 per row: its two column halves in order
    if (g == 0)
#pragma unroll
      for (int i = 0; i < WM; ++i) s_ssq[wn * AT * 16 + (wm * WM + i) * 16 + ml] = ssq[i];
    __syncthreads();
    const int m = m_lo + tid;
    if (tid < AT * 16 && m < M) e.ssq_out[(size_t)m * nblocks + cb] = s_ssq[tid] + s_ssq[AT * 16 + tid];
  }
}

struct MacroPlan {
  int wm, wn, nw, nblocks, mblocks, splits, kps;
  bool two;  // two workgroups per compute unit (the three-stage variant of a four-wavefront tile)
  int kb;    // k-tiles per pipeline stage
};

// the tile with the least estimated time: rounds of workgroups over the chip x products per workgroup, each tile charged
// for what it fetches per product (measured: see penalty), plus the partial-tile traffic of a K split
int g_macro_wgs = 256;  // workgroups a K split aims at
constexpr int NCAND = 6;
// time of a round of workgroups over the chip / tile area, relative to 128 x 256 with four wavefronts (measured on the layer
// matrices of an 8B model with random operand values)
double g_macro_penalty[NCAND] = {0.63, 1.0, 0.96, 0.86, 0.72, 0.83};
// A four-wavefront tile that needs two or more rounds runs as two workgroups per compute unit, three stages each: the pair
// hides each other's barriers, waits and output stores and takes 1.45 (128 x 256) or 1.83 (128 x 128, against its faster
// eight-wavefront variant) of one deep workgroup's time instead of 2; the odd round's workgroups run at about the deep variant's pace (measured at 256 .. 2048 rows, operands of random values:
// constant ones let the chip clock higher and flatter the large tiles).
double g_macro_shared_pair[NCAND] = {0, 1.45, 1.83, 0, 0, 0}, g_macro_shared_single[NCAND] = {0, 1.15, 1.12, 0, 0, 0};
double g_macro_us_per_mac = 6.2e-7;  // a round of 128 x 256 tiles over the chip: microseconds per element of the tile and column of K

MacroPlan macro_plan(int M, int N, int K, bool may_split) {
  // {WM, WN, wavefronts}: 256 x 256, 128 x 256, 128 x 128, 192 x 256, 256 x 192, 192 x 192
  const int cand[NCAND][3] = {{4, 8, 8}, {4, 8, 4}, {4, 4, 4}, {6, 8, 4}, {4, 6, 8}, {3, 6, 8}};
  MacroPlan best{4, 8, 4, 1, 1, 1, 0, false, 1};
  double best_cost = 1e300;
  const int KT = K >> 5;
  for (int c = 0; c < NCAND; ++c) {
    if (g_macro_penalty[c] <= 0) continue;  // (tuning: a candidate switched off)
    const int bm = 8 * cand[c][2] * cand[c][0], bn = 32 * cand[c][1];
    const int mb = (M + bm - 1) / bm, nb = (N + bn - 1) / bn, tiles = mb * nb;
    // tiles that cover at most half of the chip (narrow matrices at a few hundred rows): split K until they cover it
    int sp = may_split ? g_macro_wgs / tiles : 1;
    if (sp > 4) sp = 4;
    if (sp > KT / 32) sp = KT / 32;  // at least 32 k-tiles per workgroup: the pipeline is up to 8 stages deep
    if (sp < 1) sp = 1;
    const int kps = (KT + sp - 1) / sp;
    sp = (KT + kps - 1) / kps;  // no empty split
    const int rounds = (tiles * sp + 255) / 256;
    const bool two = g_macro_shared_pair[c] > 0 && rounds >= 2;
    const double turns = two ? (rounds / 2) * g_macro_shared_pair[c] + (rounds & 1) * g_macro_shared_single[c] : rounds;
    // microseconds: the rounds' products, 1 / sp of K each; a split launch also writes and re-reads one partial tile (8 bytes per
    // element) per workgroup, at about 2.5 TB/s over the chip, and its last arriver fetches the splits one trip after another
    const double cost = turns * bm * bn * g_macro_penalty[c] * K * g_macro_us_per_mac / sp + (sp > 1 ? (double)tiles * sp * bm * bn * 3.2e-6 : 0.0) +
                        (sp > 2 ? 4.0 * (sp - 2) : 0.0);
    // a 128 x 128 tile alone on its compute unit: eight wavefronts, and two k-tiles per stage if every workgroup has a whole
    // number of such stages
    const bool alone = cand[c][2] == 4 && cand[c][1] == 4 && !two;
    const int kb = (alone && KT % sp == 0 && (KT / sp) % 2 == 0) ? 2 : 1;
    if (cost < best_cost) { best_cost = cost; best = MacroPlan{alone ? 2 : cand[c][0], cand[c][1], alone ? 8 : cand[c][2], nb, mb, sp, kps, two, kb}; }
  }
  return best;
}

template <int WM, int WN, int NW, int PR, int EPI, bool TWO = false, int KB = 1>
void launch_one(const op_t* xt, const op_t* wt, int M, int N, int K, const MacroPlan& p, const GemmEpi& e, hipStream_t st) {
  typedef MacroShape<WM, WN, NW, TWO, KB> SH;
  static bool configured = false;  // raise the dynamic LDS limit of this instantiation once
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)gemm_macro_kernel<WM, WN, PR, EPI, NW, TWO, KB>, hipFuncAttributeMaxDynamicSharedMemorySize, SH::LDS_BYTES);
    configured = true;
  }
  const int grid = (p.nblocks + 7) / 8 * 8 * p.mblocks * p.splits;
  DLM_LAUNCH((gemm_macro_kernel<WM, WN, PR, EPI, NW, TWO, KB>), grid, SH::TPB, SH::LDS_BYTES, st, (const op8*)xt, (const op8*)wt, M, N, K, p.nblocks,
             p.mblocks, p.splits, p.kps, e);
}

template <int PR, int EPI>
void launch_shape(const op_t* xt, const op_t* wt, int M, int N, int K, const MacroPlan& p, const GemmEpi& e, hipStream_t st) {
  if (p.nw == 8 && p.wm == 2) {
    if (p.kb == 2) launch_one<2, 4, 8, PR, EPI, false, 2>(xt, wt, M, N, K, p, e, st);
    else launch_one<2, 4, 8, PR, EPI>(xt, wt, M, N, K, p, e, st);
  }
  else if (p.nw == 8 && p.wm == 3) launch_one<3, 6, 8, PR, EPI>(xt, wt, M, N, K, p, e, st);
  else if (p.nw == 8 && p.wn == 6) launch_one<4, 6, 8, PR, EPI>(xt, wt, M, N, K, p, e, st);
  else if (p.nw == 8) launch_one<4, 8, 8, PR, EPI>(xt, wt, M, N, K, p, e, st);
  else if (p.wm == 6) launch_one<6, 8, 4, PR, EPI>(xt, wt, M, N, K, p, e, st);
  else if (p.two) {
    if (p.wn == 8) launch_one<4, 8, 4, PR, EPI, true>(xt, wt, M, N, K, p, e, st);
    else launch_one<4, 4, 4, PR, EPI, true>(xt, wt, M, N, K, p, e, st);
  }
  else launch_one<4, 8, 4, PR, EPI>(xt, wt, M, N, K, p, e, st);
}

template <int EPI>
void launch_epi(const op_t* xt, const op_t* wt, int M, int N, int K, const MacroPlan& p, const GemmEpi& e, hipStream_t st) {
  if (weight_pack_rows(N) == 2) launch_shape<2, EPI>(xt, wt, M, N, K, p, e, st);
  else launch_shape<1, EPI>(xt, wt, M, N, K, p, e, st);
}

}  // namespace

int gemm_macro_ssq_chunks(int M, int N, int K) { return macro_plan(M, N, K, true).nblocks; }  // (the plan of the launch itself)
int gemm_macro_splits(int M, int N, int K) { return macro_plan(M, N, K, true).splits; }
int gemm_macro_counters(int max_rows, int max_n) { return ((max_n + 127) / 128) * ((max_rows + 127) / 128); }  // 128 x 128 tiles are the smallest
void gemm_macro_set_target(int wgs) { g_macro_wgs = wgs; }
void gemm_macro_set_penalty(int tile, double p) {
  if (tile >= 0 && tile < NCAND) g_macro_penalty[tile] = p;
}

void launch_gemm_macro(const op_t* xt, const op_t* wt, int M, int N, int K, const GemmEpi& e, hipStream_t st) {
  const MacroPlan p = macro_plan(M, N, K, e.kind != EPI_DIRECT);  // EPI_DIRECT has no workspace
  switch (e.kind) {
    case EPI_QKV: launch_epi<EPI_QKV>(xt, wt, M, N, K, p, e, st); break;
    case EPI_SWIGLU: launch_epi<EPI_SWIGLU>(xt, wt, M, N, K, p, e, st); break;
    case EPI_RESID: launch_epi<EPI_RESID>(xt, wt, M, N, K, p, e, st); break;
    default: launch_epi<EPI_SUM>(xt, wt, M, N, K, p, e, st); break;
  }
}
