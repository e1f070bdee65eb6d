// Tiled GEMM of a bf16 model (M > 32 rows, and the LM head): Y[M,N] = X[M,K] * W[N,K]^T, fp32 accumulation,
// epilogue fused.
//
// A workgroup of four wavefronts owns up to 128 rows (MT row tiles) x 128 or 256 columns; a wavefront
// owns TR = 2 or 4 adjacent 16-column tiles and all the rows.
//   * W fragments go HBM -> registers, three chunks (of 2 k-tiles) deep, each used for MT products;
//   * the X fragments of a chunk are staged through LDS once per workgroup (three buffers; the
//     global loads run three chunks ahead of their use) and every one is read back by all four
//     wavefronts, TR products per read;
//   * one barrier per chunk.
// More than 128 rows are covered by several row blocks; blocks that share columns (and so stream the
// same W) get adjacent workgroup ids congruent mod 8, i.e. they run at the same time on the same XCD
// and the second reader finds W in that XCD's L2.
// K is split across workgroups when columns x row blocks cannot fill the chip: partial tiles go to
// an fp32 workspace, written through and read with device scope (sc1; a tile row of one workgroup
// is at least 512 contiguous bytes, so no cache line has two writers).  Every wavefront waits for the
// acknowledgement of its own stores before the workgroup's barrier, the ticket is taken with release
// order at device scope, and the workgroup that arrives last passes an acquire fence before it
// re-reads the partial tiles into the accumulator layout, adds them in split order (deterministic)
// and runs the epilogue.
#include "gemm_epilogue.h"
#include "stats_part.h"

namespace {

constexpr int TPB = 256;
constexpr int KC = 2;  // k-tiles (of 32) per chunk

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int SC1 = 16;  // cache-policy bit of the raw-buffer builtins: device scope

__device__ inline __amdgpu_buffer_rsrc_t tile_rsrc(const float* base) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, 0x7fffffff, 0x00020000);
}

// The part of a row's online-softmax state that a pass without a previous-step distribution needs (stats_part.h has the whole):
// maximum (= the best logit), sum e^(z-m), sum e^(z-m)(z-m), lowest token id of the maximum.
struct LiteState {
  float m, s, t;
  int bi;
};
__device__ __attribute__((always_inline)) inline LiteState lite_merge(const LiteState a, const LiteState b) {
  LiteState r;
  r.m = fmaxf(a.m, b.m);
  const float da = a.m - r.m, db = b.m - r.m;
  const float fa = __expf(da), fb = __expf(db);
  r.s = fa * a.s + fb * b.s;
  r.t = fa * (a.t + da * a.s) + fb * (b.t + db * b.s);
  r.bi = (b.m > a.m || (b.m == a.m && b.bi < a.bi)) ? b.bi : a.bi;
  return r;
}
__device__ __attribute__((always_inline)) inline LiteState lite_shfl_xor(const LiteState p, int o) {
  return LiteState{__shfl_xor(p.m, o, 64), __shfl_xor(p.s, o, 64), __shfl_xor(p.t, o, 64), __shfl_xor(p.bi, o, 64)};
}
// state of four consecutive logits, token ids n .. n+3, token `skip` left out
__device__ __attribute__((always_inline)) inline LiteState lite_of(f32x4 v, int n, int skip) {
  float z[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) z[i] = (float)(bf16_t)v[i];  // the logit as stored
  LiteState r{NEG_BIG, 0.f, 0.f, 0x7fffffff};
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (n + i != skip && z[i] > r.m) { r.m = z[i]; r.bi = n + i; }  // ascending ids and strict '>' keep the lowest id
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (n + i == skip) continue;
    const float d = z[i] - r.m, ex = __expf(d);
    r.s += ex;
    r.t = fmaf(ex, d, r.t);
  }
  return r;
}

// TR column tiles per wavefront (workgroups of 64 TR columns); PR = 2: weights packed in interleaved pairs, 1: single runs.
template <int MT, int TR, int PR, int EPI>
__global__ __launch_bounds__(TPB) void gemm_tiled_kernel(const op8* __restrict__ xt, const op8* __restrict__ wt, int M, int N, int K,
                                                         int kt_per_split, int splits, int groups, int mblocks, GemmEpi e) {
  constexpr int XPIECES = MT * KC * 64;            // 16-byte pieces of X per chunk
  constexpr int XP = (XPIECES + TPB - 1) / TPB;    // per thread
  __shared__ op8 xs[3][XPIECES];
  __shared__ float s_rinv[MT * 16];
  __shared__ float s_ssq[4][MT * 16];
  __shared__ int s_last;

  // workgroup id -> (column group, K split, row block): ids congruent mod 8 share an XCD
  int q = blockIdx.x >> 3;
  const int rb = q % mblocks;
  q /= mblocks;
  const int split = q % splits;
  const int group = (q / splits) * 8 + (blockIdx.x & 7);
  if (group >= groups) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int KT = K >> 5, MTILES = (M + 15) >> 4, NT = N >> 4;
  const int mt0 = rb * MT;
  const int nt0 = (group * 4 + wave) * TR;
  const int t_begin = split * kt_per_split;
  const int t_end = min(KT, t_begin + kt_per_split);
  const int n_chunks = (t_end - t_begin + KC - 1) / KC;
  const op8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  const op8* wptr[TR];  // fragment (nt0 + r, k-tile t) = wptr[r][t * wstep]
  constexpr size_t wstep = PR == 2 ? 128 : 64;
#pragma unroll
  for (int r = 0; r < TR; ++r) {
    const int nt = nt0 + r;
    wptr[r] = PR == 2 ? wt + ((size_t)(nt >> 1) * KT * 2 + (nt & 1)) * 64 + lane : wt + (size_t)nt * KT * 64 + lane;
  }

  f32x4 acc[TR][MT];
#pragma unroll
  for (int r = 0; r < TR; ++r)
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  op8 wreg[3][KC][TR], xreg[3][XP];

  auto load_w = [&](op8(&dst)[KC][TR], int chunk) {
#pragma unroll
    for (int tc = 0; tc < KC; ++tc) {
      const int t = t_begin + chunk * KC + tc;
#pragma unroll
      for (int r = 0; r < TR; ++r) dst[tc][r] = (nt0 + r < NT && t < t_end) ? wptr[r][t * wstep] : zero8;
    }
  };
  auto load_x = [&](op8(&dst)[XP], int chunk) {
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const int p = tid + TPB * i;
      const int j = p / (KC * 64), tc = (p / 64) % KC, ln = p & 63;
      const int t = t_begin + chunk * KC + tc;
      dst[i] = (p < XPIECES && mt0 + j < MTILES && t < t_end) ? xt[((size_t)(mt0 + j) * KT + t) * 64 + ln] : zero8;
    }
  };
  auto store_x = [&](int buf, const op8(&src)[XP]) {
#pragma unroll
    for (int i = 0; i < XP; ++i)
      if (tid + TPB * i < XPIECES) xs[buf][tid + TPB * i] = src[i];
  };
  auto compute = [&](const op8(&w)[KC][TR], int buf) {
#pragma unroll
    for (int tc = 0; tc < KC; ++tc) {
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        const op8 xf = xs[buf][(j * KC + tc) * 64 + lane];
#pragma unroll
        for (int r = 0; r < TR; ++r) acc[r][j] = mfma_op(w[tc][r], xf, acc[r][j]);
      }
    }
  };

  // chunk k lives in register set k % 3 (W: loaded 2 chunks ahead; X: loaded 3 ahead, stored to LDS buffer k % 3 one ahead)
  load_w(wreg[0], 0);
  load_x(xreg[0], 0);
  load_w(wreg[1], 1);
  load_x(xreg[1], 1);
  load_x(xreg[2], 2);
  // 1/rms of the input rows for the epilogue, fetched while the first chunks are in flight (published by the loop's barriers)
  if (EPI != EPI_RESID) block_rinv<TPB>(e.rs, mt0 * 16, max(0, min(M, (mt0 + MT) * 16) - mt0 * 16), s_rinv);
  store_x(0, xreg[0]);
  __syncthreads();
#define STEP(S, c)                                   \
  {                                                  \
    load_w(wreg[(S + 2) % 3], (c) + 2);              \
    store_x((S + 1) % 3, xreg[(S + 1) % 3]);         \
    load_x(xreg[S], (c) + 3);                        \
    compute(wreg[S], S);                             \
    __syncthreads();                                 \
  }
  for (int c = 0; c < n_chunks; c += 3) {
    STEP(0, c)
    if (c + 1 < n_chunks) STEP(1, c + 1)
    if (c + 2 < n_chunks) STEP(2, c + 2)
  }
#undef STEP

  const int g = lane >> 4, ml = lane & 15;
  const int m_lo = mt0 * 16;
  if (splits > 1) {
    // partial tile -> workspace, in the accumulator layout, written through to device scope
    const size_t stride = (size_t)M * N;
    float* mine = e.part + split * stride;
#pragma unroll
    for (int r = 0; r < TR; ++r) {
      if (nt0 + r >= NT) continue;
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        const int m = m_lo + j * 16 + ml;
        if (m < M)
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[r][j]), tile_rsrc(mine + (size_t)m_lo * N),
                                                 ((unsigned)(j * 16 + ml) * N + (nt0 + r) * 16 + 4 * g) * 4u, 0, SC1);
      }
    }
    // Hand-off across workgroups (possibly across XCDs, whose L2s are separate): every wavefront waits until its own partial
    // stores, written through to device scope, have been acknowledged; then the workgroup takes its ticket with release order
    // at device scope, and the last arriver reads the partial tiles (device-scope loads) behind an acquire.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
      int* ticket = e.counters + group * mblocks + rb;
      const int last = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT) == splits - 1;
      if (last) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next launch
      s_last = last;
    }
    __syncthreads();
    if (!s_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    // the finished tile = the partial tiles added in split order; eight loads in flight per trip to memory
#pragma unroll
    for (int r = 0; r < TR; ++r) {
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        const int m = m_lo + j * 16 + ml;
        if (nt0 + r < NT && m < M) {
          const unsigned off = ((unsigned)(j * 16 + ml) * N + (nt0 + r) * 16 + 4 * g) * 4u;
          for (int s0 = 0; s0 < splits; s0 += 8) {
            u32x4 t[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)  // the surplus loads of the last batch repeat its last split and are not added
              t[i] = __builtin_amdgcn_raw_buffer_load_b128(tile_rsrc(e.part + min(s0 + i, splits - 1) * stride + (size_t)m_lo * N), off, 0, SC1);
#pragma unroll
            for (int i = 0; i < 8; ++i)
              if (s0 + i < splits) v += __builtin_bit_cast(f32x4, t[i]);
          }
        }
        acc[r][j] = v;
      }
    }
  }

  if constexpr (EPI == EPI_STATS) {
    // logits as EPI_DIRECT writes them, and the online-softmax state of this workgroup's columns of every row, over the values as
    // written: lane -> the four lanes of a row -> the wavefront's tiles -> the four wavefronts, each in a fixed order
    __shared__ LiteState s_state[4][MT * 16];
    LiteState acc_state[MT];
#pragma unroll
    for (int j = 0; j < MT; ++j) acc_state[j] = LiteState{NEG_BIG, 0.f, 0.f, 0x7fffffff};
#pragma unroll
    for (int r = 0; r < TR; ++r) {
      if (nt0 + r >= NT) continue;  // uniform in the wavefront
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        const int m = m_lo + j * 16 + ml, n = (nt0 + r) * 16 + 4 * g;
        const f32x4 v = acc[r][j] * s_rinv[j * 16 + ml];
        if (m < M) *(bf16x4*)(e.out_bf16 + (size_t)m * N + n) = to_bf16x4(v);
        acc_state[j] = lite_merge(acc_state[j], lite_of(v, n, e.skip_col));
      }
    }
#pragma unroll
    for (int j = 0; j < MT; ++j) {
      acc_state[j] = lite_merge(acc_state[j], lite_shfl_xor(acc_state[j], 16));
      acc_state[j] = lite_merge(acc_state[j], lite_shfl_xor(acc_state[j], 32));
      if (g == 0) s_state[wave][j * 16 + ml] = acc_state[j];
    }
    __syncthreads();
    const int m = m_lo + tid;
    if (tid < MT * 16 && m < M) {
      const LiteState w0 = s_state[0][tid], w1 = s_state[1][tid], w2 = s_state[2][tid], w3 = s_state[3][tid];
      const LiteState r = lite_merge(lite_merge(lite_merge(w0, w1), w2), w3);
      f32x4* dst = (f32x4*)((Part*)e.stat_parts + (size_t)m * groups + group);  // Part{m, s, t, w = 0, bv = m, bi, pm, ps = 0}
      static_assert(sizeof(Part) == 32 && offsetof(Part, bv) == 16 && offsetof(Part, bi) == 20, "Part is written as two vectors");
      dst[0] = f32x4{r.m, r.s, r.t, 0.f};
      dst[1] = f32x4{r.m, __int_as_float(r.bi), NEG_BIG, 0.f};
    }
    return;
  }

  float ssq[MT];
#pragma unroll
  for (int j = 0; j < MT; ++j) ssq[j] = 0.f;
#pragma unroll
  for (int r = 0; r < TR; ++r) {
    if (nt0 + r >= NT) continue;  // uniform in the wavefront
#pragma unroll
    for (int j = 0; j < MT; ++j)
      ssq[j] += finish_frag<EPI>(e, M, N, m_lo + j * 16 + ml, (nt0 + r) * 16, g, acc[r][j], EPI == EPI_RESID ? 1.f : s_rinv[j * 16 + ml]);
  }
  if (EPI == EPI_RESID) {  // the workgroup's share of sum h^2 per row: its four wavefronts in order
    if (g == 0)
#pragma unroll
      for (int j = 0; j < MT; ++j) s_ssq[wave][j * 16 + ml] = ssq[j];
    __syncthreads();
    const int m = m_lo + tid;
    if (tid < MT * 16 && m < M) e.ssq_out[(size_t)m * groups + group] = ((s_ssq[0][tid] + s_ssq[1][tid]) + s_ssq[2][tid]) + s_ssq[3][tid];
  }
}

int g_target_wgs = 384;

struct Plan {
  int pr, tr;  // packing of the weights; column tiles per wavefront
  int groups, mtiles, mblocks, mt, splits, kps;
};
Plan plan(int M, int N, int K, bool may_split = true) {
  Plan p;
  p.pr = weight_pack_rows(N);
  p.mtiles = (M + 15) >> 4;
  p.mblocks = (p.mtiles + 7) / 8;
  p.mt = (p.mtiles + p.mblocks - 1) / p.mblocks;
  // 256-column workgroups read each X fragment for twice the products, but only pay when they alone fill most of the chip
  p.tr = (p.pr == 2 && (N + 255) / 256 * p.mblocks >= 192) ? 4 : 2;
  p.groups = (N + 64 * p.tr - 1) / (64 * p.tr);
  const int KT = K >> 5;
  const int wgs = p.groups * p.mblocks;
  int s = wgs >= 160 ? 1 : (g_target_wgs + wgs - 1) / wgs;  // splitting K costs a round trip of the partial tiles through memory
  if (s > 8) s = 8;                             // a short serial tail for the last arriver
  if (s > KT / 8) s = KT / 8;                   // at least four chunks per split
  if (s < 1 || !may_split) s = 1;
  p.kps = ((KT + s - 1) / s + KC - 1) / KC * KC;
  p.splits = (KT + p.kps - 1) / p.kps;          // no empty split
  return p;
}

template <int MT, int EPI>
void launch_mt(const op_t* xt, const op_t* wt, int M, int N, int K, const Plan& p, const GemmEpi& e, hipStream_t st) {
  const int grid = (p.groups + 7) / 8 * 8 * p.splits * p.mblocks;
#define GO(TR, PR) DLM_LAUNCH((gemm_tiled_kernel<MT, TR, PR, EPI>), grid, TPB, 0, st, (const op8*)xt, (const op8*)wt, M, N, K, p.kps, p.splits, p.groups, p.mblocks, e)
  if (p.pr == 1) GO(2, 1);
  else if (p.tr == 2) GO(2, 2);
  else GO(4, 2);
#undef GO
}

// EPI_STATS serves at most GEMM_STATS_MAX_ROWS = 64 rows: four row tiles
void launch_stats(const op_t* xt, const op_t* wt, int M, int N, int K, const Plan& p, const GemmEpi& e, hipStream_t st) {
  switch (p.mt) {
    case 1: launch_mt<1, EPI_STATS>(xt, wt, M, N, K, p, e, st); break;
    case 2: launch_mt<2, EPI_STATS>(xt, wt, M, N, K, p, e, st); break;
    case 3: launch_mt<3, EPI_STATS>(xt, wt, M, N, K, p, e, st); break;
    default: launch_mt<4, EPI_STATS>(xt, wt, M, N, K, p, e, st); break;
  }
}

template <int EPI>
void launch_epi(const op_t* xt, const op_t* wt, int M, int N, int K, const Plan& p, const GemmEpi& e, hipStream_t st) {
  switch (p.mt) {
    case 1: launch_mt<1, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 2: launch_mt<2, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 3: launch_mt<3, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 4: launch_mt<4, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 5: launch_mt<5, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 6: launch_mt<6, EPI>(xt, wt, M, N, K, p, e, st); break;
    case 7: launch_mt<7, EPI>(xt, wt, M, N, K, p, e, st); break;
    default: launch_mt<8, EPI>(xt, wt, M, N, K, p, e, st); break;
  }
}

}  // namespace

void gemm_tiled_set_target(int wgs) { g_target_wgs = wgs; }
int gemm_tiled_splits(int M, int N, int K) { return plan(M, N, K).splits; }
int gemm_tiled_ssq_chunks(int M, int N) { return plan(M, N, 32).groups; }
int gemm_tiled_stat_parts(int M, int N) { return plan(M, N, 32, false).groups; }
int gemm_tiled_counters(int max_rows, int max_n) { return ((max_n + 127) / 128) * (((max_rows + 15) / 16 + 7) / 8); }  // 128-column groups are the narrowest

void launch_gemm_tiled(const op_t* xt, const op_t* wt, int M, int N, int K, const GemmEpi& e, hipStream_t st) {
  const Plan p = plan(M, N, K, e.kind != EPI_DIRECT && e.kind != EPI_STATS);  // the LM head's epilogues have no workspace
  switch (e.kind) {
    case EPI_STATS: launch_stats(xt, wt, M, N, K, p, e, st); break;
    case EPI_QKV: launch_epi<EPI_QKV>(xt, wt, M, N, K, p, e, st); break;
    case EPI_SWIGLU: launch_epi<EPI_SWIGLU>(xt, wt, M, N, K, p, e, st); break;
    // (EPI_RESID is never sent here: choose_kernel in gemm_bf16.hip)
    default: launch_epi<EPI_SUM>(xt, wt, M, N, K, p, e, st); break;
  }
}
