// Skinny GEMM of a bf16 model (M <= 64 rows): Y[M,N] = X[M,K] * W[N,K]^T, fp32 accumulation, epilogue fused.
//
// One workgroup per 16- or 32-column output tile over the whole of K.  Its wavefronts split K among
// themselves; each keeps 8 KiB of W fragments (and the matching X fragments) in flight, HBM ->
// registers, and multiplies them on the matrix cores; the accumulators are added through LDS in
// wavefront order (deterministic).  No workgroup waits for another: no workspace, no counter, no
// serial tail.  With 256 .. 768 workgroups all resident at once, HBM stays busy from the first load
// to the last.  Every workgroup re-reads X through its L2, which costs as much of the compute units'
// load bandwidth as W itself for the narrow matrices, so lanes whose row does not exist fetch no line of
// their own (they re-read a row that exists): a fragment's 128-byte lines hold 8 rows each, and a block
// of 8 rows (the minimum block length) reads half of them.
#include "gemm_epilogue.h"

namespace {

// grid.x = N / (16 R) workgroups of NWV wavefronts; wavefront w multiplies k-tiles [w*per, (w+1)*per) of the
// workgroup's R column tiles against all MT row tiles, D k-tiles per batch, two batches of registers.
// STEPS: W is read from the step-major copy (e.w_steps) instead of wt.
template <int MT, int R, int NWV, int D, int EPI, bool STEPS = false>
__global__ __launch_bounds__(NWV * 64) void gemm_skinny_kernel(const op8* __restrict__ xt, const op8* __restrict__ wt, int M, int N,
                                                               int K, GemmEpi e) {
  __shared__ f32x4 red[NWV][R * MT][64];
  __shared__ float s_rinv[MT * 16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int KT = K >> 5, MTILES = (M + 15) >> 4;
  const int per = (KT + NWV - 1) / NWV;
  const int t_begin = wave * per, t_end = min(KT, t_begin + per);
  const op8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  // lanes of the last row tile whose row does not exist re-read row 0 of their k-group (whatever they get is never stored)
  const int xlane_last = (MTILES - 1) * 16 + (lane & 15) < M ? lane : (lane & ~15);
  // the workgroup's R tiles are one interleaved run; in the step-major copy (KT a multiple of NWV: the host checks) the
  // wavefront's step s is the R fragments from ((s * workgroups + this workgroup) * NWV + wave) * R on
  constexpr bool steps = STEPS;
  const op8* wbase = steps ? (const op8*)e.w_steps + ((size_t)blockIdx.x * NWV + wave) * R * 64 + lane : wt + (size_t)blockIdx.x * KT * R * 64 + lane;
  const size_t wstride = steps ? (size_t)gridDim.x * NWV * R * 64 : R * 64;
  const int tsub = steps ? t_begin : 0;

  f32x4 acc[R][MT];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  op8 wreg[2][D][R], xreg[2][D][MT];

  auto load = [&](int buf, int tb) {
#pragma unroll
    for (int i = 0; i < D; ++i) {
      const int t = tb + i;
      const bool ok = t < t_end;
#pragma unroll
      for (int r = 0; r < R; ++r) wreg[buf][i][r] = ok ? wbase[(size_t)(t - tsub) * wstride + r * 64] : zero8;
#pragma unroll
      for (int j = 0; j < MT; ++j) xreg[buf][i][j] = (ok && j < MTILES) ? xt[((size_t)j * KT + t) * 64 + (j == MTILES - 1 ? xlane_last : lane)] : zero8;
    }
  };
  auto compute = [&](int buf) {
#pragma unroll
    for (int i = 0; i < D; ++i)
#pragma unroll
      for (int j = 0; j < MT; ++j)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r][j] = mfma_op(wreg[buf][i][r], xreg[buf][i][j], acc[r][j]);
  };

  load(0, t_begin);
  // 1/rms of the input rows, needed only by the epilogue: fetched while the first batch is in flight; so is what the epilogue
  // of the tile this wavefront finishes first reads from memory (tile rj = wave of the R * MT)
  if (EPI != EPI_RESID) block_rinv<NWV * 64>(e.rs, 0, min(M, MT * 16), s_rinv);
  EpiAhead ahead = epi_none();
  if ((EPI == EPI_RESID || EPI == EPI_QKV) && wave < R * MT)
    ahead = epi_ahead<EPI>(e, M, N, (wave % MT) * 16 + (lane & 15), (blockIdx.x * R + wave / MT) * 16, lane >> 4);
  for (int tb = t_begin; tb < t_end; tb += 2 * D) {
    load(1, tb + D);
    compute(0);
    load(0, tb + 2 * D);
    compute(1);
  }

#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < MT; ++j) red[wave][r * MT + j][lane] = acc[r][j];
  __syncthreads();

  const int g = lane >> 4, ml = lane & 15;
  for (int rj = wave; rj < R * MT; rj += NWV) {  // one wavefront finishes one 16 x 16 tile
    const int r = rj / MT, j = rj % MT;
    const int m = j * 16 + ml;
    const int nt = blockIdx.x * R + r;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < NWV; ++w) v += red[w][rj][lane];
    const float ss = finish_frag<EPI>(e, M, N, m, nt * 16, g, v, EPI == EPI_RESID ? 1.f : s_rinv[j * 16 + ml], rj == wave ? ahead : epi_none());
    if (EPI == EPI_RESID && g == 0 && m < M) e.ssq_out[(size_t)m * (N >> 4) + nt] = ss;
  }
}

// batch depth: 8 KiB of W in flight per wavefront for up to 32 rows, half of that beyond (the X fragments take the registers);
// the step-major copy reads best with batches of four (measured: deeper batches add queueing, not bandwidth)
template <int MT, int EPI>
void launch_skinny(const op_t* xt, const op_t* wt, int pr, int M, int N, int K, const GemmEpi& e, hipStream_t st) {
  if (pr == 1 && e.w_steps) DLM_LAUNCH((gemm_skinny_kernel<MT, 1, 8, 4, EPI, true>), N / 16, 512, 0, st, (const op8*)xt, (const op8*)wt, M, N, K, e);
  else if (pr == 1) DLM_LAUNCH((gemm_skinny_kernel<MT, 1, 8, (MT <= 2 ? 8 : 4), EPI>), N / 16, 512, 0, st, (const op8*)xt, (const op8*)wt, M, N, K, e);
  else if (e.w_steps) DLM_LAUNCH((gemm_skinny_kernel<MT, 2, 4, (MT <= 2 ? 4 : 2), EPI, true>), N / 32, 256, 0, st, (const op8*)xt, (const op8*)wt, M, N, K, e);
  else DLM_LAUNCH((gemm_skinny_kernel<MT, 2, 4, (MT <= 2 ? 4 : 2), EPI>), N / 32, 256, 0, st, (const op8*)xt, (const op8*)wt, M, N, K, e);
}

template <int EPI>
void launch_epi(const op_t* xt, const op_t* wt, int pr, int M, int N, int K, const GemmEpi& e, hipStream_t st) {
  if (M <= 16) launch_skinny<1, EPI>(xt, wt, pr, M, N, K, e, st);
  else if (M <= 32) launch_skinny<2, EPI>(xt, wt, pr, M, N, K, e, st);
  else if (M <= 48) launch_skinny<3, EPI>(xt, wt, pr, M, N, K, e, st);
  else launch_skinny<4, EPI>(xt, wt, pr, M, N, K, e, st);
}

}  // namespace

void launch_gemm_skinny(const op_t* xt, const op_t* wt, int pr, int M, int N, int K, const GemmEpi& e_in, hipStream_t st) {
  GemmEpi e = e_in;
  // the step-major copy serves the launches it was laid out for: pr column tiles per workgroup, 8 wavefronts (pr 1) or 4 (pr 2)
  if (!(e.w_steps && e.w_steps_ct == pr && (K >> 5) % (pr == 1 ? 8 : 4) == 0 && N % (16 * pr) == 0)) e.w_steps = nullptr;
  switch (e.kind) {
    case EPI_QKV: launch_epi<EPI_QKV>(xt, wt, pr, M, N, K, e, st); break;
    case EPI_SWIGLU: launch_epi<EPI_SWIGLU>(xt, wt, pr, M, N, K, e, st); break;
    case EPI_RESID: launch_epi<EPI_RESID>(xt, wt, pr, M, N, K, e, st); break;
    default: launch_epi<EPI_SUM>(xt, wt, pr, M, N, K, e, st); break;
  }
}
