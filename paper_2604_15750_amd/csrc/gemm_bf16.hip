// bf16 GEMM  Y[M,N] = X[M,K] * W[N,K]^T  on the gfx950 matrix cores, fp32 accumulation.
//
// At decode shapes (M = 8..384 rows against 15 GB of weights per pass) the GEMMs are bound by
// streaming W from HBM, so the design is a weight streamer that happens to multiply:
//   * W is re-tiled once, when the model is created, into 1 KiB fragments (16 rows x 32 k) that are
//     exactly the A operand of v_mfma_f32_16x16x32_bf16: a wavefront fetches a fragment as 64
//     consecutive 16-byte loads, and each wavefront walks one contiguous run of HBM along K;
//   * activations live in the same fragment tiling (B operand), written that way by their producer;
//     a workgroup stages the fragments of a K-chunk through LDS once and its four wavefronts share
//     them (each owns different output columns);
//   * the W fragments of the next K-chunk are in flight while the current one is multiplied
//     (8 KiB per wavefront), which is what keeps HBM busy;
//   * K is split across workgroups when N alone cannot fill 256 CUs; partial sums go to an fp32
//     workspace [splits][M][N] that the consumer kernel adds in a fixed order (deterministic).
// The product is computed transposed (W fragment = A operand), so that a lane ends up with four
// consecutive output columns of one row.
#include "common.h"

namespace {

constexpr int TPB = 256;
constexpr int KC = 4;  // k-tiles (of 32) per staged chunk

template <int MT, int R, bool OUT_BF16>
__global__ __launch_bounds__(TPB) void gemm_bf16_kernel(const bf16x8* __restrict__ xt, const bf16x8* __restrict__ wt,
                                                        float* __restrict__ out_f32, bf16_t* __restrict__ out_bf16, int M, int N, int K,
                                                        int kt_per_split, RowScale rs) {
  static_assert(R % 2 == 0, "row-tiles come in interleaved pairs");
  constexpr int XP = MT * KC / 4;  // 16-byte pieces of X each thread stages per chunk
  __shared__ bf16x8 xs[2][MT * KC * 64];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int KT = K >> 5, MTILES = (M + 15) >> 4, NPAIRS = N >> 5;
  const int mt0 = blockIdx.z * MT;
  const int pair0 = (blockIdx.x * 4 + wave) * (R / 2);
  const bool wave_active = pair0 < NPAIRS;
  const int t_begin = blockIdx.y * kt_per_split;
  const int t_end = min(KT, t_begin + kt_per_split);
  const int n_chunks = (t_end - t_begin + KC - 1) / KC;

  f32x4 acc[R][MT];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  bf16x8 wreg[2][KC][R];
  bf16x8 xreg[XP];
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  auto load_w = [&](bf16x8(&dst)[KC][R], int chunk) {
#pragma unroll
    for (int tc = 0; tc < KC; ++tc) {
      const int t = t_begin + chunk * KC + tc;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int pr = pair0 + (r >> 1);
        dst[tc][r] = (wave_active && t < t_end && pr < NPAIRS) ? wt[(((size_t)pr * KT + t) * 2 + (r & 1)) * 64 + lane] : zero8;
      }
    }
  };
  auto load_x = [&](int chunk) {
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const int q = tid + TPB * i;
      const int j = q / (KC * 64), tc = (q / 64) % KC, ln = q & 63;
      const int t = t_begin + chunk * KC + tc;
      xreg[i] = (mt0 + j < MTILES && t < t_end) ? xt[((size_t)(mt0 + j) * KT + t) * 64 + ln] : zero8;
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XP; ++i) xs[buf][tid + TPB * i] = xreg[i];
  };
  auto compute = [&](const bf16x8(&w)[KC][R], int buf) {
#pragma unroll
    for (int tc = 0; tc < KC; ++tc) {
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        const bf16x8 xf = xs[buf][(j * KC + tc) * 64 + lane];
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[tc][r], xf, acc[r][j], 0, 0, 0);
      }
    }
  };

  if (n_chunks > 0) {
    load_w(wreg[0], 0);
    load_x(0);
    store_x(0);
    __syncthreads();
    for (int c = 0; c < n_chunks; c += 2) {
      // even chunk: wreg[0] / xs[0] are current; prefetch chunk c+1 into wreg[1] / xs[1]
      if (c + 1 < n_chunks) { load_w(wreg[1], c + 1); load_x(c + 1); }
      compute(wreg[0], 0);
      if (c + 1 < n_chunks) store_x(1);
      __syncthreads();
      if (c + 1 >= n_chunks) break;
      if (c + 2 < n_chunks) { load_w(wreg[0], c + 2); load_x(c + 2); }
      compute(wreg[1], 1);
      if (c + 2 < n_chunks) store_x(0);
      __syncthreads();
    }
  }

  // epilogue: lane holds, per (r, j), columns n0..n0+3 of row m
  if (!wave_active) return;
  const int g = lane >> 4, ml = lane & 15;
  float sc[MT];
#pragma unroll
  for (int j = 0; j < MT; ++j) {
    sc[j] = 1.f;
    const int m = (mt0 + j) * 16 + ml;
    if (rs.ssq && m < M) {
      float ss = 0.f;
      for (int c = 0; c < rs.nch; ++c) ss += rs.ssq[(size_t)m * rs.nch + c];
      sc[j] = rsqrtf(ss * rs.inv_d + rs.eps);
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int nt = (pair0 + (r >> 1)) * 2 + (r & 1);
    if (nt * 16 >= N) continue;
    const int n0 = nt * 16 + g * 4;
#pragma unroll
    for (int j = 0; j < MT; ++j) {
      const int m = (mt0 + j) * 16 + ml;
      if (m >= M) continue;
      acc[r][j] *= sc[j];
      if (OUT_BF16) {
        bf16x4 o = {(bf16_t)acc[r][j][0], (bf16_t)acc[r][j][1], (bf16_t)acc[r][j][2], (bf16_t)acc[r][j][3]};
        *(bf16x4*)(out_bf16 + (size_t)m * N + n0) = o;
      } else {
        *(f32x4*)(out_f32 + ((size_t)blockIdx.y * M + m) * N + n0) = acc[r][j];
      }
    }
  }
}

// W [N, K] row-major -> fragment tiles, pairs of row-tiles interleaved along k.
__global__ void pack_weight_kernel(const bf16x8* __restrict__ w, bf16x8* __restrict__ out, int N, int K) {
  const int KT = K >> 5;
  const size_t total = (size_t)(N >> 4) * KT * 64;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int lane = idx & 63;
    const size_t tile = idx >> 6;
    const int sub = tile & 1;
    const size_t rest = tile >> 1;
    const int t = rest % KT;
    const int pr = rest / KT;
    const int n = (pr * 2 + sub) * 16 + (lane & 15);
    const int k8 = t * 4 + (lane >> 4);
    out[idx] = w[(size_t)n * (K >> 3) + k8];
  }
}

// X [M, K] row-major -> fragment tiles [ceil(M/16)][K/32]; rows beyond M are zero.
__global__ void pack_act_kernel(const bf16x8* __restrict__ x, bf16x8* __restrict__ out, int M, int K) {
  const int KT = K >> 5;
  const size_t total = (size_t)((M + 15) >> 4) * KT * 64;
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int lane = idx & 63;
    const size_t tile = idx >> 6;
    const int t = tile % KT;
    const int m = (int)(tile / KT) * 16 + (lane & 15);
    out[idx] = m < M ? x[(size_t)m * (K >> 3) + t * 4 + (lane >> 4)] : zero8;
  }
}

template <int MT, int R>
void launch_mt(const bf16_t* xt, const bf16_t* wt, float* out_f32, bf16_t* out_bf16, int M, int N, int K, int splits, int mblocks, RowScale rs, hipStream_t st) {
  const int KT = K >> 5;
  const int kps = ((KT + splits - 1) / splits + KC - 1) / KC * KC;
  const int groups = ((N >> 5) + 4 * (R / 2) - 1) / (4 * (R / 2));
  dim3 grid(groups, splits, mblocks);
  if (out_bf16) gemm_bf16_kernel<MT, R, true><<<grid, TPB, 0, st>>>((const bf16x8*)xt, (const bf16x8*)wt, nullptr, out_bf16, M, N, K, kps, rs);
  else gemm_bf16_kernel<MT, R, false><<<grid, TPB, 0, st>>>((const bf16x8*)xt, (const bf16x8*)wt, out_f32, nullptr, M, N, K, kps, rs);
}

}  // namespace

void launch_pack_weight(const bf16_t* w, bf16_t* out, int N, int K, hipStream_t st) {
  pack_weight_kernel<<<2048, 256, 0, st>>>((const bf16x8*)w, (bf16x8*)out, N, K);
}
void launch_pack_act(const bf16_t* x, bf16_t* out, int M, int K, hipStream_t st) {
  pack_act_kernel<<<512, 256, 0, st>>>((const bf16x8*)x, (bf16x8*)out, M, K);
}

// Number of K-splits: enough workgroups to cover the chip a few times, at least 8 k-tiles each.
int gemm_bf16_splits(int M, int N, int K) {
  const int KT = K >> 5;
  const int groups = ((N >> 5) + 3) / 4;
  const int mblocks = (((M + 15) >> 4) + 15) / 16;
  int s = (768 + groups * mblocks - 1) / (groups * mblocks);
  const int max_s = KT / 8 > 0 ? KT / 8 : 1;
  if (s > max_s) s = max_s;
  if (s > 32) s = 32;
  if (s < 1) s = 1;
  // splits that leave no empty tail
  const int kps = ((KT + s - 1) / s + KC - 1) / KC * KC;
  return (KT + kps - 1) / kps;
}

void launch_gemm_bf16(const bf16_t* xt, const bf16_t* wt, float* out_f32, bf16_t* out_bf16, int M, int N, int K, int splits, RowScale rs,
                      hipStream_t st) {
  const int mtiles = (M + 15) >> 4;
#define GO(MT) launch_mt<MT, 2>(xt, wt, out_f32, out_bf16, M, N, K, splits, (mtiles + MT - 1) / MT, rs, st)
  if (mtiles <= 1) GO(1);
  else if (mtiles <= 2) GO(2);
  else if (mtiles <= 3) GO(3);
  else if (mtiles <= 4) GO(4);
  else if (mtiles <= 6) GO(6);
  else if (mtiles <= 8) GO(8);
  else if (mtiles <= 12) GO(12);
  else GO(16);
#undef GO
}
