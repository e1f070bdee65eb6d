// fp32 GEMM  Y[M,N] = X[M,K] * W[N,K]^T  for the small fp32 model: 64x64 output tile per
// workgroup, 4x4 outputs per lane, operands staged through LDS in K-chunks of 16.
#include "common.h"

namespace {
constexpr int BM = 64, BN = 64, BK = 16;

__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ x, const float* __restrict__ w, float* __restrict__ y,
                                                       int M, int N, int K, RowScale rs) {
  __shared__ float xs[BK][BM + 1], ws[BK][BN + 1];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
    for (int i = tid; i < BM * BK; i += 256) {
      const int r = i / BK, kk = i % BK;
      xs[kk][r] = (m0 + r < M && k0 + kk < K) ? x[(size_t)(m0 + r) * K + k0 + kk] : 0.f;
      ws[kk][r] = (n0 + r < N && k0 + kk < K) ? w[(size_t)(n0 + r) * K + k0 + kk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = xs[kk][ty * 4 + i]; b[i] = ws[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
    float sc = 1.f;
    if (rs.ssq) {
      float ss = 0.f;
      for (int c = 0; c < rs.nch; ++c) ss += rs.ssq[(size_t)m * rs.nch + c];
      sc = rsqrtf(ss * rs.inv_d + rs.eps);
    }
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n < N) y[(size_t)m * N + n] = acc[i][j] * sc;
    }
  }
}
}  // namespace

void launch_gemm_f32(const float* x, const float* w, float* y, int M, int N, int K, RowScale rs, hipStream_t st) {
  dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM);
  DLM_LAUNCH(gemm_f32_kernel, grid, 256, 0, st, x, w, y, M, N, K, rs);
}
