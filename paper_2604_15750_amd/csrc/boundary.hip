// DepGA-Block boundary search (paper Sec. 4.2, Eq. 4; cumulative form of Sec. 4.4).
// One workgroup per sequence, one lane per candidate position (window <= 256).  Smoothing uses
// differences of a prefix sum, the cumulative rule a second prefix sum; both are wavefront-shuffle
// scans with a cross-wave carry, in fp64 so the decision does not depend on summation order.
#include "common.h"

namespace {

constexpr int TPB = 256;
constexpr int NW = TPB / 64;

__device__ inline double block_scan_inclusive(double v, double* carry /* [NW] shared */) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    double u = __shfl_up(v, o, 64);
    if (lane >= o) v += u;
  }
  __syncthreads();  // carry may still be read from a previous scan
  if (lane == 63) carry[wv] = v;
  __syncthreads();
  double add = 0.0;
  for (int i = 0; i < wv; ++i) add += carry[i];
  return v + add;
}

template <typename Op>
__device__ inline double block_reduce(double v, double* buf /* [NW] shared */, Op op) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = op(v, __shfl_xor(v, o, 64));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = v;
  __syncthreads();
  double r = buf[0];
  for (int i = 1; i < NW; ++i) r = op(r, buf[i]);
  return r;
}

struct OpSum { __device__ double operator()(double a, double b) const { return a + b; } };
struct OpMin { __device__ double operator()(double a, double b) const { return a < b ? a : b; } };
struct OpMax { __device__ double operator()(double a, double b) const { return a > b ? a : b; } };

// smoothed and normalised signal for position k (inactive lanes pass x = 0 and get 0)
__device__ inline double smooth_normalise(double x, int k, int W, int r, int mode, double* pre /* [TPB+1] */, double* buf) {
  const bool act = k < W;
  double inc = block_scan_inclusive(act ? x : 0.0, buf);
  if (threadIdx.x == 0) pre[0] = 0.0;
  pre[threadIdx.x + 1] = inc;
  __syncthreads();
  double sm = 0.0;
  if (act) {
    int lo = max(0, k - r), hi = min(W - 1, k + r);
    sm = (pre[hi + 1] - pre[lo]) / (double)(hi - lo + 1);
  }
  __syncthreads();
  const double eps = 1e-12;
  if (mode == 0) {
    double mean = block_reduce(sm, buf, OpSum()) / (double)W;
    return sm / (mean + eps);
  }
  if (mode == 3) return sm;
  double mx = block_reduce(act ? sm : -1.0e300, buf, OpMax());
  if (mode == 1) return sm / (mx + eps);
  double mn = block_reduce(act ? sm : 1.0e300, buf, OpMin());
  return (sm - mn) / (mx - mn + eps);
}

__global__ __launch_bounds__(TPB) void block_boundary_kernel(const float* __restrict__ I, const float* __restrict__ H, BoundaryMeta meta,
                                                             dlm_boundary_params p, int32_t* __restrict__ L_out,
                                                             float* __restrict__ S_out, float* __restrict__ margin_out) {
  __shared__ double pre[TPB + 1];
  __shared__ double buf[NW];
  __shared__ int first_neg[NW];
  const int b = blockIdx.x, k = threadIdx.x;
  const int off = meta.win_start[b], W = meta.win_len[b];
  if (meta.cold[b]) {  // first block: conservative cold start
    if (k < W && S_out) S_out[off + k] = 0.f;
    if (k == 0) {
      L_out[b] = min(p.l_min, W);
      if (margin_out) margin_out[b] = __builtin_inff();
    }
    return;
  }
  const bool act = k < W;
  double It = smooth_normalise(act ? (double)I[off + k] : 0.0, k, W, p.smooth_radius, p.norm_mode, pre, buf);
  double Ht = smooth_normalise(act ? (double)H[off + k] : 0.0, k, W, p.smooth_radius, p.norm_mode, pre, buf);
  double S = act ? It - (double)p.lambda * Ht : 0.0;
  if (act && S_out) S_out[off + k] = (float)S;
  double q = S;
  if (p.rule == 1) q = block_scan_inclusive(S, buf);
  // first position whose decision quantity is negative
  unsigned long long neg = __ballot(act && q < 0.0);
  if ((k & 63) == 0) first_neg[k >> 6] = neg ? (k + __ffsll((long long)neg) - 1) : TPB;
  __syncthreads();
  int kstar = TPB;
  for (int i = 0; i < NW; ++i) kstar = min(kstar, first_neg[i]);
  const bool crossed = kstar < W;
  double mrg = block_reduce((act && (!crossed || k <= kstar)) ? fabs(q) : 1.0e300, buf, OpMin());
  if (k == 0) {
    int L_raw = crossed ? kstar : W;
    L_out[b] = min(max(L_raw, p.l_min), W);
    if (margin_out) margin_out[b] = (float)mrg;
  }
}

}  // namespace

void launch_block_boundary(const float* I, const float* H, const BoundaryMeta& meta, int n_seqs, dlm_boundary_params p,
                                int32_t* L_out, float* S_out, float* margin_out, hipStream_t st) {
  block_boundary_kernel<<<n_seqs, TPB, 0, st>>>(I, H, meta, p, L_out, S_out, margin_out);
}
