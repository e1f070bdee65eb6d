// GEMM of a bf16 model  Y[M,N] = X[M,K] * W[N,K]^T  on the gfx950 matrix cores (operands in IEEE half, see op_t in common.h):
// operand tiling and the choice of kernel.
//
// At decode shapes (M = 8 .. 384 rows against 15 GB of weights per pass) the GEMMs are bound by
// streaming W from HBM, so both kernels are weight streamers that happen to multiply:
//   * W is re-tiled once, when the model is created, into 1 KiB fragments (16 rows x 32 k) that are
//     exactly the A operand of v_mfma_f32_16x16x32_f16: a wavefront fetches a fragment as 64
//     consecutive 16-byte loads and walks a contiguous run of HBM along K; W goes HBM -> registers;
//   * activations live in the same fragment tiling (B operand), written that way by their producer;
//   * the product is computed transposed (W fragment = A operand), so a lane ends up with four
//     consecutive output columns of one row.
// gemm_skinny.hip serves M <= 64 (except the LM head), gemm_mid.hip a block with its look-ahead window (65 .. 160 rows, all
// of them in one workgroup), gemm_macro.hip (both operands through LDS, large output tiles: bound by the matrix cores, not
// by W) wide passes, gemm_tiled.hip what is left (choose_kernel below); the layer's row-wise glue runs in their epilogues
// (gemm_epilogue.h):
//   QKV     1/rms of the input row, rotary embedding, Q row-major, K and V into the tiled KV cache
//   SWIGLU  1/rms, silu(gate) * up into the fragment tiling of the down projection
//   RESID   residual add, x = h * gain of the next RMSNorm into fragment tiling, and the share of
//           sum(h^2) per row of each column tile
//   SUM / DIRECT  the product (optionally scaled by 1/rms per row) to bf16 or fp32
// W_qkv and W_gate_up are packed with their rows permuted (weight_source_row) so that a rotary pair,
// or a gate column and its up column, sit 8 columns apart in one 16-column tile.
#include "common.h"

namespace {

// W [N, K] row-major -> fragment tiles, `pr` row-tiles interleaved along k, rows permuted by (perm, param).
__device__ inline op8 to_op8(bf16x8 v) {
  op8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = to_f16_sat((float)v[i]);
  return r;
}

__global__ void pack_weight_kernel(const bf16x8* __restrict__ w, op8* __restrict__ out, int N, int K, int pr, int perm, int param) {
  const int KT = K >> 5;
  const size_t total = (size_t)(N >> 4) * KT * 64;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int lane = idx & 63;
    const size_t tile = idx >> 6;
    const int sub = tile % pr;
    const size_t rest = tile / pr;
    const int t = rest % KT;
    const int grp = rest / KT;
    const int n = weight_source_row((grp * pr + sub) * 16 + (lane & 15), perm, param);
    const int k8 = t * 4 + (lane >> 4);
    out[idx] = to_op8(w[(size_t)n * (K >> 3) + k8]);
  }
}

__global__ void pack_weight_steps_kernel(const bf16x8* __restrict__ w, op8* __restrict__ out, int N, int K, int ct, int nwv, int perm, int param) {
  const int KT = K >> 5, G = N / (16 * ct), per = KT / nwv;
  const size_t total = (size_t)(N >> 4) * KT * 64;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int lane = idx & 63;
    size_t f = idx >> 6;
    const int r = f % ct; f /= ct;
    const int wv = f % nwv; f /= nwv;
    const int grp = f % G;
    const int s = (int)(f / G);
    const int n = weight_source_row((grp * ct + r) * 16 + (lane & 15), perm, param);
    const int k8 = (wv * per + s) * 4 + (lane >> 4);
    out[idx] = to_op8(w[(size_t)n * (K >> 3) + k8]);
  }
}

// X [M, K] row-major -> fragment tiles [ceil(M/16)][K/32]; rows beyond M are zero.
__global__ void pack_act_kernel(const bf16x8* __restrict__ x, op8* __restrict__ out, int M, int K) {
  const int KT = K >> 5;
  const size_t total = (size_t)((M + 15) >> 4) * KT * 64;
  const op8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int lane = idx & 63;
    const size_t tile = idx >> 6;
    const int t = tile % KT;
    const int m = (int)(tile / KT) * 16 + (lane & 15);
    out[idx] = m < M ? to_op8(x[(size_t)m * (K >> 3) + t * 4 + (lane >> 4)]) : zero8;
  }
}

// Which kernel serves a shape (measured crossovers on the layer shapes of 7 .. 8 B models):
//   skinny  up to 64 rows: nothing crosses workgroups, every wavefront streams W;
//   mid     65 .. 160 rows (narrow matrices to 256, O and down to 208); and below that where its wider column groups pay: from 17 rows for
//           wide matrices (QKV, gate/up) and for narrow ones whose K is long enough for a four-way split (down) - there
//           the skinny kernel's re-reads of X by every 16- or 32-column group cost more than W itself - and at any row
//           count when its 96-column groups are exactly one per compute unit (gate/up of an 8B model), or when the skinny
//           kernel would need a second round for a few column tiles (QKV of a 7B model with grouped-query heads);
//   macro   more rows than that when the matrix has enough 128 x 256 tiles of its own (wide from 161 rows, narrow from 257);
//   tiled   the rest, and the LM head up to 64 rows (no workspace: no K split), with or without the statistics epilogue.
enum { KERNEL_SKINNY, KERNEL_MID, KERNEL_MACRO, KERNEL_TILED };
int choose_kernel(int M, int N, int K, int kind) {
  if (kind == EPI_STATS) return KERNEL_TILED;  // only the tiled kernel has that epilogue (the caller keeps to GEMM_STATS_MAX_ROWS rows)
  const int pr = weight_pack_rows(N);
  const bool whole_groups = N % (16 * pr) == 0;
  if (M <= GEMM_SKINNY_MAX_ROWS && kind != EPI_DIRECT && whole_groups) {
    if (pr == 2 && (M > 16 || gemm_mid_fills_chip(M, N, K))) return KERNEL_MID;
    if (pr == 1 && M > 16 && K >= 8192) return KERNEL_MID;
    // a narrow matrix with a few more than 256 column tiles: the skinny kernel's one-tile workgroups would run a second,
    // nearly empty round over the compute units; 32-column groups fit in one
    if (pr == 1 && M <= 16 && (N >> 4) > 256 && (N >> 4) <= 384) return KERNEL_MID;
    return KERNEL_SKINNY;
  }
  // narrow matrices: to 256 rows, except that the residual projections, which have the macro kernel to go to, leave the mid
  // kernel where it starts to lose to it (measured: O and down both from 224 rows)
  const int mid_rows = pr == 2 ? GEMM_MID_MAX_ROWS : kind != EPI_RESID ? GEMM_MID_MAX_ROWS_NARROW : 208;
  if (M > GEMM_SKINNY_MAX_ROWS && M <= mid_rows && whole_groups) return KERNEL_MID;
  // EPI_RESID has no instantiation of the tiled kernel: what the mid kernel does not take goes to the macro kernel
  if (M > GEMM_MACRO_MIN_ROWS_NARROW || (M > GEMM_SKINNY_MAX_ROWS && N > 8192) || kind == EPI_RESID) return KERNEL_MACRO;
  return KERNEL_TILED;
}

}  // namespace

void launch_pack_weight(const bf16_t* w, op_t* out, int N, int K, int perm, int perm_param, hipStream_t st) {
  pack_weight_kernel<<<2048, 256, 0, st>>>((const bf16x8*)w, (op8*)out, N, K, weight_pack_rows(N), perm, perm_param);
}
void launch_pack_weight_steps(const bf16_t* w, op_t* out, int N, int K, int ct, int perm, int perm_param, hipStream_t st) {
  pack_weight_steps_kernel<<<2048, 256, 0, st>>>((const bf16x8*)w, (op8*)out, N, K, ct, ct == 1 ? 8 : 4, perm, perm_param);
}
int gemm_bf16_steps_ct(int N, int K, int kind) {
  switch (choose_kernel(16, N, K, kind)) {
    case KERNEL_MID: return gemm_mid_steps_ct(N, K);
    case KERNEL_SKINNY: {  // one column tile and 8 wavefronts per workgroup, or a pair of tiles and 4
      const int pr = weight_pack_rows(N);
      return ((K >> 5) % (pr == 1 ? 8 : 4) == 0 && N % (16 * pr) == 0) ? pr : 0;
    }
    default: return 0;
  }
}
void launch_pack_act(const bf16_t* x, op_t* out, int M, int K, hipStream_t st) {
  pack_act_kernel<<<512, 256, 0, st>>>((const bf16x8*)x, (op8*)out, M, K);
}

int gemm_bf16_splits(int M, int N, int K, int kind) {
  switch (choose_kernel(M, N, K, kind)) {
    case KERNEL_MID: return gemm_mid_splits(M, N, K);
    case KERNEL_MACRO: return gemm_macro_splits(M, N, K);
    case KERNEL_TILED: return gemm_tiled_splits(M, N, K);
    default: return 1;
  }
}
int gemm_bf16_ssq_chunks(int M, int N, int K) {
  switch (choose_kernel(M, N, K, EPI_RESID)) {
    case KERNEL_SKINNY: return N >> 4;
    case KERNEL_MID: return gemm_mid_ssq_chunks(M, N, K);
    case KERNEL_MACRO: return gemm_macro_ssq_chunks(M, N, K);
    default: return gemm_tiled_ssq_chunks(M, N);
  }
}
int gemm_bf16_stat_parts(int M, int N) { return gemm_tiled_stat_parts(M, N); }
int gemm_bf16_counters(int max_rows, int max_n) {
  const int a = gemm_tiled_counters(max_rows, max_n), b = gemm_mid_counters(max_n), c = gemm_macro_counters(max_rows, max_n);
  return a > b ? (a > c ? a : c) : (b > c ? b : c);
}

void launch_gemm_bf16(const op_t* xt, const op_t* wt, int M, int N, int K, const GemmEpi& e, hipStream_t st) {
  switch (choose_kernel(M, N, K, e.kind)) {
    case KERNEL_SKINNY: launch_gemm_skinny(xt, wt, weight_pack_rows(N), M, N, K, e, st); break;
    case KERNEL_MID: launch_gemm_mid(xt, wt, M, N, K, e, st); break;
    case KERNEL_MACRO: launch_gemm_macro(xt, wt, M, N, K, e, st); break;
    default: launch_gemm_tiled(xt, wt, M, N, K, e, st); break;
  }
}
