// CAP-Decoding (paper Sec. 4.3, Eq. 5-6, Alg. 1) and the token write of Eq. 2.
// One workgroup per sequence, one lane per block row (block <= 256 rows).  The pairwise conflict
// scores are gathered straight from the logits (two scalars per pooled pair), kept as a bit matrix
// in LDS; the confidence order is found by counting; the greedy pass is a short sequential walk
// over bit masks.
#include "common.h"

namespace {

constexpr int TPB = 256;
constexpr int WORDS = TPB / 32;
constexpr float INF = __builtin_inff();

__device__ inline float block_min(float v, float* buf) {
  v = -wave_max(-v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = buf[0];
  for (int i = 1; i < TPB / 64; ++i) r = fminf(r, buf[i]);
  return r;
}

// position of row i in the order (descending conf, ascending row) among rows with member[j] != 0
__device__ inline int rank_among(int i, int L, const float* c, const uint8_t* member) {
  int r = 0;
  const float ci = c[i];
  for (int j = 0; j < L; ++j)
    if (member[j] && (c[j] > ci || (c[j] == ci && j < i))) ++r;
  return r;
}

template <typename T>
__global__ __launch_bounds__(TPB) void select_kernel(const T* __restrict__ logits, int vocab, const float* __restrict__ lse_g,
                                                     const float* __restrict__ conf_g, const int32_t* __restrict__ argmax_g,
                                                     int32_t* __restrict__ tokens, SelectMeta meta, int mask_id, dlm_select_params p,
                                                     int apply, uint8_t* __restrict__ sel_out, int32_t* __restrict__ nsel_out,
                                                     float* __restrict__ margin_out) {
  __shared__ float c[TPB], lse[TPB], fbuf[TPB / 64];
  __shared__ int yh[TPB], order[TPB];
  __shared__ uint8_t elig[TPB], pool[TPB], alive[TPB], sel[TPB];
  __shared__ uint32_t bits[TPB][WORDS];
  __shared__ int n_alive, n_sel, top_row, second_row;

  const int b = blockIdx.x, i = threadIdx.x;
  const int row0 = meta.row_start[b], tok0 = meta.tok_start[b], L = meta.block_len[b];
  const bool act = i < L;
  float margin = INF;

  c[i] = act ? conf_g[row0 + i] : -1.f;
  lse[i] = act ? lse_g[row0 + i] : 0.f;
  yh[i] = act ? min(max(argmax_g[row0 + i], 0), vocab - 1) : 0;  // a caller-supplied prediction outside the vocabulary is clamped into it
  elig[i] = act && tokens[tok0 + i] == mask_id;
  sel[i] = 0;
  alive[i] = 0;
  for (int w = 0; w < WORDS; ++w) bits[i][w] = 0;
  if (i == 0) { n_alive = 0; n_sel = 0; top_row = -1; second_row = -1; }
  __syncthreads();

  // most confident eligible row and the runner-up (for the safeguard and modes 1, 2)
  if (elig[i]) {
    int r = rank_among(i, L, c, elig);
    if (r == 0) top_row = i;
    if (r == 1) second_row = i;
  }
  __syncthreads();
  float top_gap = INF;
  if (top_row >= 0 && second_row >= 0 && c[top_row] != c[second_row]) top_gap = c[top_row] - c[second_row];

  if (p.mode == 0) {
    if (elig[i]) margin = fminf(fabsf(c[i] - p.tau_low), fabsf(c[i] - p.tau_high));
    pool[i] = elig[i] && c[i] >= p.tau_low;
    __syncthreads();
    // conflict bit matrix over pooled pairs (Eq. 6), each unordered pair once
    for (int pr = i; pr < L * L; pr += TPB) {
      int a = pr / L, d = pr - a * L;
      if (a < d && pool[a] && pool[d]) {
        float la = to_f32(logits[(size_t)(row0 + a) * vocab + yh[d]]) - lse[a];
        float ld = to_f32(logits[(size_t)(row0 + d) * vocab + yh[a]]) - lse[d];
        float D = la + ld;
        margin = fminf(margin, fabsf(D - p.gamma));
        if (D > p.gamma) {
          atomicOr(&bits[a][d >> 5], 1u << (d & 31));
          atomicOr(&bits[d][a >> 5], 1u << (a & 31));
        }
      }
    }
    __syncthreads();
    // phase 1: every pooled row with conf >= tau_high; drop their conflicts from the pool
    const bool high = pool[i] && c[i] >= p.tau_high;
    if (high) sel[i] = 1;
    __syncthreads();
    bool dropped = false;
    if (pool[i] && !high)
      for (int j = 0; j < L; ++j)
        if (sel[j] && (bits[j][i >> 5] >> (i & 31) & 1u)) { dropped = true; break; }
    alive[i] = pool[i] && !high && !dropped;
    __syncthreads();
    // phase 2 order: descending conf, ties by row
    if (alive[i]) {
      order[rank_among(i, L, c, alive)] = i;
      atomicAdd(&n_alive, 1);
    }
    __syncthreads();
    if (i + 1 < n_alive) {
      float g = c[order[i]] - c[order[i + 1]];
      if (g != 0.f) margin = fminf(margin, g);
    }
    if (i == 0) {
      for (int r = 0; r < n_alive; ++r) {
        int a = order[r];
        if (!alive[a]) continue;
        sel[a] = 1;
        alive[a] = 0;
        for (int j = 0; j < L; ++j)
          if (bits[a][j >> 5] >> (j & 31) & 1u) alive[j] = 0;
      }
    }
    __syncthreads();
  } else if (p.mode == 1) {
    if (elig[i]) {
      margin = fabsf(c[i] - p.tau_high);
      sel[i] = c[i] >= p.tau_high;
    }
    __syncthreads();
  }
  if (sel[i]) atomicAdd(&n_sel, 1);
  __syncthreads();
  if (n_sel == 0 && top_row >= 0) {  // safeguard / top-1 rule: the most confident eligible row
    margin = fminf(margin, top_gap);
    if (i == top_row) sel[i] = 1;
  }
  __syncthreads();
  if (act) {
    sel_out[row0 + i] = sel[i];
    if (apply && sel[i]) tokens[tok0 + i] = yh[i];
  }
  float m = block_min(margin, fbuf);
  if (i == 0) {
    nsel_out[b] = n_sel ? n_sel : (top_row >= 0 ? 1 : 0);
    if (margin_out) margin_out[b] = m;
  }
}

}  // namespace

template <typename T>
void launch_select(const T* logits, int vocab, const float* lse, const float* conf, const int32_t* argmax, int32_t* tokens,
                        const SelectMeta& meta, int n_seqs, int mask_id, dlm_select_params p, int apply, uint8_t* sel,
                        int32_t* nsel, float* margin, hipStream_t st) {
  select_kernel<T><<<n_seqs, TPB, 0, st>>>(logits, vocab, lse, conf, argmax, tokens, meta, mask_id, p, apply, sel, nsel, margin);
}
template void launch_select<float>(const float*, int, const float*, const float*, const int32_t*, int32_t*, const SelectMeta&, int,
                                        int, dlm_select_params, int, uint8_t*, int32_t*, float*, hipStream_t);
template void launch_select<bf16_t>(const bf16_t*, int, const float*, const float*, const int32_t*, int32_t*, const SelectMeta&, int,
                                         int, dlm_select_params, int, uint8_t*, int32_t*, float*, hipStream_t);
