// Block-vs-prefix attention on the matrix cores for a bf16 model's KV cache: the work of one workgroup on one
// (16-query tile, head, sequence), as a device function of its own so that it can be placed inside another kernel.
// (Running it in the tail of the QKV GEMM of a narrow pass, in the workgroup that finishes a head last, was measured: the
// fused launch took 37 us against 23 + 9 us for the two launches, because the tail is a serial chain of memory round trips.)
//
// The KV cache of a bf16 model holds IEEE half (f16_t in common.h: Q, K, V and the unnormalised probabilities are the
// matrix-core operands here, and with bf16's 8 mantissa bits their rounding is the largest single part of a deep model's
// logit error; half has the same size and matrix-core rate).  It is kept per (slot, kv head) in matrix-core fragment tiles
// (kv_k_index / kv_v_index), so a wavefront fetches a K operand (16 keys x 32 dims) or a V^T operand
// (16 dims x 32 keys) as 64 consecutive 16-byte pieces.  The NWV wavefronts of the workgroup take
// every NWV-th block of 32 keys with their own online-softmax state and are merged through LDS.
// The K and V fragments of a wavefront's next block are in flight while the current one is
// multiplied.  S^T = K Q^T puts 8 keys of one query in each lane (the lane's query is lane%16 in
// both S^T and O^T), so the probabilities feed the second product straight from registers: the V
// tiling stores keys in the order the first product emits them.
#pragma once
#include "common.h"

template <int HD, int NWV, int DS = 1>
struct AttnLds {  // merge buffers of one workgroup (HD / DS of the head's dims)
  float sm[NWV][16], sl[NWV][16];
  float so[NWV][HD / DS][17];
};

// q: row-major [rows, n_q * HD]; kt / vt: the (slot, kv head) region of the tiled cache; rows [row0, row_end) x head `head`
// against keys [0, n_keys); output to out_tiles (fragment tiles [rows, n_q * HD] in half: the O projection's input) if given,
// else to out_rows (row-major bf16).  Called by every thread of a workgroup of NWV wavefronts.
// DS > 1: the workgroup produces only dims [dpart * HD / DS, (dpart + 1) * HD / DS) of the output: it reads all of K (the
// scores and the softmax are computed by each of the DS workgroups of a head, identically) but only its share of V.  What
// bounds a narrow pass is what one compute unit can pull through its L2 (about 50 GB/s), and K and V of a head are its whole
// traffic: four workgroups per head move 5/8 of it each, with nothing to merge.
template <int HD, int NWV, int DS = 1>
__device__ inline void attention_tile(const f16_t* __restrict__ q, const f16_t* __restrict__ kregion, const f16_t* __restrict__ vregion,
                                      int row0, int row_end, int n_keys, int head, int n_q, op_t* __restrict__ out_tiles, bf16_t* __restrict__ out_rows,
                                      AttnLds<HD, NWV, DS>& L, int dpart = 0) {
  constexpr int KS = HD / 32, DT = HD / 16 / DS, HDP = HD / DS;
  static_assert(HDP * 16 >= NWV * 64, "every thread finishes at least one dim");
  constexpr float NEG_BIG = -3.0e38f;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, c = lane & 15;
  const float scale = rsqrtf((float)HD);
  const f16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  f16x8 qf[KS];
  {
    const int r = row0 + c;
#pragma unroll
    for (int t = 0; t < KS; ++t)
      qf[t] = r < row_end ? *(const f16x8*)(q + (size_t)r * n_q * HD + (size_t)head * HD + 32 * t + 8 * g) : zero8;
  }
  const f16x8* kt = (const f16x8*)kregion + lane;
  const f16x8* vt = (const f16x8*)vregion + lane;
  float m = NEG_BIG, l = 0.f;
  f32x4 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nblk = (n_keys + 31) >> 5;
  f16x8 kf[2][2 * KS], vf[2][DT];
  auto load = [&](int buf, int blk) {  // blk may lie beyond the keys: nothing is fetched then
    const bool ok = blk < nblk;
#pragma unroll
    for (int t = 0; t < 2 * KS; ++t) kf[buf][t] = ok ? kt[((size_t)blk * 2 * KS + t) * 64] : zero8;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) vf[buf][dt] = ok ? vt[((size_t)blk * (DT * DS) + dpart * DT + dt) * 64] : zero8;
  };
  auto step = [&](int buf, int blk) {
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < KS; ++t) {
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[buf][t], qf[t], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[buf][KS + t], qf[t], s1, 0, 0, 0);
    }
    // lane holds, for query c, keys blk*32 + 4g + i (s0) and + 16 (s1)
    const int key0 = blk * 32 + 4 * g;
    float sv[8];
    bool ok[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ok[i] = key0 + i < n_keys;
      ok[4 + i] = key0 + 16 + i < n_keys;
      sv[i] = ok[i] ? s0[i] * scale : NEG_BIG;
      sv[4 + i] = ok[4 + i] ? s1[i] * scale : NEG_BIG;
    }
    float mx = sv[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) mx = fmaxf(mx, sv[i]);
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float mn = fmaxf(m, mx);
    const float corr = __expf(m - mn);
    float pv[8], ps = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pv[i] = ok[i] ? __expf(sv[i] - mn) : 0.f;
      ps += pv[i];
    }
    ps += __shfl_xor(ps, 16, 64);
    ps += __shfl_xor(ps, 32, 64);
    l = l * corr + ps;
    m = mn;
    const f16x8 pb = {(f16_t)pv[0], (f16_t)pv[1], (f16_t)pv[2], (f16_t)pv[3], (f16_t)pv[4], (f16_t)pv[5], (f16_t)pv[6], (f16_t)pv[7]};  // in [0, 1]
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      o[dt] *= corr;
      o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf[buf][dt], pb, o[dt], 0, 0, 0);
    }
  };
  load(0, wave);
  for (int blk = wave; blk < nblk; blk += 2 * NWV) {
    load(1, blk + NWV);
    step(0, blk);
    load(0, blk + 2 * NWV);
    if (blk + NWV < nblk) step(1, blk + NWV);
  }
  // merge the wavefronts
  if (g == 0) { L.sm[wave][c] = m; L.sl[wave][c] = l; }
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int i = 0; i < 4; ++i) L.so[wave][16 * dt + 4 * g + i][c] = o[dt][i];
  __syncthreads();
  constexpr int CH = HDP * 16 / (NWV * 64);  // each thread finishes CH consecutive dims of one query
  const int qi = tid & 15, d0 = (tid >> 4) * CH;
  float M = L.sm[0][qi];
#pragma unroll
  for (int wv = 1; wv < NWV; ++wv) M = fmaxf(M, L.sm[wv][qi]);
  float w[NWV], Lsum = 0.f;
#pragma unroll
  for (int wv = 0; wv < NWV; ++wv) { w[wv] = __expf(L.sm[wv][qi] - M); Lsum += w[wv] * L.sl[wv][qi]; }
  const int r = row0 + qi;
  if (r < row_end) {
    const int width = n_q * HD;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const int d = d0 + j;
      float acc = 0.f;
#pragma unroll
      for (int wv = 0; wv < NWV; ++wv) acc += w[wv] * L.so[wv][d][qi];
      const int col = head * HD + dpart * HDP + d;
      const float v = acc / Lsum;
      if (out_tiles) out_tiles[tile_index(r, col, width)] = to_f16_sat(v);
      else out_rows[(size_t)r * width + col] = (bf16_t)v;
    }
  }
  __syncthreads();  // the merge buffers may be reused
}
