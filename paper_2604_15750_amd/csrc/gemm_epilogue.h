// Epilogues of a bf16 model's GEMM kernels, on finished values in the accumulator layout of
// v_mfma_f32_16x16x32_f16 (transposed product): in a 16 x 16 output tile, lane ml + 16 g holds
// columns 4g .. 4g+3 of row ml.
#pragma once
#include "common.h"

__device__ inline bf16x4 to_bf16x4(f32x4 v) { return bf16x4{(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]}; }
__device__ inline f16x4 to_f16x4_sat(f32x4 v) { return f16x4{to_f16_sat(v[0]), to_f16_sat(v[1]), to_f16_sat(v[2]), to_f16_sat(v[3])}; }

// 1/rms of rows [m_lo, m_lo + rows) from the producer's partial sums of squares into s_rinv, by the whole workgroup of NT
// threads: sixteen lanes per row, each adding every sixteenth chunk in ascending order, then a fixed butterfly
// (deterministic).  A lane's sixteen loads of a block of 256 chunks are issued together and waited for once: one trip to
// memory per block instead of one per chunk.
template <int NT>
__device__ inline void block_rinv(const RowScale& rs, int m_lo, int rows, float* s_rinv) {
  const int sub = threadIdx.x & 15;
  for (int row = threadIdx.x >> 4; row < rows; row += NT / 16) {
    float ss = 0.f;
    if (rs.ssq) {
      const float* src = rs.ssq + (size_t)(m_lo + row) * rs.nch;
      for (int c0 = 0; c0 < rs.nch; c0 += 256) {
        float v[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
          const int c = c0 + sub + 16 * k;
          v[k] = c < rs.nch ? src[c] : 0.f;
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) ss += v[k];
      }
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    if (sub == 0) s_rinv[row] = rs.ssq ? rsqrtf(ss * rs.inv_d + rs.eps) : 1.f;
  }
}

// block_rinv for a workgroup of NT threads and at most ROWS rows with every load of a thread issued before the first is used
// (one trip to memory): sixteen lanes per row, each adding every sixteenth chunk in ascending order, then the same fixed
// butterfly.  Up to 64 chunks per row in one trip (what the wide-pass producers write); more fall back to block_rinv.
template <int NT, int ROWS>
__device__ inline void block_rinv_batched(const RowScale& rs, int m_lo, int rows, float* s_rinv) {
  if (rs.ssq && rs.nch > 64) { block_rinv<NT>(rs, m_lo, rows, s_rinv); return; }
  constexpr int RPT = (ROWS + NT / 16 - 1) / (NT / 16);  // rows per thread
  const int sub = threadIdx.x & 15;
  float v[RPT][4];
#pragma unroll
  for (int r = 0; r < RPT; ++r) {
    const int row = (threadIdx.x >> 4) + r * (NT / 16);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int c = sub + 16 * k;
      v[r][k] = (rs.ssq && row < rows && c < rs.nch) ? rs.ssq[(size_t)(m_lo + row) * rs.nch + c] : 0.f;
    }
  }
#pragma unroll
  for (int r = 0; r < RPT; ++r) {
    const int row = (threadIdx.x >> 4) + r * (NT / 16);
    float ss = ((v[r][0] + v[r][1]) + v[r][2]) + v[r][3];
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    if (sub == 0 && row < rows) s_rinv[row] = rs.ssq ? rsqrtf(ss * rs.inv_d + rs.eps) : 1.f;
  }
}

// What an epilogue reads from memory besides the product, fetched ahead (at the start of the kernel, while the first weights
// are in flight) for the fragment a wavefront finishes first, so that the end of a short kernel does not wait for a round
// trip: EPI_RESID the four residual values and gains of the lane, EPI_QKV the lane's rotary cosines and sines and, for the
// K and V heads, the row's position and cache slot.
struct EpiAhead {
  f32x4 a, b;
  bool have;
  int pos, slot;  // EPI_QKV, K and V heads: the row's position and cache slot (-1: not fetched)
};
__device__ inline EpiAhead epi_none() { return EpiAhead{f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}, false, -1, -1}; }
template <int EPI>
__device__ inline EpiAhead epi_ahead(const GemmEpi& e, int M, int N, int m, int nc, int g) {
  EpiAhead r = epi_none();
  if (EPI == EPI_RESID) {
    if (m < M && nc < N) {
      r.a = *(const f32x4*)(e.h + (size_t)m * N + nc + 4 * g);
      r.b = *(const f32x4*)(e.gain + nc + 4 * g);
      r.have = true;
    }
  } else if (EPI == EPI_QKV) {
    const int hd = e.hd, half = hd >> 1;
    if (m < M && nc < N && g < 2) {
      const int head = nc / hd;
      if (head < e.n_q + e.n_kv) {
        const int i = 8 * ((nc % hd) >> 4) + 4 * g;
        r.a = *(const f32x4*)(e.rope_cos + (size_t)m * half + i);
        r.b = *(const f32x4*)(e.rope_sin + (size_t)m * half + i);
        r.have = true;
      }
      if (head >= e.n_q) {
        r.pos = e.row_pos[m];
        r.slot = e.row_slot[m];
      }
    }
  }
  return r;
}

// Rotary pair group: a = packed columns nc+4gp .. +3 of a 16-column tile starting at packed column nc,
// b = the same + 8; they are dims i .. i+3 and i+half .. i+half+3 of one head (weights packed with PERM_ROTARY).
__device__ inline void finish_qkv(const GemmEpi& e, int m, int nc, int gp, f32x4 a, f32x4 b, const EpiAhead ahead = epi_none()) {
  const int hd = e.hd, half = hd >> 1;
  const int head = nc / hd, i = 8 * ((nc % hd) >> 4) + 4 * gp;
  if (head < e.n_q + e.n_kv) {
    const bool pre = ahead.have;
    const f32x4 c = pre ? ahead.a : *(const f32x4*)(e.rope_cos + (size_t)m * half + i);
    const f32x4 sn = pre ? ahead.b : *(const f32x4*)(e.rope_sin + (size_t)m * half + i);
    const f32x4 ra = a * c - b * sn, rb = b * c + a * sn;
    a = ra;
    b = rb;
  }
  const f16x4 ab = to_f16x4_sat(a), bb = to_f16x4_sat(b);
  if (head < e.n_q) {
    f16_t* dst = e.q + (size_t)m * e.n_q * hd + (size_t)head * hd;
    *(f16x4*)(dst + i) = ab;
    *(f16x4*)(dst + i + half) = bb;
    return;
  }
  const bool is_k = head < e.n_q + e.n_kv;
  const int kvh = is_k ? head - e.n_q : head - e.n_q - e.n_kv;
  // (a load here, between the stores of two fragments, has to wait for every store before it: the memory counter retires in order)
  const int pos = ahead.pos >= 0 ? ahead.pos : e.row_pos[m];
  const int slot = ahead.pos >= 0 ? ahead.slot : e.row_slot[m];
  f16_t* dst = (is_k ? e.kcache : e.vcache) + (size_t)slot * e.slot_stride + (size_t)kvh * e.head_stride;
  if (is_k) {  // four consecutive dims share a lane slot of the K tiling
    *(f16x4*)(dst + kv_k_index(pos, i, hd)) = ab;
    *(f16x4*)(dst + kv_k_index(pos, i + half, hd)) = bb;
  } else {
    // dims i .. i+3 (i a multiple of 4) lie in one 16-dim tile: consecutive dims are 8 elements apart (kv_v_index)
    const size_t va = kv_v_index(pos, i, hd), vb = kv_v_index(pos, i + half, hd);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      dst[va + 8 * j] = ab[j];
      dst[vb + 8 * j] = bb[j];
    }
  }
}

// gate = packed columns nc+4gp .. +3, up = the same + 8: output columns 8 (nc/16) + 4gp .. +3 (weights packed with PERM_GATED)
__device__ inline void finish_swiglu(const GemmEpi& e, int m, int nc, int gp, f32x4 g, f32x4 u) {
  f32x4 a;
#pragma unroll
  for (int t = 0; t < 4; ++t) a[t] = g[t] * __builtin_amdgcn_rcpf(1.f + __expf(-g[t])) * u[t];  // (the hardware reciprocal: 1 ulp)
  *(op4*)(e.act + tile_index(m, 8 * (nc >> 4) + 4 * gp, e.ffn)) = to_f16x4_sat(a);
}

// residual add and next norm's x for columns n .. n+3 of row m; returns the four columns' share of sum h^2
__device__ inline float finish_resid(const GemmEpi& e, int m, int n, int N, f32x4 y, const EpiAhead ahead = epi_none()) {
  const size_t o = (size_t)m * N + n;
  const bool pre = ahead.have;
  const f32x4 v = (pre ? ahead.a : *(const f32x4*)(e.h + o)) + y;
  *(f32x4*)(e.h + o) = v;
  const f32x4 g = pre ? ahead.b : *(const f32x4*)(e.gain + n);
  *(op4*)(e.x + tile_index(m, n, N)) = to_f16x4_sat(v * g);
  return v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
}

__device__ inline void finish_sum(const GemmEpi& e, int m, int n, int N, f32x4 v) {
  const size_t o = (size_t)m * N + n;
  if (e.out_bf16) *(bf16x4*)(e.out_bf16 + o) = to_bf16x4(v);
  else *(f32x4*)(e.out_f32 + o) = v;
}

// One 16 x 16 tile starting at packed column nc: v = this lane's four finished columns of row m, rinv = 1/rms of the input row.
// Called by all 64 lanes of a wavefront together (it exchanges values between lanes).  EPI_RESID returns the tile's share of
// sum h^2 of row m (in every lane of the row), the others 0.
template <int EPI>
__device__ inline float finish_frag(const GemmEpi& e, int M, int N, int m, int nc, int g, f32x4 v, float rinv, const EpiAhead ahead = epi_none()) {
  if (EPI == EPI_QKV || EPI == EPI_SWIGLU) {
    f32x4 b;  // the partner group, columns + 8, sits 32 lanes up
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = __shfl_xor(v[i], 32, 64);
    if (g < 2 && m < M) {
      if (EPI == EPI_QKV) finish_qkv(e, m, nc, g, v * rinv, b * rinv, ahead);
      else finish_swiglu(e, m, nc, g, v * rinv, b * rinv);
    }
    return 0.f;
  }
  if (EPI == EPI_RESID) {
    float ss = m < M ? finish_resid(e, m, nc + 4 * g, N, v, ahead) : 0.f;
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    return ss;
  }
  if (m < M) finish_sum(e, m, nc + 4 * g, N, v * rinv);
  return 0.f;
}
