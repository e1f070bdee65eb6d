// Block-vs-prefix attention: every row of a sequence's span attends, without causal mask, to keys
// [0, n_keys) of the sequence's KV-cache slot (cached prefix + the span's own rows, which the
// rotary/KV kernel has already written there).  Grouped-query heads share K/V.
//
// fp32 kernel (head_dim 32/64/128, row-major cache [pos][n_kv*hd]): one workgroup per (16-query
// tile, head, sequence); keys are streamed in tiles through LDS with an online softmax in fp32.
#include "common.h"

namespace {

constexpr int QT = 16;        // query rows per workgroup
constexpr int KTILE = 32;     // keys per LDS tile
constexpr float NEG_BIG = -3.0e38f;

template <typename T, int HD>
__global__ __launch_bounds__(256) void attention_kernel(const T* __restrict__ q, const T* __restrict__ kcache, const T* __restrict__ vcache,
                                                        size_t slot_stride, AttnMeta meta, T* __restrict__ out, bool out_tiled, int n_q,
                                                        int n_kv) {
  __shared__ float qs[QT][HD];
  __shared__ float ks[KTILE][HD + 1];
  __shared__ float vs[KTILE][HD];
  __shared__ float ps[QT][KTILE];
  constexpr int EPT = HD / 16;  // output elements per thread

  const int b = blockIdx.z, head = blockIdx.y;
  const int row0 = meta.row_off[b] + blockIdx.x * QT;
  const int row_end = meta.row_off[b + 1];
  if (row0 >= row_end) return;
  const int n_keys = meta.n_keys[b];
  const int kvh = head / (n_q / n_kv);
  const size_t kv_row = (size_t)n_kv * HD;
  const T* kbase = kcache + (size_t)meta.slot[b] * slot_stride + (size_t)kvh * HD;
  const T* vbase = vcache + (size_t)meta.slot[b] * slot_stride + (size_t)kvh * HD;
  const int tid = threadIdx.x, qi = tid >> 4, lx = tid & 15;
  const float scale = rsqrtf((float)HD);

  for (int i = tid; i < QT * HD; i += 256) {
    const int r = i / HD, e = i % HD;
    qs[r][e] = (row0 + r < row_end) ? to_f32(q[(size_t)(row0 + r) * n_q * HD + (size_t)head * HD + e]) * scale : 0.f;
  }
  float m = NEG_BIG, l = 0.f, o[EPT];
#pragma unroll
  for (int n = 0; n < EPT; ++n) o[n] = 0.f;

  for (int k0 = 0; k0 < n_keys; k0 += KTILE) {
    __syncthreads();
    for (int i = tid; i < KTILE * HD; i += 256) {
      const int kk = i / HD, e = i % HD;
      const bool ok = k0 + kk < n_keys;
      ks[kk][e] = ok ? to_f32(kbase[(size_t)(k0 + kk) * kv_row + e]) : 0.f;
      vs[kk][e] = ok ? to_f32(vbase[(size_t)(k0 + kk) * kv_row + e]) : 0.f;
    }
    __syncthreads();
    // scores: thread (qi, lx) handles keys lx and lx + 16
    float s0 = 0.f, s1 = 0.f;
#pragma unroll 8
    for (int e = 0; e < HD; ++e) {
      const float qv = qs[qi][e];
      s0 = fmaf(qv, ks[lx][e], s0);
      s1 = fmaf(qv, ks[lx + 16][e], s1);
    }
    if (k0 + lx >= n_keys) s0 = NEG_BIG;
    if (k0 + lx + 16 >= n_keys) s1 = NEG_BIG;
    float tm = fmaxf(s0, s1);
#pragma unroll
    for (int ofs = 8; ofs > 0; ofs >>= 1) tm = fmaxf(tm, __shfl_xor(tm, ofs, 64));
    const float mn = fmaxf(m, tm);
    const float corr = __expf(m - mn);
    const float p0 = (k0 + lx < n_keys) ? __expf(s0 - mn) : 0.f;
    const float p1 = (k0 + lx + 16 < n_keys) ? __expf(s1 - mn) : 0.f;
    float ts = p0 + p1;
#pragma unroll
    for (int ofs = 8; ofs > 0; ofs >>= 1) ts += __shfl_xor(ts, ofs, 64);
    l = l * corr + ts;
    m = mn;
    ps[qi][lx] = p0;
    ps[qi][lx + 16] = p1;
    __syncthreads();
#pragma unroll
    for (int n = 0; n < EPT; ++n) o[n] *= corr;
    for (int kk = 0; kk < KTILE; ++kk) {
      const float p = ps[qi][kk];
#pragma unroll
      for (int n = 0; n < EPT; ++n) o[n] = fmaf(p, vs[kk][lx + 16 * n], o[n]);
    }
  }
  const int r = row0 + qi;
  if (r < row_end) {
    const int width = n_q * HD;
#pragma unroll
    for (int n = 0; n < EPT; ++n) {
      const int col = head * HD + lx + 16 * n;
      const size_t idx = out_tiled ? Act<T>::idx(r, col, width) : (size_t)r * width + col;
      out[idx] = from_f32<T>(o[n] / l);
    }
  }
}

// ---- bf16 kernel on the matrix cores --------------------------------------------------------------
// The bf16 KV cache is kept per (slot, kv head) in matrix-core fragment tiles (kv_k_index /
// kv_v_index), so a wavefront fetches a K operand (16 keys x 32 dims) or a V^T operand
// (16 dims x 32 keys) as 64 consecutive 16-byte pieces.  One workgroup per (16-query tile, head,
// sequence); its NWV wavefronts take every NWV-th block of 32 keys with their own online-softmax
// state and are merged through LDS.  The K and V fragments of a wavefront's next block are in flight
// while the current one is multiplied.  S^T = K Q^T puts 8 keys of one query in each lane (the lane's
// query is lane%16 in both S^T and O^T), so the probabilities feed the second product straight
// from registers: the V tiling stores keys in the order the first product emits them.
// A decode pass has few (query tile, head) pairs, so it runs 8 wavefronts per workgroup to shorten
// each wavefront's chain of dependent loads; wide passes (prefill, batches) run 4.
template <int HD, int NWV>
__global__ __launch_bounds__(NWV * 64) void attention_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ kcache,
                                                                  const bf16_t* __restrict__ vcache, size_t slot_stride, size_t head_stride,
                                                                  AttnMeta meta, bf16_t* __restrict__ out, bool out_tiled, int n_q, int n_kv) {
  constexpr int KS = HD / 32, DT = HD / 16;
  __shared__ float sm[NWV][16], sl[NWV][16];
  __shared__ float so[NWV][HD][17];

  const int b = blockIdx.z, head = blockIdx.y;
  const int row0 = meta.row_off[b] + blockIdx.x * 16;
  const int row_end = meta.row_off[b + 1];
  if (row0 >= row_end) return;
  const int n_keys = meta.n_keys[b];
  const int kvh = head / (n_q / n_kv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, c = lane & 15;
  const float scale = rsqrtf((float)HD);
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  bf16x8 qf[KS];
  {
    const int r = row0 + c;
#pragma unroll
    for (int t = 0; t < KS; ++t)
      qf[t] = r < row_end ? *(const bf16x8*)(q + (size_t)r * n_q * HD + (size_t)head * HD + 32 * t + 8 * g) : zero8;
  }
  const bf16x8* kt = (const bf16x8*)(kcache + (size_t)meta.slot[b] * slot_stride + (size_t)kvh * head_stride) + lane;
  const bf16x8* vt = (const bf16x8*)(vcache + (size_t)meta.slot[b] * slot_stride + (size_t)kvh * head_stride) + lane;

  float m = NEG_BIG, l = 0.f;
  f32x4 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nblk = (n_keys + 31) >> 5;
  bf16x8 kf[2][2 * KS], vf[2][DT];
  auto load = [&](int buf, int blk) {  // blk may lie beyond the keys: nothing is fetched then
    const bool ok = blk < nblk;
#pragma unroll
    for (int t = 0; t < 2 * KS; ++t) kf[buf][t] = ok ? kt[((size_t)blk * 2 * KS + t) * 64] : zero8;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) vf[buf][dt] = ok ? vt[((size_t)blk * DT + dt) * 64] : zero8;
  };
  auto step = [&](int buf, int blk) {
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < KS; ++t) {
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[buf][t], qf[t], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[buf][KS + t], qf[t], s1, 0, 0, 0);
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
    const bf16x8 pb = {(bf16_t)pv[0], (bf16_t)pv[1], (bf16_t)pv[2], (bf16_t)pv[3], (bf16_t)pv[4], (bf16_t)pv[5], (bf16_t)pv[6], (bf16_t)pv[7]};
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      o[dt] *= corr;
      o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[buf][dt], pb, o[dt], 0, 0, 0);
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
  if (g == 0) { sm[wave][c] = m; sl[wave][c] = l; }
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int i = 0; i < 4; ++i) so[wave][16 * dt + 4 * g + i][c] = o[dt][i];
  __syncthreads();
  constexpr int CH = HD * 16 / (NWV * 64);  // each thread finishes CH consecutive dims of one query
  const int qi = tid & 15, d0 = (tid >> 4) * CH;
  float M = sm[0][qi];
#pragma unroll
  for (int wv = 1; wv < NWV; ++wv) M = fmaxf(M, sm[wv][qi]);
  float w[NWV], Lsum = 0.f;
#pragma unroll
  for (int wv = 0; wv < NWV; ++wv) { w[wv] = __expf(sm[wv][qi] - M); Lsum += w[wv] * sl[wv][qi]; }
  const int r = row0 + qi;
  if (r < row_end) {
    const int width = n_q * HD;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const int d = d0 + j;
      float acc = 0.f;
#pragma unroll
      for (int wv = 0; wv < NWV; ++wv) acc += w[wv] * so[wv][d][qi];
      const int col = head * HD + d;
      const size_t idx = out_tiled ? tile_index(r, col, width) : (size_t)r * width + col;
      out[idx] = (bf16_t)(acc / Lsum);
    }
  }
}

// K [T, n_kv, hd] and V row-major -> the tiled cache layout of one slot (test helper for dlm_attention)
__global__ void pack_kv_kernel(const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, bf16_t* __restrict__ kt, bf16_t* __restrict__ vt,
                               int T, int n_kv, int hd, size_t head_stride) {
  const size_t total = (size_t)T * n_kv * hd;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int d = i % hd, h = (i / hd) % n_kv, pos = i / ((size_t)hd * n_kv);
    kt[(size_t)h * head_stride + kv_k_index(pos, d, hd)] = k[i];
    vt[(size_t)h * head_stride + kv_v_index(pos, d, hd)] = v[i];
  }
}

}  // namespace

void launch_pack_kv(const bf16_t* k, const bf16_t* v, bf16_t* kt, bf16_t* vt, int T, int n_kv, int hd, size_t head_stride, hipStream_t st) {
  pack_kv_kernel<<<256, 256, 0, st>>>(k, v, kt, vt, T, n_kv, hd, head_stride);
}

template <>
void launch_attention<float>(const float* q, const float* kcache, const float* vcache, size_t slot_stride, size_t head_stride, const AttnMeta& meta,
                             float* out, bool out_tiled, int rows, int max_seq_rows, int n_q, int n_kv, int hd, hipStream_t st) {
  dim3 grid((max_seq_rows + QT - 1) / QT, n_q, meta.n_seqs);
  if (hd == 32) attention_kernel<float, 32><<<grid, 256, 0, st>>>(q, kcache, vcache, slot_stride, meta, out, out_tiled, n_q, n_kv);
  else if (hd == 64) attention_kernel<float, 64><<<grid, 256, 0, st>>>(q, kcache, vcache, slot_stride, meta, out, out_tiled, n_q, n_kv);
  else attention_kernel<float, 128><<<grid, 256, 0, st>>>(q, kcache, vcache, slot_stride, meta, out, out_tiled, n_q, n_kv);
}

template <>
void launch_attention<bf16_t>(const bf16_t* q, const bf16_t* kcache, const bf16_t* vcache, size_t slot_stride, size_t head_stride,
                              const AttnMeta& meta, bf16_t* out, bool out_tiled, int rows, int max_seq_rows, int n_q, int n_kv, int hd,
                              hipStream_t st) {
  dim3 grid((max_seq_rows + 15) / 16, n_q, meta.n_seqs);
  const bool wide = (size_t)grid.x * grid.y * grid.z >= 512;  // enough workgroups to fill the chip with 4 wavefronts each
#define GO(HD, NWV) attention_mfma_kernel<HD, NWV><<<grid, NWV * 64, 0, st>>>(q, kcache, vcache, slot_stride, head_stride, meta, out, out_tiled, n_q, n_kv)
  if (hd == 32) { if (wide) GO(32, 4); else GO(32, 8); }
  else if (hd == 64) { if (wide) GO(64, 4); else GO(64, 8); }
  else { if (wide) GO(128, 4); else GO(128, 8); }
#undef GO
}
