// Block-vs-prefix attention: every row of a sequence's span attends, without causal mask, to keys
// [0, n_keys) of the sequence's KV-cache slot (cached prefix + the span's own rows, which the
// rotary/KV kernel has already written there).  Grouped-query heads share K/V.
//
// fp32 model (head_dim 32/64/128, row-major cache [pos][n_kv*hd]): one workgroup per (16-query
// tile, head, sequence); keys are streamed in tiles through LDS with an online softmax in fp32.
#include "attention_core.h"

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

// ---- bf16 models: on the matrix cores, half-precision operands (attention_core.h) -----------------------------
// One workgroup per (16-query tile, head, sequence), or DS of them with a share of the head's output dims each.
// per_unit = 0: grid (tiles * DS, heads, sequences).  per_unit > 0: a 1-D grid in which the per_unit workgroups that read the
// same K and V (the query tiles, output-dim shares and query heads of one kv head of one sequence) have ids congruent mod 8:
// they run on the same XCD, and all but the first reader find K and V in its L2 (the XCDs' L2s are separate: spread over
// them, every tile of a block fetches its own copy from memory).
template <int HD, int NWV, int DS>
__global__ __launch_bounds__(NWV * 64) void attention_mfma_kernel(const f16_t* __restrict__ q, const f16_t* __restrict__ kcache,
                                                                  const f16_t* __restrict__ vcache, size_t slot_stride, size_t head_stride,
                                                                  AttnMeta meta, op_t* __restrict__ out_tiles, bf16_t* __restrict__ out_rows, int n_q, int n_kv,
                                                                  int per_unit, int tiles) {
  __shared__ AttnLds<HD, NWV, DS> L;
  int b = blockIdx.z, head = blockIdx.y, x = blockIdx.x;
  if (per_unit > 0) {
    const int j = blockIdx.x >> 3, w = j % per_unit, unit = (j / per_unit) * 8 + (blockIdx.x & 7);
    if (unit >= n_kv * meta.n_seqs) return;
    b = unit / n_kv;
    head = (unit - b * n_kv) * (n_q / n_kv) + w / (tiles * DS);
    x = w % (tiles * DS);
  }
  const int tile = x / DS, dpart = x - tile * DS;
  const int row0 = meta.row_off[b] + tile * 16;
  const int row_end = meta.row_off[b + 1];
  if (row0 >= row_end) return;
  const int kvh = head / (n_q / n_kv);
  const size_t region = (size_t)meta.slot[b] * slot_stride + (size_t)kvh * head_stride;
  attention_tile<HD, NWV, DS>(q, kcache + region, vcache + region, row0, row_end, meta.n_keys[b], head, n_q, out_tiles, out_rows, L, dpart);
}

// K [T, n_kv, hd] and V row-major bf16 -> the tiled half-precision cache layout of one slot (test helper for dlm_attention)
__global__ void pack_kv_kernel(const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, f16_t* __restrict__ kt, f16_t* __restrict__ vt,
                               int T, int n_kv, int hd, size_t head_stride) {
  const size_t total = (size_t)T * n_kv * hd;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int d = i % hd, h = (i / hd) % n_kv, pos = i / ((size_t)hd * n_kv);
    kt[(size_t)h * head_stride + kv_k_index(pos, d, hd)] = to_f16_sat((float)k[i]);
    vt[(size_t)h * head_stride + kv_v_index(pos, d, hd)] = to_f16_sat((float)v[i]);
  }
}
__global__ void to_f16_kernel(const bf16_t* __restrict__ src, f16_t* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = to_f16_sat((float)src[i]);
}

}  // namespace

void launch_pack_kv(const bf16_t* k, const bf16_t* v, f16_t* kt, f16_t* vt, int T, int n_kv, int hd, size_t head_stride, hipStream_t st) {
  pack_kv_kernel<<<256, 256, 0, st>>>(k, v, kt, vt, T, n_kv, hd, head_stride);
}
void launch_to_f16(const bf16_t* src, f16_t* dst, size_t n, hipStream_t st) { to_f16_kernel<<<256, 256, 0, st>>>(src, dst, n); }

template <>
void launch_attention<float>(const float* q, const float* kcache, const float* vcache, size_t slot_stride, size_t head_stride, const AttnMeta& meta,
                             float* out, bool out_tiled, int rows, int max_seq_rows, int n_q, int n_kv, int hd, hipStream_t st) {
  dim3 grid((max_seq_rows + QT - 1) / QT, n_q, meta.n_seqs);
  if (hd == 32) attention_kernel<float, 32><<<grid, 256, 0, st>>>(q, kcache, vcache, slot_stride, meta, out, out_tiled, n_q, n_kv);
  else if (hd == 64) attention_kernel<float, 64><<<grid, 256, 0, st>>>(q, kcache, vcache, slot_stride, meta, out, out_tiled, n_q, n_kv);
  else attention_kernel<float, 128><<<grid, 256, 0, st>>>(q, kcache, vcache, slot_stride, meta, out, out_tiled, n_q, n_kv);
}

void launch_attention_f16(const f16_t* q, const f16_t* kcache, const f16_t* vcache, size_t slot_stride, size_t head_stride, const AttnMeta& meta,
                          op_t* out_tiles, bf16_t* out_rows, int rows, int max_seq_rows, int n_q, int n_kv, int hd, hipStream_t st) {
  const int tiles = (max_seq_rows + 15) / 16;
  // a narrow pass (few query tiles x heads): eight wavefronts per workgroup to shorten each wavefront's chain of dependent
  // loads, and the output dims of a head split over four workgroups (two for 64 dims) to spread its K / V traffic
  const bool narrow = (size_t)tiles * n_q * meta.n_seqs < 128 && hd >= 64;
  const bool wide = (size_t)tiles * n_q * meta.n_seqs >= 512;  // enough workgroups to fill the chip with 4 wavefronts each
  // enough (kv head, sequence) units to keep every XCD busy (four each): the workgroups of a unit share an XCD (see the kernel)
  const int units = n_kv * meta.n_seqs;
  const bool by_unit = units >= 32;
#define GO(HD, NWV, DS)                                                                                                                          \
  do {                                                                                                                                           \
    const int per_unit = by_unit ? tiles * DS * (n_q / n_kv) : 0;                                                                                \
    const dim3 grid = by_unit ? dim3((units + 7) / 8 * 8 * per_unit) : dim3(tiles * DS, n_q, meta.n_seqs);                                       \
    attention_mfma_kernel<HD, NWV, DS><<<grid, NWV * 64, 0, st>>>(q, kcache, vcache, slot_stride, head_stride, meta, out_tiles, out_rows, n_q,   \
                                                                  n_kv, per_unit, tiles);                                                        \
  } while (0)
  if (hd == 32) { if (wide) GO(32, 4, 1); else GO(32, 8, 1); }
  else if (hd == 64) { if (narrow) GO(64, 8, 2); else if (wide) GO(64, 4, 1); else GO(64, 8, 1); }
  else { if (narrow) GO(128, 8, 4); else if (wide) GO(128, 4, 1); else GO(128, 8, 1); }
#undef GO
}
