// Row-wise glue of the transformer pass: row tables and rotary tables, embedding + RMSNorm,
// split-K reduction fused with residual add + RMSNorm, SiLU-gating, rotary embedding + KV-cache
// write.  All fp32 arithmetic; a bf16 model's GEMM inputs are written in half precision, in the fragment tiling the GEMM reads.
#include "common.h"

namespace {

// one workgroup per row: row -> (sequence, position, token index, retained-logit offsets), rotary table
__global__ void prepare_kernel(SeqMeta meta, StatsMeta sm, RowTables t, int rows, int vocab, int head_dim, float theta) {
  const int r = blockIdx.x;
  int b = 0;
  while (b + 1 < meta.n_seqs && r >= meta.row_off[b + 1]) ++b;
  const int rel = r - meta.row_off[b];
  const int pos = meta.span_start[b] + rel;
  if (threadIdx.x == 0) {
    t.row_seq[r] = b;
    t.row_pos[r] = pos;
    t.row_tok[r] = meta.tok_start[b] + rel;
    t.row_slot[r] = meta.slot[b];
    const int kr = rel - sm.kl_first[b];
    t.prev_row[r] = (kr >= 0 && kr < sm.kl_count[b]) ? sm.prev_off[b] + (int64_t)kr * vocab : -1;
    const int sr = rel - sm.save_first[b];
    t.save_row[r] = (sr >= 0 && sr < sm.save_count[b]) ? sm.save_off[b] + (int64_t)sr * vocab : -1;
  }
  const int half = head_dim / 2;
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    const double inv_freq = pow((double)theta, -2.0 * (double)i / (double)head_dim);
    double s, c;
    sincos((double)pos * inv_freq, &s, &c);
    t.rope_cos[(size_t)r * half + i] = (float)c;
    t.rope_sin[(size_t)r * half + i] = (float)s;
  }
}

__device__ inline float block_sum_256(float v, float* buf) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = v;
  __syncthreads();
  return buf[0] + buf[1] + buf[2] + buf[3];
}

// RMSNorm is split in two so that no kernel has to see a whole row: the producer writes
// x = h * gain (unnormalised) plus the sum of squares of its 1024-column chunk; since
// 1/rms is one scalar per row it commutes with the following GEMM, whose consumer multiplies
// it back in (row_rinv).
constexpr int NORM_CHUNK = 1024;

__device__ inline float row_rinv(const float* __restrict__ ssq, int r, int nch, float inv_d, float eps) {
  float s = 0.f;
  for (int c = 0; c < nch; ++c) s += ssq[(size_t)r * nch + c];
  return rsqrtf(s * inv_d + eps);
}

// grid (chunks, rows): h = embedding row, x = h * gain, ssq[row][chunk]
template <typename T>
__global__ __launch_bounds__(256) void embed_norm_kernel(const T* __restrict__ embed, const int32_t* __restrict__ tokens, RowTables t,
                                                         const float* __restrict__ gain, float* __restrict__ h,
                                                         typename Act<T>::x_t* __restrict__ x, float* __restrict__ ssq, int d, int vocab) {
  __shared__ float buf[4];
  const int r = blockIdx.y, k = blockIdx.x * NORM_CHUNK + threadIdx.x * 4;
  // the token buffer is the caller's device memory, which the host cannot validate: an id outside the vocabulary is clamped
  // into it instead of reading outside the embedding table
  const int tok = min(max(tokens[t.row_tok[r]], 0), vocab - 1);
  const T* e = embed + (size_t)tok * d;
  float ss = 0.f;
  if (k < d) {
    f32x4 v, g = *(const f32x4*)(gain + k);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = to_f32(e[k + i]);
    *(f32x4*)(h + (size_t)r * d + k) = v;
#pragma unroll
    for (int i = 0; i < 4; ++i) x[Act<T>::idx(r, k + i, d)] = from_f32<typename Act<T>::x_t>(v[i] * g[i]);
    ss = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  }
  ss = block_sum_256(ss, buf);
  if (threadIdx.x == 0) ssq[(size_t)r * gridDim.x + blockIdx.x] = ss;
}

// grid (chunks, rows): h += sum_s part[s]; x = h * gain; ssq[row][chunk]
template <typename T>
__global__ __launch_bounds__(256) void reduce_residual_norm_kernel(const float* __restrict__ part, int splits, size_t split_stride,
                                                                   float* __restrict__ h, const float* __restrict__ gain,
                                                                   T* __restrict__ x, float* __restrict__ ssq, int d) {
  __shared__ float buf[4];
  const int r = blockIdx.y, k = blockIdx.x * NORM_CHUNK + threadIdx.x * 4;
  float ss = 0.f;
  if (k < d) {
    const size_t o = (size_t)r * d + k;
    f32x4 v = *(const f32x4*)(h + o);
    f32x4 g = *(const f32x4*)(gain + k);
    for (int s = 0; s < splits; ++s) v += *(const f32x4*)(part + s * split_stride + o);
    *(f32x4*)(h + o) = v;
#pragma unroll
    for (int i = 0; i < 4; ++i) x[Act<T>::idx(r, k + i, d)] = from_f32<T>(v[i] * g[i]);
    ss = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  }
  ss = block_sum_256(ss, buf);
  if (threadIdx.x == 0) ssq[(size_t)r * gridDim.x + blockIdx.x] = ss;
}

template <typename T>
__global__ __launch_bounds__(256) void silu_mul_kernel(const float* __restrict__ part, int splits, size_t split_stride,
                                                       const float* __restrict__ ssq, int nch, float inv_d, float eps,
                                                       T* __restrict__ act, int rows, int ffn) {
  const int r = blockIdx.y;
  const int k = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (k >= ffn) return;
  const float rinv = row_rinv(ssq, r, nch, inv_d, eps);
  const float* base = part + (size_t)r * 2 * ffn;
  f32x4 g = {0.f, 0.f, 0.f, 0.f}, u = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < splits; ++s) {
    g += *(const f32x4*)(base + s * split_stride + k);
    u += *(const f32x4*)(base + s * split_stride + ffn + k);
  }
  g *= rinv;
  u *= rinv;
#pragma unroll
  for (int i = 0; i < 4; ++i) act[Act<T>::idx(r, k + i, ffn)] = from_f32<T>(g[i] / (1.f + __expf(-g[i])) * u[i]);
}

// grid (rows, n_q + 2*n_kv heads), hd/2 lanes: one rotary pair per lane
template <typename T>
__global__ void rope_kv_kernel(const float* __restrict__ part, int splits, size_t split_stride, const float* __restrict__ ssq, int nch,
                               float inv_d, float eps, RowTables t, SeqMeta meta, T* __restrict__ q, T* __restrict__ kcache,
                               T* __restrict__ vcache, size_t slot_stride, size_t head_stride, int n_q, int n_kv, int hd) {
  const int r = blockIdx.x, head = blockIdx.y, i = threadIdx.x, half = hd >> 1;
  const int width = (n_q + 2 * n_kv) * hd;
  const float* src = part + (size_t)r * width + (size_t)head * hd;
  float a = 0.f, b = 0.f;
  for (int s = 0; s < splits; ++s) {
    a += src[s * split_stride + i];
    b += src[s * split_stride + i + half];
  }
  const float rinv = row_rinv(ssq, r, nch, inv_d, eps);
  a *= rinv;
  b *= rinv;
  const int pos = t.row_pos[r];
  if (head < n_q + n_kv) {  // Q and K heads are rotated
    const float c = t.rope_cos[(size_t)r * half + i], sn = t.rope_sin[(size_t)r * half + i];
    const float ra = a * c - b * sn, rb = b * c + a * sn;
    a = ra;
    b = rb;
  }
  if (head < n_q) {
    T* dst = q + (size_t)r * n_q * hd + (size_t)head * hd;
    dst[i] = from_f32<T>(a);
    dst[i + half] = from_f32<T>(b);
    return;
  }
  const bool is_k = head < n_q + n_kv;
  const int kvh = is_k ? head - n_q : head - n_q - n_kv;
  T* base = (is_k ? kcache : vcache) + (size_t)meta.slot[t.row_seq[r]] * slot_stride;
  // fp32 cache: row-major [pos][n_kv*hd] (this kernel serves the fp32 model; a bf16 model writes its tiled half-precision
  // cache from the QKV GEMM's epilogue)
  T* dst = base + (size_t)pos * n_kv * hd + (size_t)kvh * hd;
  dst[i] = from_f32<T>(a);
  dst[i + half] = from_f32<T>(b);
}

}  // namespace

void launch_prepare(const SeqMeta& meta, const StatsMeta& sm, RowTables t, int rows, int vocab, int head_dim, float theta, hipStream_t st) {
  prepare_kernel<<<rows, 64, 0, st>>>(meta, sm, t, rows, vocab, head_dim, theta);
}

int norm_chunks(int d) { return (d + NORM_CHUNK - 1) / NORM_CHUNK; }

template <typename T>
void launch_embed_norm(const T* embed, const int32_t* tokens, const RowTables& t, const float* gain, float* h, typename Act<T>::x_t* x, float* ssq,
                       int rows, int d, int vocab, hipStream_t st) {
  embed_norm_kernel<T><<<dim3(norm_chunks(d), rows), 256, 0, st>>>(embed, tokens, t, gain, h, x, ssq, d, vocab);
}
template <typename T>
void launch_reduce_residual_norm(const float* part, int splits, float* h, const float* gain, T* x, float* ssq, int rows, int d, hipStream_t st) {
  reduce_residual_norm_kernel<T><<<dim3(norm_chunks(d), rows), 256, 0, st>>>(part, splits, (size_t)rows * d, h, gain, x, ssq, d);
}
template <typename T>
void launch_silu_mul(const float* part, int splits, const float* ssq, int d, float eps, T* act, int rows, int ffn, hipStream_t st) {
  dim3 grid((ffn / 4 + 255) / 256, rows);
  silu_mul_kernel<T><<<grid, 256, 0, st>>>(part, splits, (size_t)rows * 2 * ffn, ssq, norm_chunks(d), 1.f / (float)d, eps, act, rows, ffn);
}
template <typename T>
void launch_rope_kv(const float* part, int splits, const float* ssq, int d, float eps, const RowTables& t, const SeqMeta& meta, T* q,
                    T* kcache, T* vcache, size_t slot_stride, size_t head_stride, int rows, int n_q, int n_kv, int hd, hipStream_t st) {
  dim3 grid(rows, n_q + 2 * n_kv);
  rope_kv_kernel<T><<<grid, hd / 2, 0, st>>>(part, splits, (size_t)rows * (n_q + 2 * n_kv) * hd, ssq, norm_chunks(d), 1.f / (float)d, eps, t,
                                             meta, q, kcache, vcache, slot_stride, head_stride, n_q, n_kv, hd);
}

// the row-wise glue kernels serve the fp32 model; a bf16 model runs them in its GEMM epilogues and uses only the embedding here
template void launch_embed_norm<float>(const float*, const int32_t*, const RowTables&, const float*, float*, float*, float*, int, int, int, hipStream_t);
template void launch_embed_norm<bf16_t>(const bf16_t*, const int32_t*, const RowTables&, const float*, float*, op_t*, float*, int, int, int, hipStream_t);
template void launch_reduce_residual_norm<float>(const float*, int, float*, const float*, float*, float*, int, int, hipStream_t);
template void launch_silu_mul<float>(const float*, int, const float*, int, float, float*, int, int, hipStream_t);
template void launch_rope_kv<float>(const float*, int, const float*, int, float, const RowTables&, const SeqMeta&, float*, float*, float*, size_t,
                                    size_t, int, int, int, int, hipStream_t);
