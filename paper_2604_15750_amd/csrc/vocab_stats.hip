// Fused vocabulary reduction (paper Sec. 4.2: Eq. 3 and the entropy signal; Sec. 4.3: confidence
// and prediction).  One pass over each row of logits gives, with the mask token excluded,
//   m = max z, y = argmax, s = sum e^(z-m), t = sum e^(z-m) (z-m), w = sum e^(z-m) (z-z')
// and from those  lse = m + ln s,  conf = 1/s,  H = ln s - t/s,  KL(p||p') = w/s - lse + lse'.
// The kernel is a pure HBM stream: 16-byte loads, several in flight per lane, rows split over
// enough workgroups to fill 256 CUs; partial states are merged in a fixed order (deterministic).
#include "stats_part.h"

namespace {

constexpr int TPB = 256;
// the 64 lane states of a wavefront -> one (valid in every lane): all lanes move to the wavefront's maximum first, then the sums are
// plain butterflies in a fixed order (deterministic), which costs one exp per lane instead of four per butterfly step
__device__ inline Part part_wave_reduce(const Part& p) {
  Part r;
  r.m = wave_max(p.m);
  const float d = p.m - r.m, a = __expf(d);
  r.s = wave_sum(a * p.s);
  r.t = wave_sum(a * (p.t + d * p.s));
  r.w = wave_sum(a * p.w);
  r.bv = p.bv;
  r.bi = p.bi;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(r.bv, o, 64);
    const int oi = __shfl_xor(r.bi, o, 64);
    if (ov > r.bv || (ov == r.bv && oi < r.bi)) { r.bv = ov; r.bi = oi; }
  }
  r.pm = wave_max(p.pm);
  r.ps = wave_sum(__expf(p.pm - r.pm) * p.ps);
  return r;
}

template <typename T> struct Vec;
template <> struct Vec<bf16_t> { static constexpr int N = 8; typedef bf16x8 type; };
template <> struct Vec<float> { static constexpr int N = 4; typedef f32x4 type; };

constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;

// Running state of one lane while it streams: like Part, but the exponent-weighted sum t2 = sum e^(z-m) (z-m) log2(e) is kept
// in base-2 units so that an element costs a subtract and a multiply for the exponent, one exp2, one add and one fma (plus two for KL).
struct Run {
  float m;  // running maximum
  float s, t2, w;
  float bv;
  int bi;
  float pm, ps;
};
constexpr float RUN_MIN = -2.0e38f;  // start of the running maximum: (RUN_MIN - m) * log2(e) stays finite for real maxima m
__device__ inline Run run_init() { return Run{RUN_MIN, 0.f, 0.f, 0.f, NEG_BIG, 0x7fffffff, NEG_BIG, 0.f}; }
__device__ inline Part run_finish(const Run& r) { return Part{r.m, r.s, r.t2 * LN2, r.w, r.bv, r.bi, r.pm, r.ps}; }

// absorb N consecutive logits (first token id = v0) into the state; element `skip` (the mask token; -1: none) is left out
template <int N, bool KL, bool PREV_SUMS, bool SKIP>
__device__ inline void absorb_impl(Run& p, const float (&z)[N], const float (&zp)[N], int v0, int skip_at) {
  const int skip = SKIP ? skip_at : -1;  // compile-time "none" on the common path: no per-element tests
  float vm = RUN_MIN;
#pragma unroll
  for (int i = 0; i < N; ++i)
    if (i != skip) vm = fmaxf(vm, z[i]);
  if (vm > p.m) {  // rare after the first few vectors: rescale the sums to the new maximum
    const float d2 = (p.m - vm) * LOG2E, a = __builtin_amdgcn_exp2f(d2);
    p.t2 = a * fmaf(d2, p.s, p.t2);
    p.s *= a;
    p.w *= a;
    p.m = vm;
#pragma unroll
    for (int i = 0; i < N; ++i)
      if (i != skip && z[i] > p.bv) { p.bv = z[i]; p.bi = v0 + i; }   // ascending ids + strict '>' keep the lowest id
  }
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (i == skip) continue;
    const float d2 = (z[i] - p.m) * LOG2E, e = __builtin_amdgcn_exp2f(d2);  // the difference first: exact for nearby values
    p.s += e;
    p.t2 = fmaf(e, d2, p.t2);
    if (KL) p.w = fmaf(e, z[i] - zp[i], p.w);
  }
  if (KL && PREV_SUMS) {
    float pv = NEG_BIG;
#pragma unroll
    for (int i = 0; i < N; ++i)
      if (i != skip) pv = fmaxf(pv, zp[i]);
    if (pv > p.pm) { p.ps *= __expf(p.pm - pv); p.pm = pv; }
#pragma unroll
    for (int i = 0; i < N; ++i)
      if (i != skip) p.ps += __expf(zp[i] - p.pm);
  }
}

template <int N, bool KL, bool PREV_SUMS>
__device__ inline void absorb(Run& p, const float (&z)[N], const float (&zp)[N], int v0, int skip = -1) {
  if (skip < 0) absorb_impl<N, KL, PREV_SUMS, false>(p, z, zp, v0, -1);
  else absorb_impl<N, KL, PREV_SUMS, true>(p, z, zp, v0, skip);
}

__device__ inline void finalize(const Part& p, int row, bool has_prev, float prev_lse, const StatsOut& o, float* save_lse_slot) {
  float ls = __logf(p.s);
  float lse = p.m + ls;
  o.max_logit[row] = p.m;
  o.lse[row] = lse;
  o.conf[row] = 1.0f / p.s;
  o.entropy[row] = ls - p.t / p.s;
  o.argmax[row] = p.bi;
  o.kl[row] = has_prev ? (p.w / p.s - lse + prev_lse) : 0.f;
  if (save_lse_slot) *save_lse_slot = lse;
}

// Work item (row, c): elements [c*chunk, (c+1)*chunk) of one row; a workgroup takes every gridDim.x-th item.
// one lane's share of elements [lo, hi) of a row: U vectors (16 bytes each) in flight, then absorbed one after the other
template <typename T, bool VECTOR, bool KL, bool PREV_SUMS>
__device__ inline void stream_chunk(Run& run, const T* __restrict__ z_row, const T* __restrict__ p_row, T* __restrict__ s_row, int lo,
                                    int hi, int mask_id) {
  constexpr int N = Vec<T>::N;
  typedef typename Vec<T>::type V;
  if (VECTOR) {
    constexpr int U = 4;
    for (int v0 = lo + threadIdx.x * N; v0 < hi; v0 += TPB * N * U) {
      V zv[U], pv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int v = v0 + u * TPB * N;
        if (v < hi) {
          zv[u] = *(const V*)(z_row + v);
          if (KL) pv[u] = *(const V*)(p_row + v);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int v = v0 + u * TPB * N;
        if (v >= hi) break;
        float z[N], zp[N];
#pragma unroll
        for (int i = 0; i < N; ++i) { z[i] = to_f32(zv[u][i]); zp[i] = KL ? to_f32(pv[u][i]) : 0.f; }
        if (s_row) *(V*)(s_row + v) = zv[u];
        const int skip = (mask_id >= v && mask_id < v + N) ? mask_id - v : -1;  // the mask token takes no part
        absorb<N, KL, PREV_SUMS>(run, z, zp, v, skip);
      }
    }
  } else {
    for (int v = lo + threadIdx.x; v < hi; v += TPB) {
      float z[1] = {to_f32(z_row[v])}, zp[1] = {0.f};
      if (s_row) s_row[v] = z_row[v];
      if (KL) zp[0] = to_f32(p_row[v]);
      if (v == mask_id) continue;  // the mask token takes no part
      absorb<1, KL, PREV_SUMS>(run, z, zp, v);
    }
  }
}

template <typename T, bool VECTOR>
__global__ __launch_bounds__(TPB) void vocab_stats_kernel(const T* __restrict__ logits, int rows, int vocab, int mask_id, int chunk,
                                                          int nchunks, StatsRows sr, StatsOut o, Part* __restrict__ parts) {
  constexpr int N = Vec<T>::N;
  typedef typename Vec<T>::type V;
  __shared__ Part sh[TPB / 64];
  for (int item = blockIdx.x; item < rows * nchunks; item += gridDim.x) {
  const int row = item / nchunks, c = item - row * nchunks;
  const T* z_row = logits + (size_t)row * vocab;
  const int64_t prow = sr.prev_row ? sr.prev_row[row] : (sr.prev_base ? (int64_t)row * vocab : -1);
  const int64_t srow = sr.save_row ? sr.save_row[row] : -1;
  const T* p_row = prow >= 0 ? (const T*)sr.prev_base + prow : nullptr;
  T* s_row = srow >= 0 ? (T*)sr.save_base + srow : nullptr;
  const bool kl = p_row != nullptr;
  const bool prev_sums = kl && sr.prev_lse == nullptr;
  const int lo = c * chunk, hi = min(vocab, lo + chunk);

  Run run = run_init();
  if (!kl) stream_chunk<T, VECTOR, false, false>(run, z_row, p_row, s_row, lo, hi, mask_id);
  else if (!prev_sums) stream_chunk<T, VECTOR, true, false>(run, z_row, p_row, s_row, lo, hi, mask_id);
  else stream_chunk<T, VECTOR, true, true>(run, z_row, p_row, s_row, lo, hi, mask_id);
  Part p = run_finish(run);
  p = part_wave_reduce(p);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = p;
  __syncthreads();
  if (threadIdx.x == 0) {
    Part r = sh[0];
    for (int i = 1; i < TPB / 64; ++i) r = part_merge(r, sh[i]);
    if (nchunks == 1) {
      float pl = 0.f;
      if (kl) pl = sr.prev_lse ? sr.prev_lse[prow / vocab] : r.pm + __logf(r.ps);
      finalize(r, row, kl, pl, o, srow >= 0 && sr.save_lse ? sr.save_lse + srow / vocab : nullptr);
    } else {
      parts[(size_t)row * nchunks + c] = r;
    }
  }
  __syncthreads();  // sh is reused by the next item
  }
}

// one wavefront per row: lane c holds the partial state of chunk c (of chunks c, c + 64, ... merged in that order); fixed butterfly order
__global__ __launch_bounds__(64) void vocab_stats_merge_kernel(const Part* __restrict__ parts, int rows, int nchunks, int vocab, StatsRows sr,
                                                               StatsOut o) {
  const int row = blockIdx.x, lane = threadIdx.x;
  Part r = lane < nchunks ? parts[(size_t)row * nchunks + lane] : part_init();
  for (int c0 = 64; c0 < nchunks; c0 += 512) {  // more states than lanes (the LM-head epilogue's): eight loads in flight, added in order
    Part q[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] = c0 + 64 * i + lane < nchunks ? parts[(size_t)row * nchunks + c0 + 64 * i + lane] : part_init();
#pragma unroll
    for (int i = 0; i < 8; ++i) r = part_merge(r, q[i]);
  }
#pragma unroll
  for (int ofs = 32; ofs > 0; ofs >>= 1) r = part_merge(r, part_shfl_xor(r, ofs));
  if (lane != 0) return;
  const int64_t prow = sr.prev_row ? sr.prev_row[row] : (sr.prev_base ? (int64_t)row * vocab : -1);
  const int64_t srow = sr.save_row ? sr.save_row[row] : -1;
  float pl = 0.f;
  if (prow >= 0) pl = sr.prev_lse ? sr.prev_lse[prow / vocab] : r.pm + __logf(r.ps);
  finalize(r, row, prow >= 0, pl, o, srow >= 0 && sr.save_lse ? sr.save_lse + srow / vocab : nullptr);
}

constexpr int MAX_CHUNKS = 32;

// Chunks per row: a work item is a whole row when the rows alone fill the chip (the per-item reduction across lanes is not free),
// otherwise rows are cut so that there are about 1536 items, each at least two vectors per lane.
int pick_chunks(int rows, int vocab, int vec) {
  int want = (1536 + rows - 1) / rows;
  int maxc = (vocab + TPB * vec * 2 - 1) / (TPB * vec * 2);
  int c = want < maxc ? want : maxc;
  if (c > MAX_CHUNKS) c = MAX_CHUNKS;
  return c < 1 ? 1 : c;
}

}  // namespace

size_t stats_workspace_bytes(int rows) { return (size_t)rows * MAX_CHUNKS * sizeof(Part); }

void launch_stats_merge(const void* parts, int rows, int nparts, int vocab, const StatsRows& sr, const StatsOut& o, hipStream_t st) {
  vocab_stats_merge_kernel<<<rows, 64, 0, st>>>((const Part*)parts, rows, nparts, vocab, sr, o);
}

template <typename T>
void launch_vocab_stats(const T* logits, int rows, int vocab, int mask_id, const StatsRows& sr, const StatsOut& o, void* workspace, hipStream_t st) {
  constexpr int N = Vec<T>::N;
  const bool vec = vocab % N == 0;
  int nch = pick_chunks(rows, vocab, N);
  int chunk = (vocab + nch - 1) / nch;
  chunk = (chunk + TPB * N - 1) / (TPB * N) * (TPB * N);
  nch = (vocab + chunk - 1) / chunk;
  const int items = rows * nch;
  const int grid = items;  // the hardware dispatcher balances better than a resident grid walking the items
  if (vec) vocab_stats_kernel<T, true><<<grid, TPB, 0, st>>>(logits, rows, vocab, mask_id, chunk, nch, sr, o, (Part*)workspace);
  else vocab_stats_kernel<T, false><<<grid, TPB, 0, st>>>(logits, rows, vocab, mask_id, chunk, nch, sr, o, (Part*)workspace);
  if (nch > 1) vocab_stats_merge_kernel<<<rows, 64, 0, st>>>((const Part*)workspace, rows, nch, vocab, sr, o);
}

template void launch_vocab_stats<float>(const float*, int, int, int, const StatsRows&, const StatsOut&, void*, hipStream_t);
template void launch_vocab_stats<bf16_t>(const bf16_t*, int, int, int, const StatsRows&, const StatsOut&, void*, hipStream_t);
