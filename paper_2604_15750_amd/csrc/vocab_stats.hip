// Fused vocabulary reduction (paper Sec. 4.2: Eq. 3 and the entropy signal; Sec. 4.3: confidence
// and prediction).  One pass over each row of logits gives, with the mask token excluded,
//   m = max z, y = argmax, s = sum e^(z-m), t = sum e^(z-m) (z-m), w = sum e^(z-m) (z-z')
// and from those  lse = m + ln s,  conf = 1/s,  H = ln s - t/s,  KL(p||p') = w/s - lse + lse'.
// The kernel is a pure HBM stream: 16-byte loads, several in flight per lane, rows split over
// enough workgroups to fill 256 CUs; partial states are merged in a fixed order (deterministic).
#include "stats_part.h"

namespace {

constexpr int TPB = 256;
template <typename T> struct Vec;
template <> struct Vec<bf16_t> { static constexpr int N = 8; typedef bf16x8 type; };
template <> struct Vec<float> { static constexpr int N = 4; typedef f32x4 type; };

constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;

// Running state of a wavefront while it streams its share of a row.  The reference of the exponentials is the maximum of
// ALL the wavefront's elements so far (m, the same in every lane), not each lane's own: a new maximum then turns up a few
// times per row instead of in some lane at nearly every step, so the rescaling and the search for the maximum's token id sit
// in a wavefront-uniform branch that is almost never taken, and the common path is straight-line: per element a subtract and
// a multiply for the exponent, one exp2, one add and one fma (two more for KL).  The exponent-weighted sum
// t2 = sum e^(z-m) (z-m) log2(e) is kept in base-2 units.  bi = lowest token id of the maximum (elements are visited in
// ascending id order within a lane, lanes of one load hold ascending ids, and a later element must be strictly greater).
struct Run {
  float m;          // uniform: running maximum (= the best logit)
  int bi;           // uniform: its token id
  float s, t2, w;   // per lane, relative to m
  float pm, ps;     // previous-step row when its lse is not stored: uniform maximum, per-lane sum e^(z'-pm)
};
constexpr float RUN_MIN = -2.0e38f;  // start of the running maximum: (RUN_MIN - m) * log2(e) stays finite for real maxima m
__device__ inline Run run_init() { return Run{RUN_MIN, 0x7fffffff, 0.f, 0.f, 0.f, RUN_MIN, 0.f}; }

__device__ inline int wave_min_int(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, 64));
  return v;
}

// The 64 lane states -> the wavefront's Part (valid in every lane): the lanes share m, so the sums are plain butterflies in a
// fixed order (deterministic).
__device__ inline Part run_finish(const Run& r) {
  Part p;
  p.m = r.m;
  p.s = wave_sum(r.s);
  p.t = wave_sum(r.t2) * LN2;
  p.w = wave_sum(r.w);
  p.bv = r.m;
  p.bi = r.bi;
  p.pm = r.pm > RUN_MIN ? r.pm : NEG_BIG;
  p.ps = wave_sum(r.ps);
  return p;
}

// A new maximum somewhere in the wavefront (vm = each lane's maximum of its N elements, RUN_MIN if it has none): move the
// reference.  Called by all 64 lanes together, from a wavefront-uniform branch.
template <int N>
__device__ inline void new_maximum(Run& p, const float (&z)[N], unsigned valid, float vm, int v0) {
  const float wmax = wave_max(vm);
  int cand = 0x7fffffff;
#pragma unroll
  for (int i = N - 1; i >= 0; --i)
    if (((valid >> i) & 1u) && z[i] == wmax) cand = v0 + i;
  const float d2 = (p.m - wmax) * LOG2E, a = __builtin_amdgcn_exp2f(d2);
  p.t2 = a * fmaf(d2, p.s, p.t2);
  p.s *= a;
  p.w *= a;
  p.m = wmax;
  p.bi = wave_min_int(cand);
}
template <int N>
__device__ inline void new_prev_maximum(Run& p, float vm) {
  const float wmax = wave_max(vm);
  p.ps *= __builtin_amdgcn_exp2f((p.pm - wmax) * LOG2E);
  p.pm = wmax;
}

// Absorb N consecutive logits (first token id v0) of every lane; bit i of `valid` says that element i takes part (the mask
// token and elements past the end do not).  ALL: every element of every lane is valid (the common path: no selects).
// Called by all 64 lanes of a wavefront together.
template <int N, bool KL, bool PREV_SUMS, bool ALL>
__device__ inline void absorb(Run& p, const float (&z)[N], const float (&zp)[N], int v0, unsigned valid) {
  float vm = RUN_MIN;
#pragma unroll
  for (int i = 0; i < N; ++i) vm = fmaxf(vm, (ALL || ((valid >> i) & 1u)) ? z[i] : RUN_MIN);
  if (__builtin_amdgcn_ballot_w64(vm > p.m) != 0) new_maximum<N>(p, z, ALL ? 0xffffffffu : valid, vm, v0);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const float d2 = (z[i] - p.m) * LOG2E;  // the difference first: exact for nearby values
    float e = __builtin_amdgcn_exp2f(d2);
    if (!ALL) e = ((valid >> i) & 1u) ? e : 0.f;
    p.s += e;
    p.t2 = fmaf(e, ALL ? d2 : (((valid >> i) & 1u) ? d2 : 0.f), p.t2);
    if (KL) p.w = fmaf(e, ALL ? z[i] - zp[i] : (((valid >> i) & 1u) ? z[i] - zp[i] : 0.f), p.w);
  }
  if (KL && PREV_SUMS) {
    float pv = RUN_MIN;
#pragma unroll
    for (int i = 0; i < N; ++i) pv = fmaxf(pv, (ALL || ((valid >> i) & 1u)) ? zp[i] : RUN_MIN);
    if (__builtin_amdgcn_ballot_w64(pv > p.pm) != 0) new_prev_maximum<N>(p, pv);
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const float e = __builtin_amdgcn_exp2f((zp[i] - p.pm) * LOG2E);
      p.ps += (ALL || ((valid >> i) & 1u)) ? e : 0.f;
    }
  }
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

// One wavefront's share of elements [lo, hi) of a row (the workgroup walks them together: lane l of the workgroup takes the
// l-th vector of every stride).  Whole trips of U vectors (16 bytes each) per lane are loaded together and absorbed one after
// the other without a bounds or mask test; the trip that holds the mask token and the ragged last one take the path with
// per-element validity.  Loop bounds are uniform in the workgroup: the absorb steps exchange values between lanes.
template <typename T, bool VECTOR, bool KL, bool PREV_SUMS>
__device__ inline void stream_chunk(Run& run, const T* __restrict__ z_row, const T* __restrict__ p_row, T* __restrict__ s_row, int lo,
                                    int hi, int mask_id) {
  constexpr int N = Vec<T>::N;
  typedef typename Vec<T>::type V;
  if (VECTOR) {
    constexpr int U = 4, STRIDE = TPB * N, TRIP = U * STRIDE;
    const int base = lo + threadIdx.x * N;
    const int nfull = (hi - lo) / TRIP;
    for (int t = 0; t * TRIP < hi - lo; ++t) {
      const int t0 = lo + t * TRIP;  // first element of the trip (uniform)
      const bool plain = t < nfull && !(mask_id >= t0 && mask_id < t0 + TRIP);
      V zv[U], pv[U];
      if (plain) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          zv[u] = *(const V*)(z_row + base + t * TRIP + u * STRIDE);
          if (KL) pv[u] = *(const V*)(p_row + base + t * TRIP + u * STRIDE);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int v = base + t * TRIP + u * STRIDE;
          float z[N], zp[N];
#pragma unroll
          for (int i = 0; i < N; ++i) { z[i] = to_f32(zv[u][i]); zp[i] = KL ? to_f32(pv[u][i]) : 0.f; }
          if (s_row) *(V*)(s_row + v) = zv[u];
          absorb<N, KL, PREV_SUMS, true>(run, z, zp, v, 0xffffffffu);
        }
      } else {
#pragma unroll 1
        for (int u = 0; u < U; ++u) {
          const int v = base + t * TRIP + u * STRIDE;
          if (t0 + u * STRIDE >= hi) break;  // uniform
          const bool in = v < hi;            // vocab % N == 0 and lo % N == 0: a vector is inside or outside as a whole
          float z[N], zp[N];
          V a, b;
          if (in) { a = *(const V*)(z_row + v); if (KL) b = *(const V*)(p_row + v); }
#pragma unroll
          for (int i = 0; i < N; ++i) { z[i] = in ? to_f32(a[i]) : 0.f; zp[i] = (KL && in) ? to_f32(b[i]) : 0.f; }
          if (s_row && in) *(V*)(s_row + v) = a;
          unsigned valid = in ? (1u << N) - 1u : 0u;
          if (mask_id >= v && mask_id < v + N) valid &= ~(1u << (mask_id - v));  // the mask token takes no part
          absorb<N, KL, PREV_SUMS, false>(run, z, zp, v, valid);
        }
      }
    }
  } else {
    for (int v0 = lo; v0 < hi; v0 += TPB) {  // uniform bounds; a lane past the end or on the mask token feeds an invalid element
      const int v = v0 + threadIdx.x;
      const bool in = v < hi;
      float z[1] = {in ? to_f32(z_row[v]) : 0.f}, zp[1] = {(KL && in) ? to_f32(p_row[v]) : 0.f};
      if (s_row && in) s_row[v] = z_row[v];
      absorb<1, KL, PREV_SUMS, false>(run, z, zp, v, (in && v != mask_id) ? 1u : 0u);
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
  const Part p = run_finish(run);
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
