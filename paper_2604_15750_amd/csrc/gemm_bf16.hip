// bf16 GEMM  Y[M,N] = X[M,K] * W[N,K]^T  on the gfx950 matrix cores, fp32 accumulation, with the
// layer's row-wise glue fused into the epilogue.
//
// At decode shapes (M = 8..384 rows against 15 GB of weights per pass) the GEMMs are bound by
// streaming W from HBM, so both kernels are weight streamers that happen to multiply:
//   * W is re-tiled once, when the model is created, into 1 KiB fragments (16 rows x 32 k) that are
//     exactly the A operand of v_mfma_f32_16x16x32_bf16: a wavefront fetches a fragment as 64
//     consecutive 16-byte loads and walks a contiguous run of HBM along K, W goes HBM -> registers;
//   * activations live in the same fragment tiling (B operand), written that way by their producer;
//   * the product is computed transposed (W fragment = A operand), so a lane ends up with four
//     consecutive output columns of one row.
//
// skinny kernel (M <= 32): one workgroup per 16- or 32-column output tile over the whole of K.  Its
//   wavefronts split K among themselves, keep 8 KiB of W (and the matching X fragments) in flight each,
//   and add their accumulators through LDS in wavefront order (deterministic).  No workgroup ever
//   waits for another, so there is no workspace, no counter and no serial tail.
// tiled kernel (M > 32, and the LM head): a workgroup of four wavefronts owns 128 output columns;
//   the X fragments of a K-chunk are staged through LDS once and shared; K is split across
//   workgroups when N alone cannot fill 256 CUs.  Partial tiles go to an fp32 workspace; the
//   workgroup that arrives last at the tile's ticket adds them in split order (deterministic) and
//   runs the epilogue.
// Epilogues (on the finished tile, both kernels):
//   QKV     1/rms of the input row, rotary embedding, Q row-major, K and V into the tiled KV cache
//   SWIGLU  1/rms, silu(gate) * up into the fragment tiling of the down projection
//   RESID   residual add, x = h * gain of the next RMSNorm into fragment tiling, and the share of
//           sum(h^2) per row of each 16-column (skinny) or 128-column (tiled) tile
//   SUM     plain sum (optionally scaled per row) to bf16 or fp32
//   DIRECT  (LM head, tiled kernel without split) accumulators straight to bf16 with the 1/rms scale
// W_qkv and W_gate_up are packed with their rows permuted (weight_source_row) so that a rotary pair,
// or a gate column and its up column, sit 8 columns apart in one 16-column tile.
#include "common.h"

namespace {

constexpr int TPB = 256;
constexpr int KC = 4;  // k-tiles (of 32) per staged chunk of the tiled kernel

// 1/rms of rows [m_lo, m_lo + rows) from the producer's partial sums of squares into s_rinv, by the whole workgroup of NT
// threads: sixteen lanes per row, each adding every sixteenth chunk, then a fixed butterfly (deterministic).
template <int NT>
__device__ inline void block_rinv(const RowScale& rs, int m_lo, int rows, float* s_rinv) {
  const int sub = threadIdx.x & 15;
  for (int row = threadIdx.x >> 4; row < rows; row += NT / 16) {
    float ss = 0.f;
    if (rs.ssq)
      for (int c = sub; c < rs.nch; c += 16) ss += rs.ssq[(size_t)(m_lo + row) * rs.nch + c];
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    if (sub == 0) s_rinv[row] = rs.ssq ? rsqrtf(ss * rs.inv_d + rs.eps) : 1.f;
  }
}

__device__ inline bf16x4 to_bf16x4(f32x4 v) { return bf16x4{(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]}; }

// ---- what an epilogue does with finished values -------------------------------------------------------
// Rotary pair group: a = packed columns nc+4gp .. +3 of a 16-column tile starting at packed column nc,
// b = the same + 8; they are dims i .. i+3 and i+half .. i+half+3 of one head.
__device__ inline void finish_qkv(const GemmEpi& e, int m, int nc, int gp, f32x4 a, f32x4 b) {
  const int hd = e.hd, half = hd >> 1;
  const int head = nc / hd, i = 8 * ((nc % hd) >> 4) + 4 * gp;
  if (head < e.n_q + e.n_kv) {
    const f32x4 c = *(const f32x4*)(e.rope_cos + (size_t)m * half + i), sn = *(const f32x4*)(e.rope_sin + (size_t)m * half + i);
    const f32x4 ra = a * c - b * sn, rb = b * c + a * sn;
    a = ra;
    b = rb;
  }
  const bf16x4 ab = to_bf16x4(a), bb = to_bf16x4(b);
  if (head < e.n_q) {
    bf16_t* dst = e.q + (size_t)m * e.n_q * hd + (size_t)head * hd;
    *(bf16x4*)(dst + i) = ab;
    *(bf16x4*)(dst + i + half) = bb;
    return;
  }
  const bool is_k = head < e.n_q + e.n_kv;
  const int kvh = is_k ? head - e.n_q : head - e.n_q - e.n_kv;
  const int pos = e.row_pos[m];
  bf16_t* dst = (is_k ? e.kcache : e.vcache) + (size_t)e.slot[e.row_seq[m]] * e.slot_stride + (size_t)kvh * e.head_stride;
  if (is_k) {  // four consecutive dims share a lane slot of the K tiling
    *(bf16x4*)(dst + kv_k_index(pos, i, hd)) = ab;
    *(bf16x4*)(dst + kv_k_index(pos, i + half, hd)) = bb;
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      dst[kv_v_index(pos, i + j, hd)] = ab[j];
      dst[kv_v_index(pos, i + half + j, hd)] = bb[j];
    }
  }
}

// gate = packed columns nc+4gp .. +3, up = the same + 8: output columns 8 (nc/16) + 4gp .. +3
__device__ inline void finish_swiglu(const GemmEpi& e, int m, int nc, int gp, f32x4 g, f32x4 u) {
  bf16x4 o;
#pragma unroll
  for (int t = 0; t < 4; ++t) o[t] = (bf16_t)(g[t] / (1.f + __expf(-g[t])) * u[t]);
  *(bf16x4*)(e.act + tile_index(m, 8 * (nc >> 4) + 4 * gp, e.ffn)) = o;
}

// residual add and next norm's x for columns n .. n+3 of row m; returns the four columns' share of sum h^2
__device__ inline float finish_resid(const GemmEpi& e, int m, int n, int N, f32x4 y) {
  const size_t o = (size_t)m * N + n;
  const f32x4 v = *(const f32x4*)(e.h + o) + y;
  *(f32x4*)(e.h + o) = v;
  const f32x4 g = *(const f32x4*)(e.gain + n);
  *(bf16x4*)(e.x + tile_index(m, n, N)) = to_bf16x4(v * g);
  return v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
}

__device__ inline void finish_sum(const GemmEpi& e, int m, int n, int N, f32x4 v) {
  const size_t o = (size_t)m * N + n;
  if (e.out_bf16) *(bf16x4*)(e.out_bf16 + o) = to_bf16x4(v);
  else *(f32x4*)(e.out_f32 + o) = v;
}

// ---- skinny kernel ------------------------------------------------------------------------------------
// grid.x = N / (16 R) workgroups of NWV wavefronts; wavefront w multiplies k-tiles [w*per, (w+1)*per) of the
// workgroup's R column tiles against all MT row tiles, D k-tiles per batch, two batches of registers.
template <int MT, int R, int NWV, int D, int EPI>
__global__ __launch_bounds__(NWV * 64) void gemm_skinny_kernel(const bf16x8* __restrict__ xt, const bf16x8* __restrict__ wt, int M, int N,
                                                               int K, GemmEpi e) {
  __shared__ f32x4 red[NWV][R * MT][64];
  __shared__ float s_rinv[MT * 16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int KT = K >> 5, MTILES = (M + 15) >> 4;
  const int per = (KT + NWV - 1) / NWV;
  const int t_begin = wave * per, t_end = min(KT, t_begin + per);
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  const bf16x8* wbase = wt + (size_t)blockIdx.x * KT * R * 64 + lane;  // the workgroup's R tiles are one interleaved run

  f32x4 acc[R][MT];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  bf16x8 wreg[2][D][R], xreg[2][D][MT];

  auto load = [&](int buf, int tb) {
#pragma unroll
    for (int i = 0; i < D; ++i) {
      const int t = tb + i;
      const bool ok = t < t_end;
#pragma unroll
      for (int r = 0; r < R; ++r) wreg[buf][i][r] = ok ? wbase[((size_t)t * R + r) * 64] : zero8;
#pragma unroll
      for (int j = 0; j < MT; ++j) xreg[buf][i][j] = (ok && j < MTILES) ? xt[((size_t)j * KT + t) * 64 + lane] : zero8;
    }
  };
  auto compute = [&](int buf) {
#pragma unroll
    for (int i = 0; i < D; ++i)
#pragma unroll
      for (int j = 0; j < MT; ++j)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[buf][i][r], xreg[buf][i][j], acc[r][j], 0, 0, 0);
  };

  load(0, t_begin);
  // 1/rms of the input rows, needed only by the epilogue: fetched while the first batch is in flight
  if (EPI != EPI_RESID) block_rinv<NWV * 64>(e.rs, 0, min(M, MT * 16), s_rinv);
  for (int tb = t_begin; tb < t_end; tb += 2 * D) {
    load(1, tb + D);
    compute(0);
    load(0, tb + 2 * D);
    compute(1);
  }

#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < MT; ++j) red[wave][r * MT + j][lane] = acc[r][j];
  __syncthreads();

  const int g = lane >> 4, ml = lane & 15;
  for (int rj = wave; rj < R * MT; rj += NWV) {  // one wavefront finishes one 16 x 16 tile: lane = (row ml, columns 4g .. 4g+3)
    const int r = rj / MT, j = rj % MT;
    const int m = j * 16 + ml;
    const int nc = (blockIdx.x * R + r) * 16;
    if (EPI == EPI_QKV || EPI == EPI_SWIGLU) {
      if (g >= 2 || m >= M) continue;
      f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < NWV; ++w) {
        a += red[w][rj][lane];
        b += red[w][rj][lane + 32];
      }
      a *= s_rinv[m];
      b *= s_rinv[m];
      if (EPI == EPI_QKV) finish_qkv(e, m, nc, g, a, b);
      else finish_swiglu(e, m, nc, g, a, b);
    } else {
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < NWV; ++w) v += red[w][rj][lane];
      if (EPI == EPI_RESID) {
        float ss = m < M ? finish_resid(e, m, nc + 4 * g, N, v) : 0.f;
        ss += __shfl_xor(ss, 16, 64);
        ss += __shfl_xor(ss, 32, 64);
        if (g == 0 && m < M) e.ssq_out[(size_t)m * (N >> 4) + (nc >> 4)] = ss;
      } else if (m < M) {
        finish_sum(e, m, nc + 4 * g, N, v * s_rinv[m]);
      }
    }
  }
}

// ---- tiled kernel: partial tiles cross workgroups ------------------------------------------------------
// The partial tiles cross workgroups (and the per-XCD L2 caches) inside one launch.  They are written
// through and read with device scope (sc1) instead of bracketing them with device-scope fences, which
// would write back and invalidate a whole L2 per workgroup.  A tile row of one workgroup is 512
// contiguous bytes, so no cache line is shared between writers.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int SC1 = 16;  // cache-policy bit of the raw-buffer builtins: device scope

__device__ inline __amdgpu_buffer_rsrc_t tile_rsrc(const float* base) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, 0x7fffffff, 0x00020000);
}
__device__ inline void store4_coherent(float* base, unsigned byte_off, f32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), tile_rsrc(base), byte_off, 0, SC1);
}
// sum over the splits, in split order, of four consecutive floats at byte_off from tile (one tile per split, `stride` floats apart).
// The loads of eight splits are in flight together: one trip to memory per batch instead of one per split.
__device__ inline f32x4 sum_splits4(const float* tile, int splits, size_t stride, unsigned byte_off) {
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < splits; s0 += 8) {
    u32x4 t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int s = min(s0 + i, splits - 1);  // the surplus loads of the last batch repeat its last split and are not added
      t[i] = __builtin_amdgcn_raw_buffer_load_b128(tile_rsrc(tile + s * stride), byte_off, 0, SC1);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (s0 + i < splits) v += __builtin_bit_cast(f32x4, t[i]);
  }
  return v;
}

template <int MT, int PR, int EPI>
__global__ __launch_bounds__(TPB) void gemm_bf16_kernel(const bf16x8* __restrict__ xt, const bf16x8* __restrict__ wt, int M, int N, int K,
                                                        int kt_per_split, GemmEpi e) {
  constexpr int R = 2;  // a wavefront owns two adjacent column tiles; a workgroup 128 columns
  constexpr int XP = MT * KC / 4;  // 16-byte pieces of X each thread stages per chunk
  __shared__ bf16x8 xs[2][MT * KC * 64];
  __shared__ float s_rinv[MT * 16];
  __shared__ int s_last;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int KT = K >> 5, MTILES = (M + 15) >> 4, NPAIRS = N >> 5;
  const int mt0 = blockIdx.z * MT;
  const int pair0 = blockIdx.x * 4 + wave;
  const bool wave_active = pair0 < NPAIRS;
  const int splits = gridDim.y;
  const int t_begin = blockIdx.y * kt_per_split;
  const int t_end = min(KT, t_begin + kt_per_split);
  const int n_chunks = (t_end - t_begin + KC - 1) / KC;
  // fragment (column tile 2 pair0 + r, k-tile t): interleaved pairs (pr == 2) or one run per column tile (pr == 1)
  const size_t w_tile_step = PR == 2 ? 128 : 64, w_r_step = PR == 2 ? 64 : (size_t)KT * 64;
  const bf16x8* wbase = wt + (size_t)pair0 * KT * 128 + lane;

  f32x4 acc[R][MT];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  bf16x8 wreg[2][KC][R];
  bf16x8 xreg[XP];
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

  auto load_w = [&](bf16x8(&dst)[KC][R], int chunk) {
#pragma unroll
    for (int tc = 0; tc < KC; ++tc) {
      const int t = t_begin + chunk * KC + tc;
#pragma unroll
      for (int r = 0; r < R; ++r) dst[tc][r] = (wave_active && t < t_end) ? wbase[t * w_tile_step + r * w_r_step] : zero8;
    }
  };
  auto load_x = [&](int chunk) {
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const int q = tid + TPB * i;
      const int j = q / (KC * 64), tc = (q / 64) % KC, ln = q & 63;
      const int t = t_begin + chunk * KC + tc;
      xreg[i] = (mt0 + j < MTILES && t < t_end) ? xt[((size_t)(mt0 + j) * KT + t) * 64 + ln] : zero8;
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XP; ++i) xs[buf][tid + TPB * i] = xreg[i];
  };
  auto compute = [&](const bf16x8(&w)[KC][R], int buf) {
#pragma unroll
    for (int tc = 0; tc < KC; ++tc) {
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        const bf16x8 xf = xs[buf][(j * KC + tc) * 64 + lane];
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[tc][r], xf, acc[r][j], 0, 0, 0);
      }
    }
  };

  if (n_chunks > 0) {
    load_w(wreg[0], 0);
    load_x(0);
  }
  // 1/rms of the input rows for the epilogue, fetched while the first chunk is in flight (published by the loop's barriers)
  if (EPI != EPI_RESID) block_rinv<TPB>(e.rs, mt0 * 16, min(M, (mt0 + MT) * 16) - mt0 * 16, s_rinv);
  if (n_chunks > 0) {
    store_x(0);
    __syncthreads();
    for (int c = 0; c < n_chunks; c += 2) {
      if (c + 1 < n_chunks) { load_w(wreg[1], c + 1); load_x(c + 1); }
      compute(wreg[0], 0);
      if (c + 1 < n_chunks) store_x(1);
      __syncthreads();
      if (c + 1 >= n_chunks) break;
      if (c + 2 < n_chunks) { load_w(wreg[0], c + 2); load_x(c + 2); }
      compute(wreg[1], 1);
      if (c + 2 < n_chunks) store_x(0);
      __syncthreads();
    }
  }

  const int g = lane >> 4, ml = lane & 15;
  const int m_lo = mt0 * 16, m_hi = min(M, (mt0 + MT) * 16);
  if (EPI == EPI_DIRECT) {  // accumulators -> bf16, one pass, no workspace
    if (!wave_active) return;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int n0 = (pair0 * 2 + r) * 16 + g * 4;
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        const int m = (mt0 + j) * 16 + ml;
        if (m >= M) continue;
        *(bf16x4*)(e.out_bf16 + (size_t)m * N + n0) = to_bf16x4(acc[r][j] * s_rinv[j * 16 + ml]);
      }
    }
    return;
  }

  // partial tile -> workspace (written through to device scope)
  const size_t stride = (size_t)M * N;
  const int n0 = blockIdx.x * 128;
  float* tile = e.part + (size_t)m_lo * N + n0;  // this workgroup's tile of split 0
  if (wave_active) {
    float* mine = tile + blockIdx.y * stride;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int nl = (wave * 2 + r) * 16 + g * 4;
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        const int mrel = j * 16 + ml;
        if (m_lo + mrel < M) store4_coherent(mine, ((unsigned)mrel * N + nl) * 4u, acc[r][j]);
      }
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // every wavefront's stores have completed ...
  __syncthreads();                                        // ... before the workgroup takes its ticket
  if (tid == 0) {
    const int cidx = blockIdx.z * gridDim.x + blockIdx.x;
    int last = 1;
    if (splits > 1) {
      last = __hip_atomic_fetch_add(&e.counters[cidx], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == splits - 1;
      if (last) __hip_atomic_store(&e.counters[cidx], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next launch
    }
    s_last = last;
  }
  __syncthreads();
  if (!s_last) return;

  const int rows = m_hi - m_lo;
  if (EPI == EPI_QKV || EPI == EPI_SWIGLU) {  // item = (row, 16-column tile of the 128, rotary / gate group of four)
    for (int idx = tid; idx < rows * 16; idx += TPB) {
      const int mrel = idx >> 4, t16 = (idx >> 1) & 7, gp = idx & 1, m = m_lo + mrel;
      const unsigned off = ((unsigned)mrel * N + t16 * 16 + gp * 4) * 4u;
      const f32x4 a = sum_splits4(tile, splits, stride, off) * s_rinv[mrel];
      const f32x4 b = sum_splits4(tile, splits, stride, off + 32u) * s_rinv[mrel];
      if (EPI == EPI_QKV) finish_qkv(e, m, n0 + t16 * 16, gp, a, b);
      else finish_swiglu(e, m, n0 + t16 * 16, gp, a, b);
    }
  } else if (EPI == EPI_RESID) {
    const int iters = (rows * 32 + TPB - 1) / TPB;
    for (int it = 0; it < iters; ++it) {
      const int idx = tid + it * TPB;
      const int mrel = idx >> 5, c4 = idx & 31, m = m_lo + mrel;
      float ss = 0.f;
      if (mrel < rows) ss = finish_resid(e, m, n0 + 4 * c4, N, sum_splits4(tile, splits, stride, ((unsigned)mrel * N + 4 * c4) * 4u));
#pragma unroll
      for (int ofs = 16; ofs > 0; ofs >>= 1) ss += __shfl_xor(ss, ofs, 64);  // the 32 lanes of one row
      if (mrel < rows && c4 == 0) e.ssq_out[(size_t)m * (N >> 7) + (n0 >> 7)] = ss;
    }
  } else {
    for (int idx = tid; idx < rows * 32; idx += TPB) {
      const int mrel = idx >> 5, c4 = idx & 31;
      if (n0 + 4 * c4 >= N) continue;
      finish_sum(e, m_lo + mrel, n0 + 4 * c4, N, sum_splits4(tile, splits, stride, ((unsigned)mrel * N + 4 * c4) * 4u) * s_rinv[mrel]);
    }
  }
}

// W [N, K] row-major -> fragment tiles, `pr` row-tiles interleaved along k, rows permuted by (perm, param).
__global__ void pack_weight_kernel(const bf16x8* __restrict__ w, bf16x8* __restrict__ out, int N, int K, int pr, int perm, int param) {
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
    out[idx] = w[(size_t)n * (K >> 3) + k8];
  }
}

// X [M, K] row-major -> fragment tiles [ceil(M/16)][K/32]; rows beyond M are zero.
__global__ void pack_act_kernel(const bf16x8* __restrict__ x, bf16x8* __restrict__ out, int M, int K) {
  const int KT = K >> 5;
  const size_t total = (size_t)((M + 15) >> 4) * KT * 64;
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int lane = idx & 63;
    const size_t tile = idx >> 6;
    const int t = tile % KT;
    const int m = (int)(tile / KT) * 16 + (lane & 15);
    out[idx] = m < M ? x[(size_t)m * (K >> 3) + t * 4 + (lane >> 4)] : zero8;
  }
}

bool use_skinny(int M, int N, int pr, int kind) { return kind != EPI_DIRECT && M <= 32 && N % (16 * pr) == 0; }

template <int MT, int EPI>
void launch_skinny(const bf16_t* xt, const bf16_t* wt, int pr, int M, int N, int K, const GemmEpi& e, hipStream_t st) {
  if (pr == 1) gemm_skinny_kernel<MT, 1, 8, 8, EPI><<<N / 16, 512, 0, st>>>((const bf16x8*)xt, (const bf16x8*)wt, M, N, K, e);
  else gemm_skinny_kernel<MT, 2, 4, 4, EPI><<<N / 32, 256, 0, st>>>((const bf16x8*)xt, (const bf16x8*)wt, M, N, K, e);
}

template <int MT, int EPI>
void launch_mt(const bf16_t* xt, const bf16_t* wt, int pr, int M, int N, int K, int splits, int mblocks, const GemmEpi& e, hipStream_t st) {
  const int KT = K >> 5;
  const int kps = ((KT + splits - 1) / splits + KC - 1) / KC * KC;
  dim3 grid(((N >> 5) + 3) / 4, (KT + kps - 1) / kps, mblocks);
  if (pr == 2) gemm_bf16_kernel<MT, 2, EPI><<<grid, TPB, 0, st>>>((const bf16x8*)xt, (const bf16x8*)wt, M, N, K, kps, e);
  else gemm_bf16_kernel<MT, 1, EPI><<<grid, TPB, 0, st>>>((const bf16x8*)xt, (const bf16x8*)wt, M, N, K, kps, e);
}

template <int EPI>
void launch_epi(const bf16_t* xt, const bf16_t* wt, int pr, int M, int N, int K, const GemmEpi& e, hipStream_t st) {
  const int mtiles = (M + 15) >> 4;
  if (use_skinny(M, N, pr, EPI)) {
    constexpr int SE = EPI == EPI_DIRECT ? EPI_SUM : EPI;  // (never taken for DIRECT; keeps the instantiation list short)
    if (mtiles <= 1) launch_skinny<1, SE>(xt, wt, pr, M, N, K, e, st);
    else launch_skinny<2, SE>(xt, wt, pr, M, N, K, e, st);
    return;
  }
  const int splits = EPI == EPI_DIRECT ? 1 : gemm_bf16_splits(M, N, K);
#define GO(MT) launch_mt<MT, EPI>(xt, wt, pr, M, N, K, splits, (mtiles + MT - 1) / MT, e, st)
  if (mtiles <= 1) GO(1);
  else if (mtiles <= 2) GO(2);
  else if (mtiles <= 3) GO(3);
  else if (mtiles <= 4) GO(4);
  else if (mtiles <= 6) GO(6);
  else if (mtiles <= 8) GO(8);
  else if (mtiles <= 12) GO(12);
  else GO(16);
#undef GO
}

}  // namespace

void launch_pack_weight(const bf16_t* w, bf16_t* out, int N, int K, int pr, int perm, int perm_param, hipStream_t st) {
  pack_weight_kernel<<<2048, 256, 0, st>>>((const bf16x8*)w, (bf16x8*)out, N, K, pr, perm, perm_param);
}
void launch_pack_act(const bf16_t* x, bf16_t* out, int M, int K, hipStream_t st) {
  pack_act_kernel<<<512, 256, 0, st>>>((const bf16x8*)x, (bf16x8*)out, M, K);
}

// Number of K-splits of the tiled kernel: enough workgroups to cover the chip a few times, at least 8 k-tiles each.
int gemm_bf16_splits(int M, int N, int K) {
  const int KT = K >> 5;
  const int groups = ((N >> 5) + 3) / 4;
  const int mblocks = (((M + 15) >> 4) + 15) / 16;
  int s = (768 + groups * mblocks - 1) / (groups * mblocks);
  const int max_s = KT / 8 > 0 ? KT / 8 : 1;
  if (s > max_s) s = max_s;
  if (s > 32) s = 32;
  if (s < 1) s = 1;
  const int kps = ((KT + s - 1) / s + KC - 1) / KC * KC;  // splits that leave no empty tail
  return (KT + kps - 1) / kps;
}

int gemm_bf16_counters(int max_rows, int max_n) { return ((max_n >> 5) + 3) / 4 * ((max_rows + 15) / 16); }

int gemm_bf16_ssq_chunks(int M, int N) { return M <= 32 ? N >> 4 : N >> 7; }

void launch_gemm_bf16(const bf16_t* xt, const bf16_t* wt, int pr, int M, int N, int K, const GemmEpi& e, hipStream_t st) {
  switch (e.kind) {
    case EPI_DIRECT: launch_epi<EPI_DIRECT>(xt, wt, pr, M, N, K, e, st); break;
    case EPI_QKV: launch_epi<EPI_QKV>(xt, wt, pr, M, N, K, e, st); break;
    case EPI_SWIGLU: launch_epi<EPI_SWIGLU>(xt, wt, pr, M, N, K, e, st); break;
    case EPI_RESID: launch_epi<EPI_RESID>(xt, wt, pr, M, N, K, e, st); break;
    default: launch_epi<EPI_SUM>(xt, wt, pr, M, N, K, e, st); break;
  }
}
