// Internal declarations shared by the HIP sources of libdlm (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/dlm.h"

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// IEEE half: what a bf16 model's matrix-core operands are stored as.  Same bytes and matrix-core rate as bf16 with three more
// mantissa bits; values beyond +-65504 saturate (to_f16_sat).
//   * attention: Q, the KV cache, the unnormalised probabilities;
//   * GEMMs (op_t): every activation a GEMM reads (the norm outputs h * gain, the attention output, the gated FFN activation)
//     and the packed weights.  A bf16 weight converts exactly unless it is below 2^-14 in magnitude (then it keeps an absolute
//     error of at most 2^-25).  Rounding the activations to bf16's 8 mantissa bits instead is what carries most of a deep
//     model's logit error: at 32 layers of the 8B shape the worst logit error is 1.4e-2 of the row's scale with bf16 norm
//     outputs (whatever the precision of the others) and 0.5e-2 with all of them in half.
// The residual stream stays fp32, the logits bf16.
typedef _Float16 f16_t;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef f16_t op_t;
typedef f16x8 op8;
typedef f16x4 op4;

#define DLM_WAVE 64

int dlm_fail(int code, const char* fmt, ...);
#define DLM_HIP(expr)                                                                        \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess) return dlm_fail(DLM_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// ---- activation layouts -------------------------------------------------------------------
// fp32 models keep activations row-major.  bf16 models keep every GEMM input (op_t) in "fragment tiles":
// element (m, k) of an [M, K] matrix lives in the 1 KiB tile (m/16, k/32), at lane
// (m%16) + 16*((k%32)/8), slot k%8 -- exactly one operand of the 16x16x32 half-precision matrix-core
// instruction per tile, so a wavefront fetches an operand as 64 consecutive 16-byte pieces.
__host__ __device__ inline size_t tile_index(int m, int k, int K) {
  return ((size_t)(m >> 4) * (size_t)(K >> 5) + (size_t)(k >> 5)) * 512 + (size_t)(((m & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7));
}
// bf16 KV cache of one (slot, kv head): K in tiles of 16 positions x 32 dims (A operand of S^T = K Q^T), V in tiles of 16 dims x 32
// positions (A operand of O^T = V^T P^T) whose 8-element lane slots hold positions {4g..4g+3, 16+4g..16+4g+3} of the 32-block: the order in
// which the first product leaves the keys in a lane's registers.
__host__ __device__ inline size_t kv_k_index(int pos, int d, int hd) {
  return ((size_t)(pos >> 4) * (size_t)(hd >> 5) + (size_t)(d >> 5)) * 512 + (size_t)(((pos & 15) + 16 * ((d & 31) >> 3)) * 8 + (d & 7));
}
__host__ __device__ inline size_t kv_v_index(int pos, int d, int hd) {
  const int p32 = pos & 31, r = p32 & 15, g = r >> 2, j = (r & 3) + 4 * (p32 >> 4);
  return ((size_t)(pos >> 5) * (size_t)(hd >> 4) + (size_t)(d >> 4)) * 512 + (size_t)(((d & 15) + 16 * g) * 8 + j);
}

template <typename T> struct Act;
template <> struct Act<float> {  // x_t: what the model's GEMM inputs are stored as
  typedef float x_t;
  static __device__ inline size_t idx(int m, int k, int K) { return (size_t)m * K + k; }
};
template <> struct Act<bf16_t> {
  typedef op_t x_t;
  static __device__ inline size_t idx(int m, int k, int K) { return tile_index(m, k, K); }
};

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(bf16_t x) { return (float)x; }
__device__ inline float to_f32(f16_t x) { return (float)x; }
__device__ inline f16_t to_f16_sat(float x) { return (f16_t)__builtin_amdgcn_fmed3f(x, -65504.f, 65504.f); }
template <typename T> __device__ inline T from_f32(float x);
template <> __device__ inline float from_f32<float>(float x) { return x; }
template <> __device__ inline bf16_t from_f32<bf16_t>(float x) { return (bf16_t)x; }
template <> __device__ inline f16_t from_f32<f16_t>(float x) { return to_f16_sat(x); }
__device__ inline f32x4 mfma_op(op8 a, op8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- per-pass metadata, passed to kernels by value -------------------------------------------
#define DLM_MAX_SEQS 32

struct SeqMeta {
  int32_t n_seqs;
  int32_t row_off[DLM_MAX_SEQS + 1];
  int32_t span_start[DLM_MAX_SEQS];
  int32_t slot[DLM_MAX_SEQS];
  int32_t tok_start[DLM_MAX_SEQS];
};
struct StatsMeta {  // which rows are compared with / retained as p^prev; offsets in elements of the retained-logit buffer
  int32_t kl_first[DLM_MAX_SEQS], kl_count[DLM_MAX_SEQS], save_first[DLM_MAX_SEQS], save_count[DLM_MAX_SEQS];
  int64_t prev_off[DLM_MAX_SEQS], save_off[DLM_MAX_SEQS];
};
struct AttnMeta {
  int32_t n_seqs;
  int32_t row_off[DLM_MAX_SEQS + 1];
  int32_t n_keys[DLM_MAX_SEQS];   // keys [0, n_keys) of the slot's cache are visible to every row of the sequence
  int32_t slot[DLM_MAX_SEQS];
};
struct BoundaryMeta {
  int32_t win_start[DLM_MAX_SEQS];
  int32_t win_len[DLM_MAX_SEQS];
  int32_t cold[DLM_MAX_SEQS];
};
struct SelectMeta {
  int32_t row_start[DLM_MAX_SEQS];
  int32_t tok_start[DLM_MAX_SEQS];
  int32_t block_len[DLM_MAX_SEQS];
};
struct RowTables {  // device arrays of one pass, [rows]
  int32_t* row_seq;   // packed sequence index of the row
  int32_t* row_pos;   // absolute position
  int32_t* row_tok;   // index of the row's token in the caller's token array
  int32_t* row_slot;  // KV-cache slot of the row's sequence
  float* rope_cos;    // [rows, hd/2]
  float* rope_sin;
  int64_t* prev_row;  // element offset of the row's retained p^prev logits, or -1
  int64_t* save_row;  // element offset where the row's logits are retained, or -1
};

// ---- launchers (callers have validated shapes) -------------------------------------------------
// weight tiling: W [N, K] row-major bf16 -> 1 KiB fragments of 16 rows x 32 k in half precision (op_t), `pr` (1 or 2) row-tiles interleaved along k:
// fragment (nt, kt) sits at ((nt/pr * K/32 + kt) * pr + nt%pr) KiB.  The rows may be permuted first so that the columns an
// epilogue has to combine share one 16-column output tile (packed row n holds source row weight_source_row(n, ...)):
//   PERM_ROTARY (param = head_dim): tile b of a head holds dims 8b..8b+7 and their rotary partners 8b+hd/2..8b+hd/2+7
//   PERM_GATED  (param = d_ffn):    tile g holds gate rows 8g..8g+7 and the up rows 8g..8g+7
enum { PERM_NONE = 0, PERM_ROTARY = 1, PERM_GATED = 2 };
__host__ __device__ inline int weight_source_row(int n, int perm, int param) {
  if (perm == PERM_ROTARY) {
    const int head = n / param, w = n % param, c = w & 15;
    return head * param + 8 * (w >> 4) + (c & 7) + (c >= 8 ? param / 2 : 0);
  }
  if (perm == PERM_GATED) {
    const int c = n & 15, o = 8 * (n >> 4) + (c & 7);
    return c < 8 ? o : param + o;
  }
  return n;
}
__host__ __device__ inline int weight_pack_rows(int N) { return N <= 8192 ? 1 : 2; }  // narrow matrices: one run per 16-column tile
void launch_pack_weight(const bf16_t* w, op_t* out, int N, int K, int perm, int perm_param, hipStream_t st);
// W [N, K] row-major -> step-major fragments for the kernel that serves (N, K) at up to 16 rows: column groups of ct tiles
// and W = 4 wavefronts per workgroup (the mid kernel's no-split launches), or ct = 1 and W = 8 (the skinny kernel's 16-column
// workgroups).  The fragment (column tile g ct + r, k-tile w KT/W + s) that wavefront w of workgroup g reads at its step s sits
// at (((s G + g) W + w) ct + r) KiB, G = N / (16 ct): what all workgroups read at the same step is one run of memory, and the
// chip's reads at any moment are one moving window instead of thousands of separate streams.
void launch_pack_weight_steps(const bf16_t* w, op_t* out, int N, int K, int ct, int perm, int perm_param, hipStream_t st);
int gemm_bf16_steps_ct(int N, int K, int kind);  // ct of that layout for (N, K) under epilogue `kind`, 0 if the kernel that serves 16 rows has none
int gemm_mid_steps_ct(int N, int K);   // ... if the mid kernel serves (N, K) at up to 16 rows without a K split, else 0
void launch_pack_act(const bf16_t* x, op_t* out, int M, int K, hipStream_t st);  // row-major bf16 -> fragment tiles in half (rows padded to 16 with zeros)
int gemm_bf16_splits(int M, int N, int K, int kind);  // partial tiles [splits][M][N] the launch of this shape and epilogue needs in GemmEpi::part (1: none)
int gemm_bf16_ssq_chunks(int M, int N, int K);     // chunks per row of the sums of squares an EPI_RESID launch of this shape writes
int gemm_bf16_counters(int max_rows, int max_n);   // ticket counters a state needs in GemmEpi::counters (zero-initialised, self-resetting)
int gemm_tiled_counters(int max_rows, int max_n);
int gemm_tiled_splits(int M, int N, int K);
int gemm_tiled_ssq_chunks(int M, int N);
int gemm_tiled_stat_parts(int M, int N);
void gemm_tiled_set_target(int wgs);               // tuning: workgroups the K split aims at
// rs (optional): every output row m is multiplied by rsqrt(sum_c rs.ssq[m][c] * rs.inv_d + rs.eps).
struct RowScale {
  const float* ssq;
  int nch;
  float inv_d, eps;
};
enum { EPI_DIRECT = 0, EPI_QKV = 1, EPI_SWIGLU = 2, EPI_RESID = 3, EPI_SUM = 4, EPI_STATS = 5 };
// What the bf16 GEMM does with a finished output tile (see gemm_bf16.hip).
struct GemmEpi {
  int kind;
  float* part;        // [gemm_bf16_splits][M][N] fp32 partial tiles of the tiled kernel when it splits K
  int* counters;      // gemm_bf16_counters tickets, one per (column group, row block) of a launch that splits K
  RowScale rs;        // 1/rms of the GEMM's input rows (QKV, SWIGLU, DIRECT, SUM; ssq may be null)
  // EPI_QKV (weights packed with PERM_ROTARY)
  const int32_t *row_pos, *row_slot;
  const float *rope_cos, *rope_sin;
  f16_t *q, *kcache, *vcache;  // IEEE half (see f16_t)
  size_t slot_stride, head_stride;
  int n_q, n_kv, hd;
  // EPI_SWIGLU (weights packed with PERM_GATED): act in fragment tiles
  op_t* act;
  int ffn;
  // EPI_RESID: h += y; x = h * gain (fragment tiles); ssq_out[m][gemm_bf16_ssq_chunks(M, N, K)] = each column tile's share of sum h^2
  float* h;
  const float* gain;
  op_t* x;
  float* ssq_out;
  // EPI_DIRECT (bf16) / EPI_SUM (either)
  bf16_t* out_bf16;
  float* out_f32;
  // EPI_STATS (the LM head of a pass that compares and retains no row; at most GEMM_STATS_MAX_ROWS rows): logits to out_bf16 as
  // EPI_DIRECT does, and per row and column group the online-softmax state of the group's logits as written (rounded to bf16,
  // token skip_col left out) to stat_parts[m][gemm_bf16_stat_parts(N)]
  void* stat_parts;
  int skip_col;
  // optional second copy of W in the step-major layout (launch_pack_weight_steps) of column groups of w_steps_ct tiles
  const op_t* w_steps;
  int w_steps_ct;
};
constexpr int GEMM_STATS_MAX_ROWS = 64;
int gemm_bf16_stat_parts(int M, int N);              // column groups per row an EPI_STATS launch of this shape writes states for
// The GEMM kernels are launched through hipExtLaunchKernelGGL, which can stamp two events with the kernel's own start and end
// (the dispatch's timestamps: what a profiler reports, with no marker packets between dependent kernels).  A caller that
// wants the next GEMM launch of this thread timed sets g_launch_stamp; the launch takes the events and clears it.
struct LaunchStamp { hipEvent_t start, stop; };
extern thread_local LaunchStamp g_launch_stamp;
#define DLM_LAUNCH(kernel, grid, block, lds, st, ...)                                                                           \
  do {                                                                                                                          \
    const LaunchStamp ls_ = g_launch_stamp;                                                                                     \
    g_launch_stamp = LaunchStamp{nullptr, nullptr};                                                                             \
    hipExtLaunchKernelGGL((kernel), dim3(grid), dim3(block), (unsigned)(lds), (st), ls_.start, ls_.stop, 0, __VA_ARGS__);       \
  } while (0)
// Y = X * W^T.  xt: fragment-tiled [Mpad, K]; wt: weights [N, K] as packed by launch_pack_weight.
void launch_gemm_bf16(const op_t* xt, const op_t* wt, int M, int N, int K, const GemmEpi& e, hipStream_t st);
#define GEMM_SKINNY_MAX_ROWS 64
void launch_gemm_skinny(const op_t* xt, const op_t* wt, int pr, int M, int N, int K, const GemmEpi& e, hipStream_t st);  // M <= GEMM_SKINNY_MAX_ROWS
void launch_gemm_tiled(const op_t* xt, const op_t* wt, int M, int N, int K, const GemmEpi& e, hipStream_t st);
#define GEMM_MID_MAX_ROWS 160  // 65 .. this many rows: the mid kernel (all rows in one workgroup, wavefronts split K)
#define GEMM_MID_MAX_ROWS_NARROW 256  // ... for matrices of at most 8192 columns
int gemm_mid_splits(int M, int N, int K);
int gemm_mid_ssq_chunks(int M, int N, int K);
bool gemm_mid_fills_chip(int M, int N, int K);  // its column groups are a whole number of rounds over the compute units, without a K split
int gemm_mid_counters(int max_n);
void gemm_mid_set_target(int wgs);  // tuning: workgroups the K split aims at
void launch_gemm_mid(const op_t* xt, const op_t* wt, int M, int N, int K, const GemmEpi& e, hipStream_t st);  // M <= GEMM_MID_MAX_ROWS(_NARROW); narrow matrices from 17 rows
#define GEMM_MACRO_MIN_ROWS_NARROW 256  // more rows than this: the macro-tile kernel whatever the width
int gemm_macro_ssq_chunks(int M, int N, int K);
int gemm_macro_splits(int M, int N, int K);
int gemm_macro_counters(int max_rows, int max_n);
void gemm_macro_set_target(int wgs);  // tuning: workgroups the K split aims at
void gemm_macro_set_penalty(int tile, double p);  // tuning: relative cost per product of tile candidate 0 .. 5 (256x256, 128x256, 128x128, 192x256, 256x192, 192x192); 0 switches it off
void launch_gemm_macro(const op_t* xt, const op_t* wt, int M, int N, int K, const GemmEpi& e, hipStream_t st);
void launch_gemm_f32(const float* x, const float* w, float* y, int M, int N, int K, RowScale rs, hipStream_t st);

void launch_prepare(const SeqMeta& meta, const StatsMeta& sm, RowTables t, int rows, int vocab, int head_dim, float theta, hipStream_t st);
// RMSNorm in two halves: producers write x = h * gain and per-row sums of squares ssq [rows][norm_chunks(d)]; the consumer of the
// following GEMM multiplies rsqrt(sum(ssq)/d + eps) back in (a per-row scalar commutes with the GEMM).
int norm_chunks(int d);
template <typename T>
void launch_embed_norm(const T* embed, const int32_t* tokens, const RowTables& t, const float* gain, float* h, typename Act<T>::x_t* x, float* ssq, int rows,
                       int d, int vocab, hipStream_t st);
// h += sum_s part[s]; x = h * gain; ssq
template <typename T>
void launch_reduce_residual_norm(const float* part, int splits, float* h, const float* gain, T* x, float* ssq, int rows, int d, hipStream_t st);
// act = silu(gate) * up from rinv * part [splits][rows][2*ffn]
template <typename T>
void launch_silu_mul(const float* part, int splits, const float* ssq, int d, float eps, T* act, int rows, int ffn, hipStream_t st);
// rinv * part -> rotary embedding of Q and K; Q -> q [rows, n_q*hd] row-major; K, V -> cache[slot][pos]
template <typename T>
void launch_rope_kv(const float* part, int splits, const float* ssq, int d, float eps, const RowTables& t, const SeqMeta& meta, T* q,
                    T* kcache, T* vcache, size_t slot_stride, size_t head_stride, int rows, int n_q, int n_kv, int hd, hipStream_t st);
// softmax(q k^T / sqrt(hd)) v over keys [0, n_keys) of the row's slot; q row-major, out in the activation layout [rows, n_q*hd]
// (out_tiled) or row-major.  fp32 cache: row-major [pos][n_kv*hd] per slot (head_stride unused); bf16 cache: per (slot, kv head)
// a region of head_stride elements in the fragment tiling below.
template <typename T>
void launch_attention(const T* q, const T* kcache, const T* vcache, size_t slot_stride, size_t head_stride, const AttnMeta& meta, T* out,
                      bool out_tiled, int rows, int max_seq_rows, int n_q, int n_kv, int hd, hipStream_t st);
// bf16 models: q and the KV cache hold IEEE half; the output goes to out_tiles (fragment tiles [rows, n_q*hd] in half: the O
// projection's input) if that is given, else to out_rows (row-major bf16)
void launch_attention_f16(const f16_t* q, const f16_t* kcache, const f16_t* vcache, size_t slot_stride, size_t head_stride, const AttnMeta& meta,
                          op_t* out_tiles, bf16_t* out_rows, int rows, int max_seq_rows, int n_q, int n_kv, int hd, hipStream_t st);
// test helper of dlm_attention: K, V [T, n_kv, hd] row-major bf16 -> the tiled half-precision cache layout of one slot; q -> half
void launch_pack_kv(const bf16_t* k, const bf16_t* v, f16_t* kt, f16_t* vt, int T, int n_kv, int hd, size_t head_stride, hipStream_t st);
void launch_to_f16(const bf16_t* src, f16_t* dst, size_t n, hipStream_t st);

struct StatsOut {
  float *max_logit, *lse, *entropy, *kl, *conf;
  int32_t* argmax;
};
struct StatsRows {
  const int64_t* prev_row;  // DEVICE [rows] or null: offset (elements) of the row's p^prev logits in prev_base, -1 = none
  const int64_t* save_row;  // DEVICE [rows] or null: offset where the row's logits are copied, -1 = none
  const void* prev_base;
  void* save_base;
  const float* prev_lse;    // indexed by prev_row / vocab; null = recompute from the logits
  float* save_lse;          // indexed by save_row / vocab
};
size_t stats_workspace_bytes(int rows);
constexpr size_t STATS_STATE_BYTES = 32;  // one online-softmax state (stats_part.h)
// Finishes rows whose online-softmax states were written per column group by an EPI_STATS GEMM: parts [rows][nparts] states
// (stats_part.h), merged in a fixed order.
void launch_stats_merge(const void* parts, int rows, int nparts, int vocab, const StatsRows& sr, const StatsOut& o, hipStream_t st);
template <typename T>
void launch_vocab_stats(const T* logits, int rows, int vocab, int mask_id, const StatsRows& sr, const StatsOut& o, void* workspace, hipStream_t st);

void launch_block_boundary(const float* I, const float* H, const BoundaryMeta& meta, int n_seqs, dlm_boundary_params p, int32_t* L_out,
                           float* S_out, float* margin_out, hipStream_t st);
template <typename T>
void launch_select(const T* logits, int vocab, const float* lse, const float* conf, const int32_t* argmax, int32_t* tokens,
                   const SelectMeta& meta, int n_seqs, int mask_id, dlm_select_params p, int apply, uint8_t* sel, int32_t* nsel,
                   float* margin, hipStream_t st);
