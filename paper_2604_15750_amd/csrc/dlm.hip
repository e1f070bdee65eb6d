// C ABI of libdlm: argument validation, model / state ownership, and the host-side sequencing of
// one denoising step.  No kernel code here.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "common.h"
#include <cstdlib>

// ---- errors ------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

int dlm_fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}
extern "C" const char* dlm_last_error(void) { return g_err; }

#define REQUIRE(cond, code, ...) \
  do {                           \
    if (!(cond)) return dlm_fail(code, __VA_ARGS__); \
  } while (0)

// ---- file-scope scratch of the entry point that allocates nothing (dlm_vocab_stats_static) -------------
// The partial online-softmax states of the vocabulary reduction, one per (row, chunk): what dlm_vocab_stats takes as its
// workspace argument.  Every GPU the library runs on holds its own copy of the array, at its own address, until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress: kernels and copies get the resolved pointer.
constexpr int STATIC_STATS_MAX_ROWS = 4096;
constexpr size_t STATIC_STATS_BYTES = (size_t)STATIC_STATS_MAX_ROWS * 1024;  // 32 chunks x 32 bytes per row: 4 MiB
static __device__ __align__(256) unsigned char scratch[STATIC_STATS_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device, resolved once per device with that device current.
int scratch_address(void** out) {
  int dev = -1;
  DLM_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return dlm_fail(DLM_ECAPACITY, "device ordinal %d beyond the %d this library keeps scratch addresses for", dev, MAX_DEVICES);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    DLM_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return dlm_fail(DLM_EHIP, "hipGetSymbolAddress returned a null address for the scratch array");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return DLM_OK;
}

size_t elem_size(int dtype) { return dtype == DLM_BF16 ? 2 : 4; }

struct DevBuf {  // owned device allocation
  void* p = nullptr;
  ~DevBuf() { if (p) (void)hipFree(p); }
  int alloc(size_t bytes) {
    if (hipMalloc(&p, bytes ? bytes : 16) != hipSuccess) { p = nullptr; (void)hipGetLastError(); return dlm_fail(DLM_ENOMEM, "hipMalloc of %zu bytes failed", bytes); }
    return DLM_OK;
  }
  DevBuf() = default;
  DevBuf(const DevBuf&) = delete;
  DevBuf& operator=(const DevBuf&) = delete;
};

__global__ void to_f32_kernel(const void* src, float* dst, int n, int dtype) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = dtype == DLM_BF16 ? (float)((const bf16_t*)src)[i] : ((const float*)src)[i];
}

}  // namespace

struct dlm_model {
  dlm_config cfg;
  DevBuf embed, final_norm, lm_head;
  std::vector<DevBuf> wqkv, wo, w_gate_up, w_down, norm1, norm2;
  // second copies of the layer matrices in the step-major layout of the kernel that serves narrow passes (empty when that
  // kernel has no such layout for the shape): 0.44 GB per layer of an 8B model, 14 GB of 288 in all
  std::vector<DevBuf> w_steps[4];  // QKV, O, gate/up, down
  int steps_ct[4] = {0, 0, 0, 0};
};

thread_local LaunchStamp g_launch_stamp = {nullptr, nullptr};

enum { PC_QKV = 0, PC_O = 1, PC_GATE_UP = 2, PC_DOWN = 3, PC_LM_HEAD = 4, PC_ATTENTION = 5, PC_STATS = 6, PC_OTHER = 7 };
struct Profile {
  unsigned mask = 0;  // classes whose launches are bracketed by events
  static constexpr int NC = 8;
  double ms[NC] = {};
  int64_t launches[NC] = {};
  struct Span { hipEvent_t a, b; int cls; };
  std::vector<Span> pending;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;
};

struct dlm_state {
  const dlm_model* m;
  int max_seqs, max_seq_len, max_rows, max_rows_pad, max_lookahead;
  size_t slot_stride;   // elements per slot per layer in the KV cache
  size_t head_stride;   // bf16: elements per (slot, kv head) region of the tiled cache
  size_t layer_stride;  // elements per layer
  DevBuf kcache, vcache, prev_logits, prev_lse;
  DevBuf h, x, x2, act, q, part, stats_ws, ssq, counters;
  DevBuf row_seq, row_pos, row_tok, row_slot, rope_cos, rope_sin, prev_row, save_row;
  std::vector<int> kv_len, covered_end, prev_cur, prev_base, prev_count;  // covered_end: positions [0, covered_end) hold K and V of some pass
  size_t part_elems;
  bool fuse_stats = true;  // passes that qualify take their statistics from the LM head's epilogue (dlm_state_fuse_stats)
  Profile prof;
};

namespace {

// Times the launches of one kernel class when profiling is on.  A GEMM class is one kernel per scope: its launch stamps the
// two events itself (kernel start and end, nothing added to the queue).  The other classes are bracketed by recorded events.
struct ProfScope {
  Profile& p; hipStream_t st; int cls; bool on, stamped; hipEvent_t a = nullptr, b = nullptr;
  ProfScope(Profile& p_, hipStream_t st_, int cls_, int n_launches = 1)
      : p(p_), st(st_), cls(cls_), on((p_.mask >> cls_) & 1u), stamped(cls_ <= PC_LM_HEAD && n_launches == 1) {
    if (!on) return;
    p.launches[cls] += n_launches;
    if (p.pool.empty()) { (void)hipEventCreate(&a); (void)hipEventCreate(&b); }
    else { a = p.pool.back().first; b = p.pool.back().second; p.pool.pop_back(); }
    if (stamped) g_launch_stamp = LaunchStamp{a, b};
    else (void)hipEventRecord(a, st);
  }
  ~ProfScope() {
    if (!on) return;
    if (stamped && g_launch_stamp.start == a) {  // no launch took the events: record them, or reading them would fail
      g_launch_stamp = LaunchStamp{nullptr, nullptr};
      (void)hipEventRecord(a, st);
      stamped = false;
    }
    if (!stamped) (void)hipEventRecord(b, st);
    p.pending.push_back({a, b, cls});
  }
};

template <typename T>
int copy_plain(DevBuf& dst, const void* src, size_t n, hipStream_t st) {
  int rc = dst.alloc(n * sizeof(T));
  if (rc) return rc;
  DLM_HIP(hipMemcpyAsync(dst.p, src, n * sizeof(T), hipMemcpyDeviceToDevice, st));
  return DLM_OK;
}

int copy_gain(DevBuf& dst, const void* src, int n, int dtype, hipStream_t st) {
  int rc = dst.alloc((size_t)n * 4);
  if (rc) return rc;
  to_f32_kernel<<<(n + 255) / 256, 256, 0, st>>>(src, (float*)dst.p, n, dtype);
  return DLM_OK;
}

int copy_matrix(DevBuf& dst, const void* src, int N, int K, int dtype, hipStream_t st, int perm = PERM_NONE, int perm_param = 0) {
  int rc = dst.alloc((size_t)N * K * elem_size(dtype));
  if (rc) return rc;
  if (dtype == DLM_BF16) launch_pack_weight((const bf16_t*)src, (op_t*)dst.p, N, K, perm, perm_param, st);
  else DLM_HIP(hipMemcpyAsync(dst.p, src, (size_t)N * K * 4, hipMemcpyDeviceToDevice, st));
  return DLM_OK;
}

bool mult32(int v) { return v > 0 && v % 32 == 0; }

}  // namespace

extern "C" int dlm_model_create(const dlm_config* cfg, const dlm_weights* w, void* stream, dlm_model** out) {
  REQUIRE(cfg && w && out, DLM_EINVAL, "dlm_model_create: null argument");
  *out = nullptr;
  REQUIRE(cfg->dtype == DLM_F32 || cfg->dtype == DLM_BF16, DLM_EINVAL, "dlm_model_create: dtype %d", cfg->dtype);
  REQUIRE(cfg->n_layers >= 1 && cfg->d_model >= 1 && cfg->n_q_heads >= 1 && cfg->n_kv_heads >= 1 && cfg->d_ffn >= 1 && cfg->vocab >= 2,
          DLM_ESHAPE, "dlm_model_create: non-positive dimension");
  REQUIRE(cfg->head_dim == 32 || cfg->head_dim == 64 || cfg->head_dim == 128, DLM_ESHAPE, "dlm_model_create: head_dim %d not in {32,64,128}", cfg->head_dim);
  REQUIRE(cfg->n_q_heads % cfg->n_kv_heads == 0, DLM_ESHAPE, "dlm_model_create: n_q_heads %% n_kv_heads != 0");
  REQUIRE(cfg->mask_id >= 0 && cfg->mask_id < cfg->vocab, DLM_EINVAL, "dlm_model_create: mask_id out of range");
  REQUIRE(cfg->d_model % 4 == 0 && cfg->d_ffn % 4 == 0, DLM_ESHAPE, "dlm_model_create: d_model and d_ffn must be multiples of 4");
  if (cfg->dtype == DLM_BF16)  // whole 128-column output tiles (64 + 64 for the gated FFN); the LM head may end on a 32-column group
    REQUIRE(cfg->d_model % 256 == 0 && cfg->d_ffn % 64 == 0 && mult32(cfg->vocab) && (cfg->n_q_heads * cfg->head_dim) % 128 == 0 &&
                (cfg->n_kv_heads * cfg->head_dim) % 128 == 0,
            DLM_ESHAPE, "dlm_model_create: bf16 needs d_model %% 256 == 0, n_q*head_dim and n_kv*head_dim %% 128 == 0, d_ffn %% 64 == 0, vocab %% 32 == 0");
  REQUIRE(w->embed && w->wqkv && w->wo && w->w_gate_up && w->w_down && w->norm1 && w->norm2 && w->final_norm && w->lm_head,
          DLM_EINVAL, "dlm_model_create: null weight pointer");
  for (int l = 0; l < cfg->n_layers; ++l)
    REQUIRE(w->wqkv[l] && w->wo[l] && w->w_gate_up[l] && w->w_down[l] && w->norm1[l] && w->norm2[l], DLM_EINVAL,
            "dlm_model_create: null weight pointer in layer %d", l);

  hipStream_t st = (hipStream_t)stream;
  { void* sp = nullptr; (void)scratch_address(&sp); }  // set-up on this device: callers of dlm_vocab_stats_static find the address resolved
  dlm_model* m = new (std::nothrow) dlm_model();
  REQUIRE(m, DLM_ENOMEM, "dlm_model_create: host allocation failed");
  m->cfg = *cfg;
  const int L = cfg->n_layers, d = cfg->d_model, dt = cfg->dtype;
  const int qkv = (cfg->n_q_heads + 2 * cfg->n_kv_heads) * cfg->head_dim, qd = cfg->n_q_heads * cfg->head_dim;
  m->wqkv = std::vector<DevBuf>(L); m->wo = std::vector<DevBuf>(L); m->w_gate_up = std::vector<DevBuf>(L);
  m->w_down = std::vector<DevBuf>(L); m->norm1 = std::vector<DevBuf>(L); m->norm2 = std::vector<DevBuf>(L);
  int rc = DLM_OK;
  auto step = [&](int r) { if (rc == DLM_OK) rc = r; return rc == DLM_OK; };
  if (dt == DLM_BF16) step(copy_plain<bf16_t>(m->embed, w->embed, (size_t)cfg->vocab * d, st));
  else step(copy_plain<float>(m->embed, w->embed, (size_t)cfg->vocab * d, st));
  if (rc == DLM_OK) step(copy_gain(m->final_norm, w->final_norm, d, dt, st));
  if (rc == DLM_OK) step(copy_matrix(m->lm_head, w->lm_head, cfg->vocab, d, dt, st));
  for (int l = 0; l < L && rc == DLM_OK; ++l) {
    step(copy_matrix(m->wqkv[l], w->wqkv[l], qkv, d, dt, st, PERM_ROTARY, cfg->head_dim)) && step(copy_matrix(m->wo[l], w->wo[l], d, qd, dt, st)) &&
        step(copy_matrix(m->w_gate_up[l], w->w_gate_up[l], 2 * cfg->d_ffn, d, dt, st, PERM_GATED, cfg->d_ffn)) &&
        step(copy_matrix(m->w_down[l], w->w_down[l], d, cfg->d_ffn, dt, st)) && step(copy_gain(m->norm1[l], w->norm1[l], d, dt, st)) &&
        step(copy_gain(m->norm2[l], w->norm2[l], d, dt, st));
  }
  // Second copies of the layer matrices in the step-major layout of the kernel that serves narrow passes (gemm_bf16_steps_ct),
  // unless the environment says DLM_W_STEPS=0.  They are an optimisation: a matrix whose copy does not fit goes without.
  if (rc == DLM_OK && dt == DLM_BF16 && !(getenv("DLM_W_STEPS") && atoi(getenv("DLM_W_STEPS")) == 0)) {
    const int shape[4][4] = {{qkv, d, PERM_ROTARY, cfg->head_dim}, {d, qd, PERM_NONE, 0}, {2 * cfg->d_ffn, d, PERM_GATED, cfg->d_ffn}, {d, cfg->d_ffn, PERM_NONE, 0}};
    const int kinds[4] = {EPI_QKV, EPI_RESID, EPI_SWIGLU, EPI_RESID};
    for (int k = 0; k < 4; ++k) {
      m->steps_ct[k] = gemm_bf16_steps_ct(shape[k][0], shape[k][1], kinds[k]);
      if (!m->steps_ct[k]) continue;
      m->w_steps[k] = std::vector<DevBuf>(L);
      for (int l = 0; l < L; ++l) {
        void* p = nullptr;
        if (hipMalloc(&p, (size_t)shape[k][0] * shape[k][1] * 2) != hipSuccess) {
          (void)hipGetLastError();
          (void)hipStreamSynchronize(st);  // the packing kernels of the earlier layers write into what is released next
          m->w_steps[k].clear();
          m->steps_ct[k] = 0;
          break;
        }
        m->w_steps[k][l].p = p;
        const void* src = k == 0 ? w->wqkv[l] : k == 1 ? w->wo[l] : k == 2 ? w->w_gate_up[l] : w->w_down[l];
        launch_pack_weight_steps((const bf16_t*)src, (op_t*)p, shape[k][0], shape[k][1], m->steps_ct[k], shape[k][2], shape[k][3], st);
      }
    }
  }
  if (rc != DLM_OK) { delete m; return rc; }
  *out = m;
  return DLM_OK;
}

extern "C" void dlm_model_destroy(dlm_model* m) { delete m; }

extern "C" int dlm_state_create(const dlm_model* m, int max_seqs, int max_seq_len, int max_rows, int max_lookahead, dlm_state** out) {
  REQUIRE(m && out, DLM_EINVAL, "dlm_state_create: null argument");
  *out = nullptr;
  REQUIRE(max_seqs >= 1 && max_seq_len >= 1 && max_rows >= 1 && max_lookahead >= 0, DLM_ECAPACITY, "dlm_state_create: non-positive size");
  REQUIRE(max_seqs <= DLM_MAX_SEQS, DLM_ECAPACITY, "dlm_state_create: max_seqs %d > %d", max_seqs, DLM_MAX_SEQS);
  const dlm_config& c = m->cfg;
  dlm_state* s = new (std::nothrow) dlm_state();
  REQUIRE(s, DLM_ENOMEM, "dlm_state_create: host allocation failed");
  s->m = m; s->max_seqs = max_seqs; s->max_seq_len = max_seq_len; s->max_rows = max_rows; s->max_lookahead = max_lookahead;
  s->max_rows_pad = (max_rows + 15) / 16 * 16;
  const size_t es = elem_size(c.dtype);
  const int kvw = c.n_kv_heads * c.head_dim, qd = c.n_q_heads * c.head_dim, qkv = qd + 2 * kvw;
  s->head_stride = (size_t)((max_seq_len + 31) / 32 * 32) * c.head_dim;
  s->slot_stride = c.dtype == DLM_BF16 ? s->head_stride * c.n_kv_heads : (size_t)max_seq_len * kvw;
  s->layer_stride = s->slot_stride * max_seqs;
  // split-K workspace: the largest [splits][rows][N] over the four per-layer GEMMs
  size_t pe = 0;
  const int shapes[4][3] = {{qkv, c.d_model, EPI_QKV}, {c.d_model, qd, EPI_RESID}, {2 * c.d_ffn, c.d_model, EPI_SWIGLU}, {c.d_model, c.d_ffn, EPI_RESID}};
  for (auto& sh : shapes) {
    int maxsp = 1;
    if (c.dtype == DLM_BF16)
      for (int mt = 1; mt <= (max_rows + 15) / 16; ++mt) {  // the split count depends on the rows only through their 16-row tiles
        const int sp = gemm_bf16_splits(mt * 16 < max_rows ? mt * 16 : max_rows, sh[0], sh[1], sh[2]);
        if (sp > maxsp) maxsp = sp;
      }
    size_t e = (size_t)maxsp * max_rows * sh[0];
    if (e > pe) pe = e;
  }
  s->part_elems = pe;
  const int xw = c.d_model > qd ? c.d_model : qd;
  const size_t look = (size_t)(max_lookahead ? max_lookahead : 1);
  int rc = DLM_OK;
  auto A = [&](DevBuf& b, size_t bytes) { if (rc == DLM_OK) rc = b.alloc(bytes); };
  A(s->kcache, s->layer_stride * c.n_layers * es);
  A(s->vcache, s->layer_stride * c.n_layers * es);
  A(s->prev_logits, (size_t)max_seqs * 2 * look * c.vocab * es);
  A(s->prev_lse, (size_t)max_seqs * 2 * look * 4);
  A(s->h, (size_t)max_rows * c.d_model * 4);
  A(s->x, (size_t)s->max_rows_pad * xw * es);
  A(s->x2, (size_t)s->max_rows_pad * xw * es);
  A(s->act, (size_t)s->max_rows_pad * c.d_ffn * es);
  A(s->q, (size_t)max_rows * qd * es);
  A(s->part, pe * 4);
  size_t stats_bytes = stats_workspace_bytes(max_rows);
  if (c.dtype == DLM_BF16) {  // or one state per row and column group of the LM head, for the passes that take the statistics from its epilogue
    const int fr = max_rows < GEMM_STATS_MAX_ROWS ? max_rows : GEMM_STATS_MAX_ROWS;
    for (int mt = 1; mt <= (fr + 15) / 16; ++mt) {
      const size_t b = (size_t)fr * gemm_bf16_stat_parts(mt * 16 < fr ? mt * 16 : fr, c.vocab) * STATS_STATE_BYTES;
      if (b > stats_bytes) stats_bytes = b;
    }
  }
  A(s->stats_ws, stats_bytes);
  const int ssq_chunks = c.dtype == DLM_BF16 ? c.d_model / 16 : norm_chunks(c.d_model);
  A(s->ssq, (size_t)max_rows * ssq_chunks * 4);
  int n_counters = 1;
  if (c.dtype == DLM_BF16)
    for (auto& sh : shapes) { int k = gemm_bf16_counters(max_rows, sh[0]); if (k > n_counters) n_counters = k; }
  A(s->counters, (size_t)n_counters * 4);
  A(s->row_seq, (size_t)max_rows * 4); A(s->row_pos, (size_t)max_rows * 4); A(s->row_tok, (size_t)max_rows * 4); A(s->row_slot, (size_t)max_rows * 4);
  A(s->rope_cos, (size_t)max_rows * (c.head_dim / 2) * 4); A(s->rope_sin, (size_t)max_rows * (c.head_dim / 2) * 4);
  A(s->prev_row, (size_t)max_rows * 8); A(s->save_row, (size_t)max_rows * 8);
  if (rc == DLM_OK) {
    // padding rows of the tiled activations are read by the matrix cores: keep them finite
    // cache positions beyond a sequence's keys are multiplied by zero probabilities: keep them finite too
    hipError_t e = hipMemset(s->x.p, 0, (size_t)s->max_rows_pad * xw * es);
    if (e == hipSuccess) e = hipMemset(s->kcache.p, 0, s->layer_stride * c.n_layers * es);
    if (e == hipSuccess) e = hipMemset(s->vcache.p, 0, s->layer_stride * c.n_layers * es);
    if (e == hipSuccess) e = hipMemset(s->x2.p, 0, (size_t)s->max_rows_pad * xw * es);
    if (e == hipSuccess) e = hipMemset(s->act.p, 0, (size_t)s->max_rows_pad * c.d_ffn * es);
    if (e == hipSuccess) e = hipMemset(s->counters.p, 0, (size_t)n_counters * 4);
    if (e != hipSuccess) rc = dlm_fail(DLM_EHIP, "dlm_state_create: hipMemset: %s", hipGetErrorString(e));
  }
  if (rc != DLM_OK) { delete s; return rc; }
  s->kv_len.assign(max_seqs, 0); s->covered_end.assign(max_seqs, 0); s->prev_cur.assign(max_seqs, 0); s->prev_base.assign(max_seqs, 0); s->prev_count.assign(max_seqs, 0);
  *out = s;
  return DLM_OK;
}

extern "C" void dlm_state_destroy(dlm_state* s) {
  if (!s) return;
  for (auto& sp : s->prof.pending) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
  for (auto& pr : s->prof.pool) { (void)hipEventDestroy(pr.first); (void)hipEventDestroy(pr.second); }
  delete s;
}

extern "C" int dlm_state_reset(dlm_state* s, int slot) {
  REQUIRE(s, DLM_EINVAL, "dlm_state_reset: null state");
  REQUIRE(slot >= 0 && slot < s->max_seqs, DLM_EINVAL, "dlm_state_reset: slot %d out of range", slot);
  s->kv_len[slot] = 0; s->covered_end[slot] = 0; s->prev_count[slot] = 0; s->prev_base[slot] = 0;
  return DLM_OK;
}

extern "C" int dlm_state_kv_len(const dlm_state* s, int slot) {
  REQUIRE(s, DLM_EINVAL, "dlm_state_kv_len: null state");
  REQUIRE(slot >= 0 && slot < s->max_seqs, DLM_EINVAL, "dlm_state_kv_len: slot %d out of range", slot);
  return s->kv_len[slot];
}

extern "C" int dlm_state_fuse_stats(dlm_state* s, int enable) {
  REQUIRE(s, DLM_EINVAL, "dlm_state_fuse_stats: null state");
  s->fuse_stats = enable != 0;
  return DLM_OK;
}

extern "C" int dlm_profile_enable(dlm_state* s, unsigned class_mask) {
  REQUIRE(s, DLM_EINVAL, "dlm_profile_enable: null state");
  s->prof.mask = class_mask & ((1u << Profile::NC) - 1);
  return DLM_OK;
}

extern "C" int dlm_profile_read(dlm_state* s, int n, double* ms_out, int64_t* launches_out, int reset) {
  REQUIRE(s && ms_out && launches_out, DLM_EINVAL, "dlm_profile_read: null argument");
  Profile& p = s->prof;
  for (auto& sp : p.pending) {
    DLM_HIP(hipEventSynchronize(sp.b));
    float ms = 0.f;
    DLM_HIP(hipEventElapsedTime(&ms, sp.a, sp.b));
    p.ms[sp.cls] += ms;
    p.pool.push_back({sp.a, sp.b});
  }
  p.pending.clear();
  for (int i = 0; i < n; ++i) { ms_out[i] = i < Profile::NC ? p.ms[i] : 0.0; launches_out[i] = i < Profile::NC ? p.launches[i] : 0; }
  if (reset) for (int i = 0; i < Profile::NC; ++i) { p.ms[i] = 0; p.launches[i] = 0; }
  return DLM_OK;
}

// ---- dlm_step ------------------------------------------------------------------------------------
namespace {

// fp32 model: plain GEMMs with the row-wise glue in kernels of their own
int run_step_f32(dlm_state* s, const dlm_step_desc* d, const SeqMeta& meta, const StatsMeta& sm, const AttnMeta& am, int rows, int max_seq_rows,
                 hipStream_t st) {
  typedef float T;
  const dlm_model* m = s->m;
  const dlm_config& c = m->cfg;
  const int dm = c.d_model, hd = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads, qd = nq * hd, ffn = c.d_ffn;
  RowTables t{(int32_t*)s->row_seq.p, (int32_t*)s->row_pos.p, (int32_t*)s->row_tok.p, (int32_t*)s->row_slot.p, (float*)s->rope_cos.p, (float*)s->rope_sin.p,
              (int64_t*)s->prev_row.p, (int64_t*)s->save_row.p};
  float* h = (float*)s->h.p;
  T *x = (T*)s->x.p, *x2 = (T*)s->x2.p, *act = (T*)s->act.p, *q = (T*)s->q.p;
  float* part = (float*)s->part.p;
  float* ssq = (float*)s->ssq.p;
  Profile& pf = s->prof;
  const RowScale none{nullptr, 0, 0.f, 0.f};
  auto gemm = [&](int cls, const float* a, const void* w, int N, int K) {
    ProfScope ps(pf, st, cls);
    launch_gemm_f32(a, (const float*)w, part, rows, N, K, none, st);
  };
  {
    ProfScope ps(pf, st, PC_OTHER, 2);
    launch_prepare(meta, sm, t, rows, c.vocab, hd, c.rope_theta, st);
    launch_embed_norm<T>((const T*)m->embed.p, d->tokens, t, (const float*)m->norm1[0].p, h, x, ssq, rows, dm, c.vocab, st);
  }
  for (int l = 0; l < c.n_layers; ++l) {
    T* kc = (T*)s->kcache.p + s->layer_stride * l;
    T* vc = (T*)s->vcache.p + s->layer_stride * l;
    gemm(PC_QKV, x, m->wqkv[l].p, qd + 2 * nkv * hd, dm);
    { ProfScope ps(pf, st, PC_OTHER);
      launch_rope_kv<T>(part, 1, ssq, dm, c.rms_eps, t, meta, q, kc, vc, s->slot_stride, s->head_stride, rows, nq, nkv, hd, st); }
    { ProfScope ps(pf, st, PC_ATTENTION);
      launch_attention<T>(q, kc, vc, s->slot_stride, s->head_stride, am, x2, true, rows, max_seq_rows, nq, nkv, hd, st); }
    gemm(PC_O, x2, m->wo[l].p, dm, qd);
    { ProfScope ps(pf, st, PC_OTHER);
      launch_reduce_residual_norm<T>(part, 1, h, (const float*)m->norm2[l].p, x, ssq, rows, dm, st); }
    gemm(PC_GATE_UP, x, m->w_gate_up[l].p, 2 * ffn, dm);
    { ProfScope ps(pf, st, PC_OTHER);
      launch_silu_mul<T>(part, 1, ssq, dm, c.rms_eps, act, rows, ffn, st); }
    gemm(PC_DOWN, act, m->w_down[l].p, dm, ffn);
    { ProfScope ps(pf, st, PC_OTHER);
      const float* g = l + 1 < c.n_layers ? (const float*)m->norm1[l + 1].p : (const float*)m->final_norm.p;
      launch_reduce_residual_norm<T>(part, 1, h, g, x, ssq, rows, dm, st); }
  }
  {
    ProfScope ps(pf, st, PC_LM_HEAD);
    const RowScale rs{ssq, norm_chunks(dm), 1.f / (float)dm, c.rms_eps};
    launch_gemm_f32((const float*)x, (const float*)m->lm_head.p, (float*)d->logits, rows, c.vocab, dm, rs, st);
  }
  {
    ProfScope ps(pf, st, PC_STATS);
    StatsRows sr{t.prev_row, t.save_row, s->prev_logits.p, s->prev_logits.p, (const float*)s->prev_lse.p, (float*)s->prev_lse.p};
    StatsOut so{d->max_logit, d->lse, d->entropy, d->kl, d->conf, d->argmax};
    launch_vocab_stats<T>((const T*)d->logits, rows, c.vocab, c.mask_id, sr, so, s->stats_ws.p, st);
  }
  return DLM_OK;
}

// bf16 models: five launches per layer; every row-wise step between two GEMMs runs in the producing GEMM's epilogue
int run_step_bf16(dlm_state* s, const dlm_step_desc* d, const SeqMeta& meta, const StatsMeta& sm, const AttnMeta& am, int rows,
                  int max_seq_rows, hipStream_t st) {
  typedef bf16_t T;
  const dlm_model* m = s->m;
  const dlm_config& c = m->cfg;
  const int dm = c.d_model, hd = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads, qd = nq * hd, ffn = c.d_ffn;
  RowTables t{(int32_t*)s->row_seq.p, (int32_t*)s->row_pos.p, (int32_t*)s->row_tok.p, (int32_t*)s->row_slot.p, (float*)s->rope_cos.p, (float*)s->rope_sin.p,
              (int64_t*)s->prev_row.p, (int64_t*)s->save_row.p};
  float* h = (float*)s->h.p;
  op_t *x = (op_t*)s->x.p, *x2 = (op_t*)s->x2.p, *act = (op_t*)s->act.p;  // GEMM inputs: IEEE half in fragment tiles (common.h)
  f16_t* q = (f16_t*)s->q.p;  // Q and the KV cache hold IEEE half (common.h)
  float* ssq = (float*)s->ssq.p;
  Profile& pf = s->prof;
  GemmEpi base;
  memset(&base, 0, sizeof base);
  base.part = (float*)s->part.p;
  base.counters = (int*)s->counters.p;
  // every layer GEMM of this pass must fit the partial-tile workspace the state was created with
  {
    const int shapes[4][3] = {{qd + 2 * nkv * hd, dm, EPI_QKV}, {dm, qd, EPI_RESID}, {2 * ffn, dm, EPI_SWIGLU}, {dm, ffn, EPI_RESID}};
    for (auto& sh : shapes)
      if ((size_t)gemm_bf16_splits(rows, sh[0], sh[1], sh[2]) * rows * sh[0] > s->part_elems)
        return dlm_fail(DLM_ECAPACITY, "dlm_step: split-K workspace too small for %d rows x %d columns", rows, sh[0]);
  }
  auto gemm = [&](int cls, const op_t* a, const void* w, int N, int K, const GemmEpi& e) {
    ProfScope ps(pf, st, cls);
    launch_gemm_bf16(a, (const op_t*)w, rows, N, K, e, st);
  };
  {
    ProfScope ps(pf, st, PC_OTHER, 2);
    launch_prepare(meta, sm, t, rows, c.vocab, hd, c.rope_theta, st);
    launch_embed_norm<T>((const T*)m->embed.p, d->tokens, t, (const float*)m->norm1[0].p, h, x, ssq, rows, dm, c.vocab, st);
  }
  // chunks of the row sums of squares the next consumer reads: the embedding's, then those of the GEMM that produced them
  int nch = norm_chunks(dm);
  for (int l = 0; l < c.n_layers; ++l) {
    f16_t* kc = (f16_t*)s->kcache.p + s->layer_stride * l;
    f16_t* vc = (f16_t*)s->vcache.p + s->layer_stride * l;
    {
      GemmEpi e = base;
      e.kind = EPI_QKV;
      e.rs = RowScale{ssq, nch, 1.f / (float)dm, c.rms_eps};
      e.row_pos = t.row_pos; e.row_slot = t.row_slot; e.rope_cos = t.rope_cos; e.rope_sin = t.rope_sin;
      e.q = q; e.kcache = kc; e.vcache = vc; e.slot_stride = s->slot_stride; e.head_stride = s->head_stride;
      e.n_q = nq; e.n_kv = nkv; e.hd = hd;
      if (m->steps_ct[0]) { e.w_steps = (const op_t*)m->w_steps[0][l].p; e.w_steps_ct = m->steps_ct[0]; }
      gemm(PC_QKV, x, m->wqkv[l].p, qd + 2 * nkv * hd, dm, e);
    }
    { ProfScope ps(pf, st, PC_ATTENTION);
      launch_attention_f16(q, kc, vc, s->slot_stride, s->head_stride, am, x2, nullptr, rows, max_seq_rows, nq, nkv, hd, st); }
    {
      GemmEpi e = base;
      e.kind = EPI_RESID;
      e.h = h; e.gain = (const float*)m->norm2[l].p; e.x = x; e.ssq_out = ssq;
      if (m->steps_ct[1]) { e.w_steps = (const op_t*)m->w_steps[1][l].p; e.w_steps_ct = m->steps_ct[1]; }
      gemm(PC_O, x2, m->wo[l].p, dm, qd, e);
      nch = gemm_bf16_ssq_chunks(rows, dm, qd);
    }
    {
      GemmEpi e = base;
      e.kind = EPI_SWIGLU;
      e.rs = RowScale{ssq, nch, 1.f / (float)dm, c.rms_eps};
      e.act = act; e.ffn = ffn;
      if (m->steps_ct[2]) { e.w_steps = (const op_t*)m->w_steps[2][l].p; e.w_steps_ct = m->steps_ct[2]; }
      gemm(PC_GATE_UP, x, m->w_gate_up[l].p, 2 * ffn, dm, e);
    }
    {
      GemmEpi e = base;
      e.kind = EPI_RESID;
      e.h = h; e.gain = l + 1 < c.n_layers ? (const float*)m->norm1[l + 1].p : (const float*)m->final_norm.p;
      e.x = x; e.ssq_out = ssq;
      if (m->steps_ct[3]) { e.w_steps = (const op_t*)m->w_steps[3][l].p; e.w_steps_ct = m->steps_ct[3]; }
      gemm(PC_DOWN, act, m->w_down[l].p, dm, ffn, e);
      nch = gemm_bf16_ssq_chunks(rows, dm, ffn);
    }
  }
  // A pass that compares no row with a retained distribution and retains none (every in-block pass) needs no second trip over
  // its logits: the LM head's epilogue leaves one online-softmax state per row and column group, and a small merge finishes them.
  bool fused = s->fuse_stats && rows <= GEMM_STATS_MAX_ROWS;
  for (int b = 0; b < meta.n_seqs; ++b) fused = fused && sm.kl_count[b] == 0 && sm.save_count[b] == 0;
  StatsRows sr{t.prev_row, t.save_row, s->prev_logits.p, s->prev_logits.p, (const float*)s->prev_lse.p, (float*)s->prev_lse.p};
  StatsOut so{d->max_logit, d->lse, d->entropy, d->kl, d->conf, d->argmax};
  {
    GemmEpi e = base;
    e.kind = fused ? EPI_STATS : EPI_DIRECT;
    e.rs = RowScale{ssq, nch, 1.f / (float)dm, c.rms_eps};
    e.out_bf16 = (T*)d->logits;
    e.stat_parts = s->stats_ws.p;
    e.skip_col = c.mask_id;
    gemm(PC_LM_HEAD, x, m->lm_head.p, c.vocab, dm, e);
  }
  {
    ProfScope ps(pf, st, PC_STATS);
    if (fused) launch_stats_merge(s->stats_ws.p, rows, gemm_bf16_stat_parts(rows, c.vocab), c.vocab, sr, so, st);
    else launch_vocab_stats<T>((const T*)d->logits, rows, c.vocab, c.mask_id, sr, so, s->stats_ws.p, st);
  }
  return DLM_OK;
}

}  // namespace

extern "C" int dlm_step(dlm_state* s, const dlm_step_desc* d, void* stream) {
  REQUIRE(s && d, DLM_EINVAL, "dlm_step: null argument");
  REQUIRE(d->row_offsets && d->span_start && d->commit_len && d->tok_start && d->tokens && d->logits && d->max_logit && d->lse &&
              d->entropy && d->kl && d->conf && d->argmax,
          DLM_EINVAL, "dlm_step: null pointer in descriptor");
  REQUIRE((d->kl_first != nullptr) == (d->kl_count != nullptr) && (d->save_first != nullptr) == (d->save_count != nullptr), DLM_EINVAL,
          "dlm_step: kl_first/kl_count (save_first/save_count) must be given together");
  const int n = d->n_seqs;
  REQUIRE(n >= 1, DLM_EINVAL, "dlm_step: n_seqs %d < 1", n);
  REQUIRE(n <= s->max_seqs, DLM_ECAPACITY, "dlm_step: n_seqs %d > max_seqs %d", n, s->max_seqs);
  REQUIRE(d->row_offsets[0] == 0, DLM_EINVAL, "dlm_step: row_offsets[0] != 0");
  const dlm_config& c = s->m->cfg;
  SeqMeta meta; StatsMeta sm; AttnMeta am;
  memset(&meta, 0, sizeof meta); memset(&sm, 0, sizeof sm); memset(&am, 0, sizeof am);
  meta.n_seqs = am.n_seqs = n;
  bool used[DLM_MAX_SEQS] = {};
  int max_seq_rows = 0;
  const size_t look = (size_t)(s->max_lookahead ? s->max_lookahead : 1);
  for (int b = 0; b < n; ++b) {
    const int slot = d->slot ? d->slot[b] : b;
    REQUIRE(slot >= 0 && slot < s->max_seqs, DLM_EINVAL, "dlm_step: slot %d of sequence %d out of range", slot, b);
    REQUIRE(!used[slot], DLM_EINVAL, "dlm_step: slot %d given twice", slot);
    used[slot] = true;
    const int r0 = d->row_offsets[b], r1 = d->row_offsets[b + 1], nr = r1 - r0;
    REQUIRE(nr >= 1, DLM_EINVAL, "dlm_step: row_offsets not increasing at sequence %d", b);
    REQUIRE(r1 <= s->max_rows, DLM_ECAPACITY, "dlm_step: %d rows > max_rows %d", r1, s->max_rows);
    REQUIRE(d->span_start[b] == s->kv_len[slot], DLM_EINVAL, "dlm_step: span_start %d != cached length %d (sequence %d)", d->span_start[b], s->kv_len[slot], b);
    REQUIRE(d->span_start[b] + nr <= s->max_seq_len, DLM_ECAPACITY, "dlm_step: span end %d > max_seq_len %d", d->span_start[b] + nr, s->max_seq_len);
    REQUIRE(d->commit_len[b] >= 0 && d->commit_len[b] <= nr, DLM_EINVAL, "dlm_step: commit_len %d outside the span (sequence %d)", d->commit_len[b], b);
    REQUIRE(d->tok_start[b] >= 0, DLM_EINVAL, "dlm_step: negative tok_start");
    meta.row_off[b] = am.row_off[b] = r0;
    meta.row_off[b + 1] = am.row_off[b + 1] = r1;
    meta.span_start[b] = d->span_start[b];
    meta.slot[b] = am.slot[b] = slot;
    meta.tok_start[b] = d->tok_start[b];
    const int suffix = d->suffix_len ? d->suffix_len[b] : 0;
    REQUIRE(suffix >= 0 && d->span_start[b] + nr + suffix <= (suffix ? s->covered_end[slot] : s->max_seq_len), DLM_EINVAL,
            "dlm_step: suffix of %d positions after the span of sequence %d reaches beyond the %d positions an earlier pass has covered", suffix, b,
            s->covered_end[slot]);
    am.n_keys[b] = d->span_start[b] + nr + suffix;
    if (nr > max_seq_rows) max_seq_rows = nr;
    const int kc = d->kl_count ? d->kl_count[b] : 0, kf = d->kl_count ? d->kl_first[b] : 0;
    const int sc = d->save_count ? d->save_count[b] : 0, sf = d->save_count ? d->save_first[b] : 0;
    REQUIRE(kc >= 0 && kf >= 0 && kf + kc <= nr, DLM_EINVAL, "dlm_step: kl rows [%d,+%d) outside the span (sequence %d)", kf, kc, b);
    REQUIRE(sc >= 0 && sf >= 0 && sf + sc <= nr, DLM_EINVAL, "dlm_step: save rows [%d,+%d) outside the span (sequence %d)", sf, sc, b);
    REQUIRE(sc <= s->max_lookahead, DLM_ECAPACITY, "dlm_step: save_count %d > max_lookahead %d", sc, s->max_lookahead);
    sm.kl_first[b] = kf; sm.kl_count[b] = kc; sm.save_first[b] = sf; sm.save_count[b] = sc;
    if (kc > 0) {
      const int p0 = d->span_start[b] + kf - s->prev_base[slot];
      REQUIRE(p0 >= 0 && p0 + kc <= s->prev_count[slot], DLM_EINVAL,
              "dlm_step: kl rows at positions [%d,+%d) have no retained p^prev (retained: [%d,+%d))", d->span_start[b] + kf, kc,
              s->prev_base[slot], s->prev_count[slot]);
      sm.prev_off[b] = (int64_t)(((size_t)slot * 2 + s->prev_cur[slot]) * look + p0) * c.vocab;
    }
    if (sc > 0) sm.save_off[b] = (int64_t)(((size_t)slot * 2 + (1 - s->prev_cur[slot])) * look) * c.vocab;
  }
  const int rows = d->row_offsets[n];
  hipStream_t st = (hipStream_t)stream;
  int rc = c.dtype == DLM_BF16 ? run_step_bf16(s, d, meta, sm, am, rows, max_seq_rows, st)
                               : run_step_f32(s, d, meta, sm, am, rows, max_seq_rows, st);
  if (rc != DLM_OK) return rc;
  // a launch that the runtime refused (bad configuration, no resources) would otherwise go unnoticed until a later call
  DLM_HIP(hipGetLastError());
  for (int b = 0; b < n; ++b) {  // host bookkeeping: commit the prefix, flip the retained-logit buffers
    const int slot = meta.slot[b];
    s->kv_len[slot] += d->commit_len[b];
    if (am.row_off[b + 1] - am.row_off[b] + d->span_start[b] > s->covered_end[slot]) s->covered_end[slot] = am.row_off[b + 1] - am.row_off[b] + d->span_start[b];
    if (sm.save_count[b] > 0) {
      s->prev_cur[slot] ^= 1;
      s->prev_base[slot] = d->span_start[b] + sm.save_first[b];
      s->prev_count[slot] = sm.save_count[b];
    }
  }
  return DLM_OK;
}

// ---- block_boundary / select_parallel ------------------------------------------------------------
extern "C" int block_boundary(const float* I, const float* H, const int32_t* win_start, const int32_t* win_len, const int32_t* cold, int n_seqs,
                              const dlm_boundary_params* p, int32_t* L_out, float* S_out, float* margin_out, void* stream) {
  REQUIRE(I && H && win_start && win_len && p && L_out, DLM_EINVAL, "block_boundary: null argument");
  REQUIRE(n_seqs >= 1, DLM_EINVAL, "block_boundary: n_seqs %d < 1", n_seqs);
  REQUIRE(n_seqs <= DLM_MAX_SEQS, DLM_ECAPACITY, "block_boundary: n_seqs %d > %d", n_seqs, DLM_MAX_SEQS);
  REQUIRE(p->lambda > 0.f, DLM_EINVAL, "block_boundary: lambda must be positive");
  REQUIRE(p->l_min >= 1, DLM_EINVAL, "block_boundary: l_min %d < 1", p->l_min);
  REQUIRE(p->smooth_radius >= 0, DLM_EINVAL, "block_boundary: negative smooth_radius");
  REQUIRE(p->norm_mode >= 0 && p->norm_mode <= 3, DLM_EINVAL, "block_boundary: norm_mode %d", p->norm_mode);
  REQUIRE(p->rule == 0 || p->rule == 1, DLM_EINVAL, "block_boundary: rule %d", p->rule);
  BoundaryMeta meta;
  memset(&meta, 0, sizeof meta);
  for (int b = 0; b < n_seqs; ++b) {
    const int W = win_len[b];
    REQUIRE(W >= 1 && W <= 256, DLM_ECAPACITY, "block_boundary: window %d of sequence %d not in [1,256]", W, b);
    REQUIRE(win_start[b] >= 0, DLM_EINVAL, "block_boundary: negative offset");
    meta.cold[b] = cold ? (cold[b] != 0) : 0;
    meta.win_start[b] = win_start[b];
    meta.win_len[b] = W;
  }
  launch_block_boundary(I, H, meta, n_seqs, *p, L_out, S_out, margin_out, (hipStream_t)stream);
  return DLM_OK;
}

extern "C" int select_parallel(const void* logits, int vocab, int dtype, const float* lse, const float* conf, const int32_t* argmax,
                               int32_t* tokens, const int32_t* row_start, const int32_t* tok_start, const int32_t* block_len, int n_seqs,
                               int mask_id, const dlm_select_params* p, int apply_tokens, uint8_t* selected_out, int32_t* n_selected_out,
                               float* margin_out, void* stream) {
  REQUIRE(logits && lse && conf && argmax && tokens && row_start && tok_start && block_len && p && selected_out && n_selected_out,
          DLM_EINVAL, "select_parallel: null argument");
  REQUIRE(n_seqs >= 1, DLM_EINVAL, "select_parallel: n_seqs %d < 1", n_seqs);
  REQUIRE(n_seqs <= DLM_MAX_SEQS, DLM_ECAPACITY, "select_parallel: n_seqs %d > %d", n_seqs, DLM_MAX_SEQS);
  REQUIRE(dtype == DLM_F32 || dtype == DLM_BF16, DLM_EINVAL, "select_parallel: dtype %d", dtype);
  REQUIRE(vocab >= 2, DLM_EINVAL, "select_parallel: vocab %d < 2", vocab);
  REQUIRE(p->mode >= 0 && p->mode <= 2, DLM_EINVAL, "select_parallel: mode %d", p->mode);
  REQUIRE(p->mode != 0 || p->tau_high >= p->tau_low, DLM_EINVAL, "select_parallel: tau_high < tau_low");
  SelectMeta meta;
  memset(&meta, 0, sizeof meta);
  for (int b = 0; b < n_seqs; ++b) {
    REQUIRE(block_len[b] >= 0 && block_len[b] <= 256, DLM_ECAPACITY, "select_parallel: block_len %d of sequence %d not in [0,256]", block_len[b], b);
    REQUIRE(row_start[b] >= 0 && tok_start[b] >= 0, DLM_EINVAL, "select_parallel: negative start");
    meta.row_start[b] = row_start[b]; meta.tok_start[b] = tok_start[b]; meta.block_len[b] = block_len[b];
  }
  hipStream_t st = (hipStream_t)stream;
  if (dtype == DLM_BF16) launch_select<bf16_t>((const bf16_t*)logits, vocab, lse, conf, argmax, tokens, meta, n_seqs, mask_id, *p, apply_tokens, selected_out, n_selected_out, margin_out, st);
  else launch_select<float>((const float*)logits, vocab, lse, conf, argmax, tokens, meta, n_seqs, mask_id, *p, apply_tokens, selected_out, n_selected_out, margin_out, st);
  return DLM_OK;
}

// ---- component entry points ----------------------------------------------------------------------
extern "C" size_t dlm_vocab_stats_workspace(int rows) { return rows > 0 ? stats_workspace_bytes(rows) : 0; }

extern "C" int dlm_vocab_stats(const void* logits, const void* prev, const float* prev_lse, int rows, int vocab, int dtype, int mask_id, float* max_logit,
                               float* lse, float* entropy, float* kl, float* conf, int32_t* argmax, void* workspace,
                               size_t workspace_bytes, void* stream) {
  REQUIRE(logits && max_logit && lse && entropy && kl && conf && argmax && workspace, DLM_EINVAL, "dlm_vocab_stats: null argument");
  REQUIRE(dtype == DLM_F32 || dtype == DLM_BF16, DLM_EINVAL, "dlm_vocab_stats: dtype %d", dtype);
  REQUIRE(rows >= 1, DLM_ECAPACITY, "dlm_vocab_stats: rows %d < 1", rows);
  REQUIRE(workspace_bytes >= stats_workspace_bytes(rows), DLM_ECAPACITY, "dlm_vocab_stats: workspace of %zu bytes < %zu", workspace_bytes,
          stats_workspace_bytes(rows));
  REQUIRE(vocab >= 2 && mask_id >= 0 && mask_id < vocab, DLM_EINVAL, "dlm_vocab_stats: vocab/mask_id");
  StatsRows sr{nullptr, nullptr, prev, nullptr, prev ? prev_lse : nullptr, nullptr};  // prev without a row table: row r pairs with row r
  StatsOut so{max_logit, lse, entropy, kl, conf, argmax};
  hipStream_t st = (hipStream_t)stream;
  if (dtype == DLM_BF16) launch_vocab_stats<bf16_t>((const bf16_t*)logits, rows, vocab, mask_id, sr, so, workspace, st);
  else launch_vocab_stats<float>((const float*)logits, rows, vocab, mask_id, sr, so, workspace, st);
  return DLM_OK;
}

extern "C" int dlm_vocab_stats_static(const void* logits, const void* prev, const float* prev_lse, int rows, int vocab, int dtype, int mask_id, float* max_logit,
                                      float* lse, float* entropy, float* kl, float* conf, int32_t* argmax, void* stream) {
  REQUIRE(logits && max_logit && lse && entropy && kl && conf && argmax, DLM_EINVAL, "dlm_vocab_stats_static: null argument");
  REQUIRE(dtype == DLM_F32 || dtype == DLM_BF16, DLM_EINVAL, "dlm_vocab_stats_static: dtype %d", dtype);
  REQUIRE(rows >= 1, DLM_ECAPACITY, "dlm_vocab_stats_static: rows %d < 1", rows);
  REQUIRE(rows <= STATIC_STATS_MAX_ROWS && stats_workspace_bytes(rows) <= STATIC_STATS_BYTES, DLM_ECAPACITY,
          "dlm_vocab_stats_static: %d rows > the %d rows the static scratch holds (use dlm_vocab_stats with a workspace)", rows, STATIC_STATS_MAX_ROWS);
  REQUIRE(vocab >= 2 && mask_id >= 0 && mask_id < vocab, DLM_EINVAL, "dlm_vocab_stats_static: vocab/mask_id");
  void* ws = nullptr;
  const int rc = scratch_address(&ws);
  if (rc != DLM_OK) return rc;
  // every partial state the merge reads is written by this call's first kernel: nothing has to start at zero
  StatsRows sr{nullptr, nullptr, prev, nullptr, prev ? prev_lse : nullptr, nullptr};
  StatsOut so{max_logit, lse, entropy, kl, conf, argmax};
  hipStream_t st = (hipStream_t)stream;
  if (dtype == DLM_BF16) launch_vocab_stats<bf16_t>((const bf16_t*)logits, rows, vocab, mask_id, sr, so, ws, st);
  else launch_vocab_stats<float>((const float*)logits, rows, vocab, mask_id, sr, so, ws, st);
  return DLM_OK;
}

extern "C" int dlm_gemm_nt(const void* x, const void* w, void* y, int M, int N, int K, int dtype, void* stream) {
  REQUIRE(x && w && y, DLM_EINVAL, "dlm_gemm_nt: null argument");
  REQUIRE(dtype == DLM_F32 || dtype == DLM_BF16, DLM_EINVAL, "dlm_gemm_nt: dtype %d", dtype);
  REQUIRE(M >= 1 && N >= 1 && K >= 1, DLM_ESHAPE, "dlm_gemm_nt: non-positive dimension");
  hipStream_t st = (hipStream_t)stream;
  if (dtype == DLM_F32) { launch_gemm_f32((const float*)x, (const float*)w, (float*)y, M, N, K, RowScale{nullptr, 0, 0.f, 0.f}, st); return DLM_OK; }
  REQUIRE(N % 32 == 0 && K % 32 == 0, DLM_ESHAPE, "dlm_gemm_nt: bf16 needs N and K to be multiples of 32");
  const size_t mp = (size_t)(M + 15) / 16 * 16;
  const int n_counters = gemm_bf16_counters(M, N);
  const size_t tiled_bytes = ((mp * K + (size_t)N * K) * 2 + 15) / 16 * 16;
  const size_t part_bytes = (size_t)gemm_bf16_splits(M, N, K, EPI_SUM) * M * N * 4;
  void* ws = nullptr;
  if (hipMalloc(&ws, tiled_bytes + part_bytes + (size_t)n_counters * 4) != hipSuccess) { (void)hipGetLastError(); return dlm_fail(DLM_ENOMEM, "dlm_gemm_nt: workspace allocation failed"); }
  op_t* xt = (op_t*)ws;
  op_t* wt = xt + mp * K;
  float* part = (float*)((char*)ws + tiled_bytes);
  launch_pack_act((const bf16_t*)x, xt, M, K, st);
  launch_pack_weight((const bf16_t*)w, wt, N, K, PERM_NONE, 0, st);
  const int splits = gemm_bf16_splits(M, N, K, EPI_SUM);
  GemmEpi ge;
  memset(&ge, 0, sizeof ge);
  ge.out_bf16 = (bf16_t*)y;
  hipError_t e = hipSuccess;
  // partial tiles and ticket counters (used when the tiled kernel splits K) follow the tiled operands in the scratch
  ge.kind = EPI_SUM;
  ge.part = part;
  ge.counters = (int*)(part + (size_t)splits * M * N);
  e = hipMemsetAsync(ge.counters, 0, (size_t)n_counters * 4, st);
  launch_gemm_bf16(xt, wt, M, N, K, ge, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  (void)hipFree(ws);
  if (e != hipSuccess) return dlm_fail(DLM_EHIP, "dlm_gemm_nt: %s", hipGetErrorString(e));
  return DLM_OK;
}

extern "C" int dlm_attention(const void* q, const void* k, const void* v, void* out, int A, int T, int n_q, int n_kv, int head_dim, int dtype,
                             void* stream) {
  REQUIRE(q && k && v && out, DLM_EINVAL, "dlm_attention: null argument");
  REQUIRE(dtype == DLM_F32 || dtype == DLM_BF16, DLM_EINVAL, "dlm_attention: dtype %d", dtype);
  REQUIRE(A >= 1 && T >= 1 && n_q >= 1 && n_kv >= 1 && n_q % n_kv == 0, DLM_ESHAPE, "dlm_attention: bad shape");
  REQUIRE(head_dim == 32 || head_dim == 64 || head_dim == 128, DLM_ESHAPE, "dlm_attention: head_dim %d not in {32,64,128}", head_dim);
  AttnMeta am;
  memset(&am, 0, sizeof am);
  am.n_seqs = 1; am.row_off[1] = A; am.n_keys[0] = T;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == DLM_F32) {
    launch_attention<float>((const float*)q, (const float*)k, (const float*)v, 0, 0, am, (float*)out, false, A, A, n_q, n_kv, head_dim, st);
    return DLM_OK;
  }
  // bf16: K and V re-tiled into the half-precision cache layout, q converted to half (test helper: allocates and synchronises)
  const size_t head_stride = (size_t)((T + 31) / 32 * 32) * head_dim, bytes = head_stride * n_kv * 2;
  const size_t q_elems = (size_t)A * n_q * head_dim, q_bytes = (q_elems * 2 + 255) / 256 * 256;
  void* ws = nullptr;
  if (hipMalloc(&ws, 2 * bytes + q_bytes) != hipSuccess) { (void)hipGetLastError(); return dlm_fail(DLM_ENOMEM, "dlm_attention: workspace allocation failed"); }
  f16_t* kt = (f16_t*)ws;
  f16_t* vt = kt + head_stride * n_kv;
  f16_t* qh = vt + head_stride * n_kv;
  hipError_t e = hipMemsetAsync(ws, 0, 2 * bytes, st);
  launch_pack_kv((const bf16_t*)k, (const bf16_t*)v, kt, vt, T, n_kv, head_dim, head_stride, st);
  launch_to_f16((const bf16_t*)q, qh, q_elems, st);
  launch_attention_f16(qh, kt, vt, 0, head_stride, am, nullptr, (bf16_t*)out, A, A, n_q, n_kv, head_dim, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  (void)hipFree(ws);
  if (e != hipSuccess) return dlm_fail(DLM_EHIP, "dlm_attention: %s", hipGetErrorString(e));
  return DLM_OK;
}
