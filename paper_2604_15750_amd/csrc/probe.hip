// What this GPU achieves on the two resources the rooflines are drawn against, measured with kernels that do nothing else:
// a streaming read of HBM (every byte once, 16-byte loads, two trips in flight per workgroup: the access pattern of the
// weight-streaming GEMMs) and a loop of independent bf16 matrix-core products out of registers.  Both time themselves with
// events on the caller's stream and synchronise it: measurement helpers, not part of a decoding pass.
#include "common.h"

#define REQUIRE(cond, code, ...) \
  do {                           \
    if (!(cond)) return dlm_fail(code, __VA_ARGS__); \
  } while (0)

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// workgroup b reads pieces [b * per_wg, (b + 1) * per_wg) of 16 bytes; U pieces per thread and trip, one trip ahead in flight
template <int U>
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ src, size_t per_wg, unsigned* __restrict__ sink) {
  const u32x4* p = src + (size_t)blockIdx.x * per_wg + threadIdx.x;
  const size_t trips = per_wg / (256 * U);
  u32x4 a[U], b[U];
  unsigned acc = 0;
#pragma unroll
  for (int i = 0; i < U; ++i) a[i] = p[(size_t)i * 256];
  for (size_t t = 0; t < trips; t += 2) {
    const size_t t1 = t + 1 < trips ? t + 1 : t, t2 = t + 2 < trips ? t + 2 : t;
#pragma unroll
    for (int i = 0; i < U; ++i) b[i] = p[(t1 * U + i) * 256];
#pragma unroll
    for (int i = 0; i < U; ++i) acc += a[i].x ^ a[i].w;
#pragma unroll
    for (int i = 0; i < U; ++i) a[i] = p[(t2 * U + i) * 256];
#pragma unroll
    for (int i = 0; i < U; ++i) acc += b[i].y ^ b[i].z;
  }
  if (acc == 0x12345678u) sink[0] = acc;  // keeps the loads alive; practically never true
}

// every wavefront: `iters` rounds of 32 independent 16x16x32 half-precision products out of registers, 8 x 4 operand fragments
// of pseudo-random values (standard-normal-like, as a pass's activations and scaled weights are).  With constant or regular
// operands the chip holds 2.4 GHz and the loop reaches the published rate; with operands that switch like real data it is
// power-limited well below that, and that is the rate a GEMM can be held against.
__device__ inline unsigned probe_hash(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}
__device__ inline float probe_normal(unsigned s) {  // sum of four uniforms, centred and scaled to unit variance
  float t = 0.f;
  for (int i = 0; i < 4; ++i) { s = probe_hash(s + 977u * i); t += (s >> 8) * (1.0f / 16777216.0f); }
  return (t - 2.0f) * 1.7320508f;
}
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* __restrict__ sink) {
  const unsigned id = blockIdx.x * blockDim.x + threadIdx.x;
  op8 a[8], b[4];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) a[j][i] = (op_t)(0.02f * probe_normal(id * 131u + j * 17u + i));
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) b[j][i] = (op_t)probe_normal(id * 977u + j * 29u + i + 12345u);
  f32x4 acc[32];
#pragma unroll
  for (int i = 0; i < 32; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[j * 4 + i] = mfma_op(a[j], b[i], acc[j * 4 + i]);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 32; ++i) s += acc[i][0] + acc[i][3];
  if (s == 12345.678f) sink[0] = s;
}

template <typename F>
int timed(F&& launch, int reps, hipStream_t st, float* ms_out) {
  hipEvent_t a, b;
  DLM_HIP(hipEventCreate(&a));
  DLM_HIP(hipEventCreate(&b));
  launch();  // warm-up
  DLM_HIP(hipEventRecord(a, st));
  for (int i = 0; i < reps; ++i) launch();
  DLM_HIP(hipEventRecord(b, st));
  DLM_HIP(hipEventSynchronize(b));
  DLM_HIP(hipEventElapsedTime(ms_out, a, b));
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  DLM_HIP(hipGetLastError());
  return DLM_OK;
}

}  // namespace

extern "C" int dlm_probe_hbm_read(const void* src, size_t bytes, int reps, double* gb_per_s, void* stream) {
  REQUIRE(src && gb_per_s, DLM_EINVAL, "dlm_probe_hbm_read: null argument");
  constexpr int U = 4, WGS = 1024;
  const size_t per_wg = bytes / 16 / WGS / (256 * U) * (256 * U);
  REQUIRE(per_wg >= 256 * U && reps >= 1, DLM_ESHAPE, "dlm_probe_hbm_read: at least %zu bytes and one repetition", (size_t)16 * WGS * 256 * U);
  hipStream_t st = (hipStream_t)stream;
  unsigned* sink = nullptr;
  if (hipMalloc(&sink, 4) != hipSuccess) { (void)hipGetLastError(); return dlm_fail(DLM_ENOMEM, "dlm_probe_hbm_read: allocation failed"); }
  float ms = 0.f;
  const int rc = timed([&] { probe_read_kernel<U><<<WGS, 256, 0, st>>>((const u32x4*)src, per_wg, sink); }, reps, st, &ms);
  (void)hipFree(sink);
  if (rc != DLM_OK) return rc;
  *gb_per_s = (double)per_wg * WGS * 16 * reps / (ms * 1e-3) / 1e9;
  return DLM_OK;
}

extern "C" int dlm_probe_mfma(int reps, double* tflop_per_s, void* stream) {
  REQUIRE(tflop_per_s && reps >= 1, DLM_EINVAL, "dlm_probe_mfma: bad argument");
  constexpr int WGS = 2048, ITERS = 8192;  // 14 ms per launch: long enough for the clock to settle at what the power limit allows
  hipStream_t st = (hipStream_t)stream;
  float* sink = nullptr;
  if (hipMalloc(&sink, 4) != hipSuccess) { (void)hipGetLastError(); return dlm_fail(DLM_ENOMEM, "dlm_probe_mfma: allocation failed"); }
  float ms = 0.f;
  const int rc = timed([&] { probe_mfma_kernel<<<WGS, 256, 0, st>>>(ITERS, sink); }, reps, st, &ms);
  (void)hipFree(sink);
  if (rc != DLM_OK) return rc;
  *tflop_per_s = (double)WGS * 4 * ITERS * 32 * (2.0 * 16 * 16 * 32) * reps / (ms * 1e-3) / 1e12;
  return DLM_OK;
}
