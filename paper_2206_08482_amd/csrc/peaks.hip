// Achievable-peak probes: a pure matrix-core loop and a streaming copy, so that measured kernel rates can
// be stated as fractions of what this device actually sustains as well as of its published peaks.
#include "internal.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

// Every wave keeps 4 independent accumulator tiles busy; no memory traffic inside the loop.
__global__ __launch_bounds__(256) void mfma_peak_kernel(int iters, float* __restrict__ sink) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(1.0f + 0.001f * (float)(threadIdx.x & 7));
    b[i] = (__bf16)(0.5f);
  }
  floatx16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[t][v];
  if (s == 12345.678f) sink[0] = s;   // keeps the loop alive without a store on the normal path
}

__global__ __launch_bounds__(256) void copy_peak_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

// Every workgroup streams the same buffer of n 16-byte words `reps` times: with a small buffer this is
// the cache-to-CU read bandwidth, with a large one the memory read bandwidth.
__global__ __launch_bounds__(256) void read_peak_kernel(const uint4* __restrict__ src, int64_t n, int reps,
                                                        uint32_t* __restrict__ sink) {
  uint32_t acc = 0;
  const int64_t start = ((int64_t)blockIdx.x * 1237) % n;     // workgroups start at different places
  for (int r = 0; r < reps; ++r)
    for (int64_t j = threadIdx.x; j < n; j += 256 * 4) {
      int64_t i0 = start + j; if (i0 >= n) i0 -= n;
      int64_t i1 = i0 + 256; if (i1 >= n) i1 -= n;
      int64_t i2 = i1 + 256; if (i2 >= n) i2 -= n;
      int64_t i3 = i2 + 256; if (i3 >= n) i3 -= n;
      const uint4 a = src[i0], b = src[i1], c = src[i2], d = src[i3];
      acc ^= a.x ^ b.y ^ c.z ^ d.w;
    }
  if (acc == 0x12345678u) sink[0] = acc;
}

}  // namespace

// what = 0: dense bf16 MFMA rate in TFLOP/s; what = 1: copy bandwidth in GB/s (read + write bytes).
// scratch: device buffer of scratch_bytes (copy probe uses two halves; MFMA probe needs 4 bytes).
extern "C" int gmi_measure_peak(gmi_t g, int what, void* scratch, size_t scratch_bytes, double* result) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_measure_peak: bad handle");
  if (!result || !scratch) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_measure_peak: NULL argument");
  hipEvent_t e0, e1;
  GMI_HIP(hipEventCreate(&e0));
  GMI_HIP(hipEventCreate(&e1));
  float ms = 0.f;
  int rc = GMI_OK;
  if (what == 0) {
    if (scratch_bytes < 4) GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_measure_peak: scratch too small");
    const int iters = 20000, grid = g->cu_count * 8;
    mfma_peak_kernel<<<grid, 256, 0, g->stream>>>(100, (float*)scratch);      // warm-up
    (void)hipEventRecord(e0, g->stream);
    mfma_peak_kernel<<<grid, 256, 0, g->stream>>>(iters, (float*)scratch);
    (void)hipEventRecord(e1, g->stream);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = GMI_ERR_HIP;
    *result = (double)grid * 4.0 * iters * 4.0 * 32768.0 / (ms * 1e-3) / 1e12;
  } else if (what == 1) {
    const int64_t n = (int64_t)(scratch_bytes / 2 / 16);
    if (n < 1024) GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_measure_peak: scratch too small");
    const uint4* src = (const uint4*)scratch;
    uint4* dst = (uint4*)scratch + n;
    const int grid = g->cu_count * 16;
    copy_peak_kernel<<<grid, 256, 0, g->stream>>>(src, dst, n);
    (void)hipEventRecord(e0, g->stream);
    for (int r = 0; r < 5; ++r) copy_peak_kernel<<<grid, 256, 0, g->stream>>>(src, dst, n);
    (void)hipEventRecord(e1, g->stream);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = GMI_ERR_HIP;
    *result = 5.0 * 2.0 * 16.0 * (double)n / (ms * 1e-3) / 1e9;
  } else if (what >= 2 && what <= 40) {
    // read bandwidth over the first 2^what bytes of scratch, every workgroup reading all of it
    const int64_t bytes = 1ll << what;
    if ((size_t)bytes + 64 > scratch_bytes || bytes < 16384) GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_measure_peak: bad size");
    const int64_t n = bytes / 16;
    const int grid = g->cu_count * 4;
    int reps = (int)((1ll << 28) / bytes);
    if (reps < 1) reps = 1;
    if (reps > 4096) reps = 4096;
    uint32_t* sink = (uint32_t*)((char*)scratch + bytes);
    read_peak_kernel<<<grid, 256, 0, g->stream>>>((const uint4*)scratch, n, 1, sink);
    (void)hipEventRecord(e0, g->stream);
    read_peak_kernel<<<grid, 256, 0, g->stream>>>((const uint4*)scratch, n, reps, sink);
    (void)hipEventRecord(e1, g->stream);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = GMI_ERR_HIP;
    *result = (double)grid * (double)reps * (double)bytes / (ms * 1e-3) / 1e9;
  } else {
    rc = GMI_ERR_INVALID_ARG;
    gmi::set_error("gmi_measure_peak: what must be 0 (MFMA), 1 (copy) or log2(bytes) of a read sweep");
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc == GMI_ERR_HIP) gmi::set_error("gmi_measure_peak: timing failed");
  return rc;
}

// Micro-benchmark of one linear-layer product on synthetic operands carved out of `scratch`:
// kind 0 = forward (bias + ELU), 2 = input gradient (ELU' epilogue), 3 = weight gradient (the split count a model of these tiles would get).
// rows x K -> F (all padded to multiples of 32 by the caller), n_nets problems per launch, bf16.
// Returns the average microseconds per launch over `reps` back-to-back launches.
extern "C" int gmi_bench_linear(gmi_t g, int kind, int rows, int K, int F, int n_nets, int reps, void* scratch,
                                size_t scratch_bytes, double* us_per_launch) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_bench_linear: bad handle");
  if (!scratch || !us_per_launch) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_bench_linear: NULL argument");
  if (rows < 1 || (K & 31) || (F & 31) || K < 32 || F < 32 || n_nets < 1 || n_nets > 2 || reps < 1)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_bench_linear: rows >= 1, K and F multiples of 32, 1..2 nets, reps >= 1");
  char* p = (char*)scratch;
  size_t off = 0;
  auto take = [&](size_t bytes) { char* q = p + off; off += (bytes + 255) & ~(size_t)255; return q; };
  gmi::LinearBatch lb;
  gmi::WgradBatch wb;
  lb.n = n_nets;
  wb.n = n_nets;
  float* part = nullptr;
  const int64_t P = (int64_t)n_nets * ((int64_t)K * F + F);
  for (int z = 0; z < n_nets; ++z) {
    void* x = take((size_t)rows * K * 2);
    void* w = take((size_t)F * K * 2);
    float* bias = (float*)take((size_t)F * 4);
    void* h = take((size_t)rows * F * 2);
    void* y = take((size_t)rows * F * 2);
    gmi::LinearProblem& q = lb.p[z];
    q.x = x; q.ldx = K; q.w = w; q.ldw = K; q.wsf = K; q.wsk = 1; q.bias = bias; q.h = h; q.ldh = F; q.y = y; q.ldy = F;
    q.K = K; q.F = F; q.F_store = F; q.K_log = K; q.F_log = F;
    gmi::WgradProblem& r = wb.p[z];            // dW[F, K] = y^T x
    r.dz = y; r.lddz = F; r.x = x; r.ldx = K; r.out = F; r.in = K; r.out_pad = F; r.in_pad = K; r.dz_blocks = r.x_blocks = 0;
    r.w_off = (int64_t)z * ((int64_t)K * F + F); r.b_off = r.w_off + (int64_t)K * F;
  }
  const int n_split = gmi::wgrad_split_limit(n_nets * ((F + 127) / 128) * ((K + 127) / 128));
  if (kind == 3) part = (float*)take((size_t)n_split * P * 4);
  if (off > scratch_bytes) GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_bench_linear: scratch too small (%zu needed)", off);
  const int chunk = ((rows + n_split - 1) / n_split + 63) / 64 * 64;
  auto launch = [&]() -> int {
    if (kind == 3) return gmi::launch_wgrad(g, GMI_DTYPE_BF16, rows, n_split, chunk, wb, part, P);
    return gmi::launch_linear(g, GMI_DTYPE_BF16, kind == 0 ? gmi::kEpiBiasElu : gmi::kEpiEluGrad, rows, lb);
  };
  hipEvent_t e0, e1;
  GMI_HIP(hipEventCreate(&e0));
  GMI_HIP(hipEventCreate(&e1));
  int rc = launch();
  if (rc == GMI_OK) {
    (void)hipEventRecord(e0, g->stream);
    for (int r = 0; r < reps && rc == GMI_OK; ++r) rc = launch();
    (void)hipEventRecord(e1, g->stream);
    float ms = 0.f;
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
      rc = GMI_ERR_HIP;
      gmi::set_error("gmi_bench_linear: timing failed");
    }
    *us_per_launch = ms * 1e3 / reps;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return rc;
}
