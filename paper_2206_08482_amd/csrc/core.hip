// Instances (CU-masked streams), hand-off between instances, error reporting, RNG utilities.
#include <stdarg.h>
#include <string.h>

#include "internal.h"
#include "rng.h"

namespace gmi {
static thread_local char g_err[512] = "";
void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
}  // namespace gmi

extern "C" const char* gmi_last_error(void) { return gmi::g_err; }

namespace gmi {
ProfScope::ProfScope(gmi_instance* g_, int cls_) : g(g_), cls(cls_), on((g_->prof_mask >> cls_) & 1u) {}
void ProfScope::work(double flops, double bytes) {
  if (on) { g->prof[cls].flops += flops; g->prof[cls].bytes += bytes; }
}
bool ProfScope::next_events(hipEvent_t* a, hipEvent_t* b) {
  ProfSlot& s = g->prof[cls];
  if (s.used == s.start.size()) {
    hipEvent_t ea, eb;
    if (hipEventCreate(&ea) != hipSuccess) return false;
    if (hipEventCreate(&eb) != hipSuccess) { (void)hipEventDestroy(ea); return false; }
    s.start.push_back(ea);
    s.stop.push_back(eb);
  }
  *a = s.start[s.used];
  *b = s.stop[s.used];
  ++s.used;
  return true;
}
static const char* kClassNames[kClsCount] = {
    "gather", "wgrad", "loss", "adam", "shadow_transpose", "env_step", "sample", "collect", "gae", "permutation",
    "fused_agent", "fused_rollout", "linear_f32", "chain_train",
    "linear_big256_fwd", "linear_big256_head", "linear_big256_dgrad",
    "linear_big128_fwd", "linear_big128_head", "linear_big128_dgrad",
    "linear_t128_fwd", "linear_t128_head", "linear_t128_dgrad",
    "linear_t256x64_fwd", "linear_t256x64_head", "linear_t256x64_dgrad",
    "linear_t128x64_fwd", "linear_t128x64_head", "linear_t128x64_dgrad"};
}  // namespace gmi

extern "C" int gmi_profile_enable(gmi_t g, uint32_t class_mask) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_profile_enable: bad handle");
  GMI_HIP(hipStreamSynchronize(g->stream));
  g->prof_mask = class_mask & ((1u << gmi::kClsCount) - 1u);
  for (int c = 0; c < gmi::kClsCount; ++c) {
    g->prof[c].used = 0;
    g->prof[c].flops = g->prof[c].bytes = 0.0;
  }
  return GMI_OK;
}

extern "C" int gmi_profile_work(gmi_t g, int cls, double* flops, double* bytes) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_profile_work: bad handle");
  if (cls < 0 || cls >= gmi::kClsCount) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_profile_work: class %d out of range", cls);
  if (!flops || !bytes) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_profile_work: NULL output");
  *flops = g->prof[cls].flops;
  *bytes = g->prof[cls].bytes;
  return GMI_OK;
}

extern "C" int gmi_profile_classes(void) { return gmi::kClsCount; }

extern "C" const char* gmi_profile_class_name(int cls) {
  return (cls >= 0 && cls < gmi::kClsCount) ? gmi::kClassNames[cls] : nullptr;
}

extern "C" int gmi_profile_read(gmi_t g, int cls, double* total_ms, int64_t* launches) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_profile_read: bad handle");
  if (cls < 0 || cls >= gmi::kClsCount) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_profile_read: class %d out of range", cls);
  if (!total_ms || !launches) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_profile_read: NULL output");
  GMI_HIP(hipStreamSynchronize(g->stream));
  gmi::ProfSlot& s = g->prof[cls];
  double sum = 0.0;
  for (size_t i = 0; i < s.used; ++i) {
    float ms = 0.f;
    GMI_HIP(hipEventElapsedTime(&ms, s.start[i], s.stop[i]));
    sum += ms;
  }
  *total_ms = sum;
  *launches = (int64_t)s.used;
  return GMI_OK;
}

extern "C" int gmi_create(const uint32_t* cu_mask, uint32_t n_words, int device, gmi_t* out) {
  if (!out) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_create: out is NULL");
  *out = nullptr;
  int n_dev = 0;
  GMI_HIP(hipGetDeviceCount(&n_dev));
  if (device < 0 || device >= n_dev)
    GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_create: device %d out of range (have %d)", device, n_dev);
  GMI_HIP(hipSetDevice(device));
  hipDeviceProp_t prop;
  GMI_HIP(hipGetDeviceProperties(&prop, device));
  const int n_cu = prop.multiProcessorCount;
  int cu_count = n_cu;
  hipStream_t stream = nullptr;
  if (cu_mask && n_words > 0) {
    const uint32_t need_words = (uint32_t)((n_cu + 31) / 32);
    std::vector<uint32_t> mask(need_words, 0u);
    int bits = 0;
    for (uint32_t w = 0; w < n_words; ++w) {
      uint32_t v = cu_mask[w];
      if (w >= need_words) {
        if (v) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_create: cu_mask names CUs beyond the device's %d", n_cu);
        continue;
      }
      if (w == need_words - 1 && (n_cu % 32) != 0 && (v >> (n_cu % 32)))
        GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_create: cu_mask names CUs beyond the device's %d", n_cu);
      mask[w] = v;
      bits += __builtin_popcount(v);
    }
    if (bits == 0) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_create: cu_mask enables no compute unit");
    const hipError_t ce = hipExtStreamCreateWithCUMask(&stream, need_words, mask.data());
    if (ce != hipSuccess) {
      (void)hipGetLastError();
      // Observed on gfx950: bit i addresses a CU of accelerator die i % 8 and the runtime refuses a mask
      // that leaves a die without any CU (it reports "out of memory").
      GMI_FAIL(GMI_ERR_INVALID_ARG,
               "gmi_create: the runtime refused this CU mask (%s); every one of the 8 dies (bit index mod 8) "
               "needs at least one CU", hipGetErrorString(ce));
    }
    cu_count = bits;
  } else {
    GMI_HIP(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking));
  }
  gmi_instance* g = new gmi_instance();
  g->magic = gmi::kMagicInstance;
  g->device = device;
  g->stream = stream;
  g->cu_count = cu_count;
  g->prof_mask = 0;
  g->fusion = 1;
  hipError_t e = hipEventCreateWithFlags(&g->event, hipEventDisableTiming);
  if (e == hipSuccess) {
    e = hipEventCreateWithFlags(&g->wait_event, hipEventDisableTiming);
    if (e != hipSuccess) (void)hipEventDestroy(g->event);
  }
  if (e != hipSuccess) {
    hipStreamDestroy(stream);
    delete g;
    GMI_FAIL(GMI_ERR_HIP, "gmi_create: hipEventCreate failed: %s", hipGetErrorString(e));
  }
  *out = g;
  return GMI_OK;
}

extern "C" int gmi_destroy(gmi_t g) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_destroy: bad handle");
  (void)hipStreamSynchronize(g->stream);
  for (int c = 0; c < gmi::kClsCount; ++c)
    for (size_t i = 0; i < g->prof[c].start.size(); ++i) {
      (void)hipEventDestroy(g->prof[c].start[i]);
      (void)hipEventDestroy(g->prof[c].stop[i]);
    }
  (void)hipEventDestroy(g->event);
  (void)hipEventDestroy(g->wait_event);
  (void)hipStreamDestroy(g->stream);
  g->magic = 0;
  delete g;
  return GMI_OK;
}

extern "C" int gmi_set_fusion(gmi_t g, int enable) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_set_fusion: bad handle");
  g->fusion = enable > 0 ? 1 : 0;
  return GMI_OK;
}

extern "C" void* gmi_stream(gmi_t g) { return valid(g) ? (void*)g->stream : nullptr; }

extern "C" int gmi_cu_count(gmi_t g) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_cu_count: bad handle");
  return g->cu_count;
}

extern "C" int gmi_sync(gmi_t g) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_sync: bad handle");
  GMI_HIP(hipStreamSynchronize(g->stream));
  return GMI_OK;
}

extern "C" int gmi_wait_stream(gmi_t g, void* hip_stream) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_wait_stream: bad handle");
  hipStream_t other = static_cast<hipStream_t>(hip_stream);
  if (other == g->stream) return GMI_OK;
  GMI_HIP(hipEventRecord(g->wait_event, other));
  GMI_HIP(hipStreamWaitEvent(g->stream, g->wait_event, 0));
  return GMI_OK;
}

extern "C" int gmi_transfer(gmi_t src, gmi_t dst, const void* src_ptr, void* dst_ptr, size_t bytes) {
  if (!valid(src) || !valid(dst)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_transfer: bad handle");
  if (src->device != dst->device)
    GMI_FAIL(GMI_ERR_UNSUPPORTED, "gmi_transfer: instances live on different devices");
  if (bytes > 0 && src_ptr != dst_ptr) {
    if (!src_ptr || !dst_ptr) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_transfer: NULL pointer with bytes > 0");
    GMI_HIP(hipMemcpyAsync(dst_ptr, src_ptr, bytes, hipMemcpyDeviceToDevice, src->stream));
  }
  if (src != dst) {
    GMI_HIP(hipEventRecord(src->event, src->stream));
    GMI_HIP(hipStreamWaitEvent(dst->stream, src->event, 0));
  }
  return GMI_OK;
}

// ---------------------------------------------------------------------------------------------
namespace {

__global__ void noise_fill_kernel(uint32_t k0, uint32_t k1, uint32_t stream, uint32_t step,
                                  uint32_t env_offset, int n_envs, int dim, int n_blocks,
                                  float* __restrict__ out) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (int64_t)n_envs * n_blocks) return;
  const int e = (int)(gid / n_blocks), b = (int)(gid % n_blocks);
  float z[4];
  gmi::normal_block(env_offset + (uint32_t)e, step, stream, (uint32_t)b, k0, k1, z);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int j = 4 * b + i;
    if (j < dim) out[(int64_t)e * dim + j] = z[i];
  }
}

__global__ void permutation_kernel(int n, int bits, uint32_t iteration, uint32_t epoch, uint32_t k0,
                                   uint32_t k1, int32_t* __restrict__ out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;      // blockIdx.y: epoch after the first
  if (i < n)
    out[(int64_t)blockIdx.y * n + i] = (int32_t)gmi::feistel_perm((uint32_t)i, (uint32_t)n, bits, iteration, epoch + blockIdx.y, k0, k1);
}

}  // namespace

namespace gmi {
int launch_permutation(gmi_instance* g, int n, uint64_t seed, uint32_t iteration, uint32_t epoch, int n_epochs, int32_t* out) {
  if (n <= 0 || n_epochs <= 0) return GMI_OK;
  ProfScope ps(g, kClsPermutation);
  int bits = 0;
  while ((1ll << bits) < (long long)n) ++bits;
  ps.launch(permutation_kernel, dim3((n + 255) / 256, n_epochs), dim3(256), 0, n, bits, iteration, epoch, (uint32_t)seed,
                                                     (uint32_t)(seed >> 32), out);
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}
}  // namespace gmi

extern "C" int gmi_noise_fill(gmi_t g, uint64_t seed, uint32_t stream, uint32_t step, uint32_t env_offset,
                              int32_t n_envs, int32_t dim, float* out) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_noise_fill: bad handle");
  if (n_envs < 0 || dim < 0) GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_noise_fill: negative size");
  if (n_envs == 0 || dim == 0) return GMI_OK;
  if (!out) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_noise_fill: out is NULL");
  const int n_blocks = (dim + 3) / 4;
  const int64_t total = (int64_t)n_envs * n_blocks;
  noise_fill_kernel<<<(unsigned)((total + 255) / 256), 256, 0, g->stream>>>(
      (uint32_t)seed, (uint32_t)(seed >> 32), stream, step, env_offset, n_envs, dim, n_blocks, out);
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}

extern "C" int gmi_permutation(gmi_t g, int32_t n, uint64_t seed, uint32_t iteration, uint32_t epoch,
                               int32_t* out) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_permutation: bad handle");
  if (n < 0) GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_permutation: negative n");
  if (n == 0) return GMI_OK;
  if (!out) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_permutation: out is NULL");
  return gmi::launch_permutation(g, n, seed, iteration, epoch, 1, out);
}
