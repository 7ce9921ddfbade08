// Experience buffer (one array per data type, time major), its filling, and GAE.
#include <mutex>

#include "internal.h"

namespace {

// Copies step t's experience into slot t of every channel.  A slot of a channel is one contiguous slab
// (time-major layout), so the bulk of the work (obs, act) is a straight 16-byte-per-lane copy when the
// slab and the source are 16-byte aligned; the scalar channels and the unaligned case go element-wise.
__global__ __launch_bounds__(256) void collect_kernel(gmi_buffer_desc d, int t, const float* __restrict__ obs,
                                                      const float* __restrict__ act, const float* __restrict__ logp,
                                                      const float* __restrict__ value, const float* __restrict__ reward,
                                                      const uint8_t* __restrict__ done, int vec_obs, int vec_act) {
  const int64_t slot0 = (int64_t)t * d.ld_envs;
  const int64_t n_obs = (int64_t)d.n_envs * d.obs_dim, n_act = (int64_t)d.n_envs * d.act_dim;
  const int64_t stride = (int64_t)gridDim.x * 256;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  float* o_dst = d.obs + slot0 * d.obs_dim;
  float* a_dst = d.act + slot0 * d.act_dim;
  if (vec_obs) {
    const float4* s4 = reinterpret_cast<const float4*>(obs);
    float4* d4 = reinterpret_cast<float4*>(o_dst);
    for (int64_t i = gid; i < n_obs / 4; i += stride) d4[i] = s4[i];
  } else {
    for (int64_t i = gid; i < n_obs; i += stride) o_dst[i] = obs[i];
  }
  if (vec_act) {
    const float4* s4 = reinterpret_cast<const float4*>(act);
    float4* d4 = reinterpret_cast<float4*>(a_dst);
    for (int64_t i = gid; i < n_act / 4; i += stride) d4[i] = s4[i];
  } else {
    for (int64_t i = gid; i < n_act; i += stride) a_dst[i] = act[i];
  }
  for (int64_t e = gid; e < d.n_envs; e += stride) {
    d.logp[slot0 + e] = logp[e];
    d.val[slot0 + e] = value[e];
    d.rew[slot0 + e] = reward[e];
    d.done[slot0 + e] = done[e];
  }
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}

// Reverse recurrence over the horizon, one lane per env: the time-major layout makes every step's
// loads and stores of a wave one contiguous segment.  Also leaves per-workgroup sums of A and A^2.
__global__ __launch_bounds__(256) void gae_kernel(gmi_buffer_desc d, const float* __restrict__ last_value,
                                                  float gamma, float gl, double* __restrict__ part) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  double s1 = 0.0, s2 = 0.0;
  if (e < d.n_envs) {
    float adv_next = 0.f;
    float v_next = last_value[e];
#pragma unroll 4
    for (int t = d.horizon - 1; t >= 0; --t) {
      const int64_t i = (int64_t)t * d.ld_envs + e;
      const float r = d.rew[i], v = d.val[i];
      const float nd = 1.0f - (float)d.done[i];
      const float delta = r + gamma * v_next * nd - v;
      adv_next = delta + gl * nd * adv_next;
      d.adv[i] = adv_next;
      d.ret[i] = adv_next + v;
      v_next = v;
      s1 += (double)adv_next;
      s2 += (double)adv_next * (double)adv_next;
    }
  }
  if (part) {
    __shared__ double sh[2][4];
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { sh[0][w] = s1; sh[1][w] = s2; }
    __syncthreads();
    if (threadIdx.x == 0) {
      part[2 * blockIdx.x + 0] = sh[0][0] + sh[0][1] + sh[0][2] + sh[0][3];
      part[2 * blockIdx.x + 1] = sh[1][0] + sh[1][1] + sh[1][2] + sh[1][3];
    }
  }
}

// The same recurrence as a wavefront scan: A_t = f_t(A_{t+1}) with the affine maps f_t(x) = delta_t + c_t x,
// c_t = gamma lambda (1 - d_t), and composition of affine maps is associative -- (c_a, d_a) o (c_b, d_b) =
// (c_a c_b, d_a + c_a d_b) -- so the TP = 2^k >= T consecutive lanes of one env compose their suffixes in log2 TP
// shuffle steps (Hillis-Steele, reverse direction).  A workgroup takes 64 envs: their [T, 64] slices travel through
// LDS so that memory is touched with lanes over envs (coalesced on the time-major layout) and the scan runs with
// lanes over time.  Horizons up to 64.  The sums are formed in another order than the serial walk's (a tree instead
// of a chain): equal within the fp32 rounding of T terms.
constexpr int kScanEnvs = 64;
template <int TP>
__global__ __launch_bounds__(256) void gae_scan_kernel(gmi_buffer_desc d, const float* __restrict__ last_value,
                                                       float gamma, float gl, double* __restrict__ part) {
  extern __shared__ float s_gae[];                      // [T + 1][65] values, [T][65] rewards -> advantages, [T][65] done
  const int T = d.horizon, ldl = kScanEnvs + 1;
  float* s_v = s_gae;
  float* s_r = s_v + (T + 1) * ldl;
  float* s_d = s_r + T * ldl;
  const int e0 = blockIdx.x * kScanEnvs, tid = threadIdx.x;
  for (int i = tid; i < T * kScanEnvs; i += 256) {
    const int t = i / kScanEnvs, e = i % kScanEnvs;
    const bool ok = e0 + e < d.n_envs;
    const int64_t g = (int64_t)t * d.ld_envs + e0 + e;
    s_v[t * ldl + e] = ok ? d.val[g] : 0.f;
    s_r[t * ldl + e] = ok ? d.rew[g] : 0.f;
    s_d[t * ldl + e] = ok ? (float)d.done[g] : 0.f;
  }
  if (tid < kScanEnvs) s_v[T * ldl + tid] = e0 + tid < d.n_envs ? last_value[e0 + tid] : 0.f;
  __syncthreads();
  double s1 = 0.0, s2 = 0.0;
  for (int slot = tid; slot < kScanEnvs * TP; slot += 256) {       // TP consecutive lanes = one env's timeline
    const int e = slot / TP, t = slot % TP;
    const bool in = t < T;
    float c = 1.f, a = 0.f, v = 0.f;                    // past the horizon: the identity map
    if (in) {
      const float nd = 1.0f - s_d[t * ldl + e];
      v = s_v[t * ldl + e];
      c = gl * nd;
      a = s_r[t * ldl + e] + gamma * s_v[(t + 1) * ldl + e] * nd - v;
    }
#pragma unroll
    for (int off = 1; off < TP; off <<= 1) {
      const float cp = __shfl_down(c, off, TP), ap = __shfl_down(a, off, TP);
      if (t + off < TP) { a = a + c * ap; c = c * cp; }
    }
    if (in) {
      s_r[t * ldl + e] = a;                              // the advantage takes the reward's place
      if (e0 + e < d.n_envs) { s1 += (double)a; s2 += (double)a * (double)a; }
    }
  }
  __syncthreads();
  for (int i = tid; i < T * kScanEnvs; i += 256) {
    const int t = i / kScanEnvs, e = i % kScanEnvs;
    if (e0 + e < d.n_envs) {
      const int64_t g = (int64_t)t * d.ld_envs + e0 + e;
      const float a = s_r[t * ldl + e];
      d.adv[g] = a;
      d.ret[g] = a + s_v[t * ldl + e];
    }
  }
  if (part) {
    __shared__ double sh[2][4];
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    const int w = tid >> 6;
    if ((tid & 63) == 0) { sh[0][w] = s1; sh[1][w] = s2; }
    __syncthreads();
    if (tid == 0) {
      part[2 * blockIdx.x + 0] = sh[0][0] + sh[0][1] + sh[0][2] + sh[0][3];
      part[2 * blockIdx.x + 1] = sh[1][0] + sh[1][1] + sh[1][2] + sh[1][3];
    }
  }
}

// Which of the two GAE kernels a call takes: 0 the serial walk (lane per env), 1 the wavefront scan.  The serial
// walk is the default at every size (measured: it is the faster one wherever the two differ, see the profiles);
// the measurement interface can force either.
int g_gae_variant = 0;

// Launches the chosen GAE kernel on `stream`; returns the number of partial-sum pairs it leaves in `part`.
template <typename Launch>
int launch_gae(int variant, const gmi_buffer_desc& d, const float* last_value, float gamma, float gl, double* part,
               Launch&& launch) {
  if (variant == 1 && d.horizon <= 64) {
    const int n_part = (d.n_envs + kScanEnvs - 1) / kScanEnvs;
    const size_t lds = sizeof(float) * (size_t)(3 * d.horizon + 1) * (kScanEnvs + 1);
    int tp = 1;
    while (tp < d.horizon) tp <<= 1;
    switch (tp) {
      case 1: launch(gae_scan_kernel<1>, n_part, lds); break;
      case 2: launch(gae_scan_kernel<2>, n_part, lds); break;
      case 4: launch(gae_scan_kernel<4>, n_part, lds); break;
      case 8: launch(gae_scan_kernel<8>, n_part, lds); break;
      case 16: launch(gae_scan_kernel<16>, n_part, lds); break;
      case 32: launch(gae_scan_kernel<32>, n_part, lds); break;
      default: launch(gae_scan_kernel<64>, n_part, lds); break;
    }
    return n_part;
  }
  const int n_part = (d.n_envs + 255) / 256;
  launch(gae_kernel, n_part, (size_t)0);
  return n_part;
}

// A <- (A - mean) / (std + 1e-8); every workgroup re-reduces the (small) partial array in the same
// order, so the statistics are identical everywhere and reproducible.
__global__ __launch_bounds__(256) void normalize_kernel(gmi_buffer_desc d, const double* __restrict__ part,
                                                        int n_part) {
  __shared__ double sh[2][4];
  __shared__ float s_mean, s_inv;
  double s1 = 0.0, s2 = 0.0;
  for (int i = threadIdx.x; i < n_part; i += 256) { s1 += part[2 * i]; s2 += part[2 * i + 1]; }
  s1 = wave_sum(s1);
  s2 = wave_sum(s2);
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { sh[0][w] = s1; sh[1][w] = s2; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const double n = (double)d.horizon * (double)d.n_envs;
    const double mean = (sh[0][0] + sh[0][1] + sh[0][2] + sh[0][3]) / n;
    double var = (sh[1][0] + sh[1][1] + sh[1][2] + sh[1][3]) / n - mean * mean;
    if (var < 0.0) var = 0.0;
    s_mean = (float)mean;
    s_inv = 1.0f / ((float)sqrt(var) + 1e-8f);
  }
  __syncthreads();
  const float mean = s_mean, inv = s_inv;
  const int64_t total = (int64_t)d.horizon * d.n_envs;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
    const int t = (int)(idx / d.n_envs), e = (int)(idx % d.n_envs);
    const int64_t i = (int64_t)t * d.ld_envs + e;
    d.adv[i] = (d.adv[i] - mean) * inv;
  }
}

}  // namespace

extern "C" int gmi_buffer_bind(gmi_t g, const gmi_buffer_desc* d, gmi_buffer_t* out) {
  if (!out) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_buffer_bind: out is NULL");
  *out = nullptr;
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_buffer_bind: bad instance");
  if (!d) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_buffer_bind: desc is NULL");
  if (d->horizon < 0 || d->n_envs < 0 || d->ld_envs < d->n_envs || d->obs_dim < 1 || d->act_dim < 1)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_buffer_bind: need horizon, n_envs >= 0, ld_envs >= n_envs, dims >= 1");
  if ((int64_t)d->horizon * d->ld_envs > 0 &&
      (!d->obs || !d->act || !d->logp || !d->val || !d->rew || !d->done || !d->adv || !d->ret))
    GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_buffer_bind: NULL array");
  if ((int64_t)d->horizon * d->n_envs >= (1ll << 31))
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_buffer_bind: horizon * n_envs must be below 2^31");
  gmi_buffer* b = new gmi_buffer();
  b->magic = gmi::kMagicBuffer;
  b->d = *d;
  b->n_part = (d->n_envs + kScanEnvs - 1) / kScanEnvs;      // room for either GAE kernel's partial sums
  b->part = nullptr;
  b->perm = nullptr;
  b->obs16 = nullptr;
  if (b->n_part > 0) {
    hipError_t e = hipMalloc(&b->part, sizeof(double) * 2 * (size_t)b->n_part);
    if (e == hipSuccess && d->horizon > 0) {
      e = hipMalloc(&b->perm, sizeof(int32_t) * (size_t)gmi::kPermEpochs * d->horizon * d->n_envs);
      if (e != hipSuccess) (void)hipFree(b->part);
      // observation rows that 16-byte loads cannot read: room for their bf16 copy (the trainer's chained kernel)
      if (e == hipSuccess && (d->obs_dim % 4 != 0 || ((uintptr_t)d->obs & 15) != 0)) {
        e = hipMalloc(&b->obs16, sizeof(uint16_t) * (size_t)d->horizon * d->n_envs * gmi::pad32(d->obs_dim));
        if (e != hipSuccess) { (void)hipFree(b->part); (void)hipFree(b->perm); }
      }
    }
    if (e != hipSuccess) {
      delete b;
      GMI_FAIL(GMI_ERR_HIP, "gmi_buffer_bind: hipMalloc failed: %s", hipGetErrorString(e));
    }
  }
  *out = b;
  return GMI_OK;
}

extern "C" int gmi_buffer_destroy(gmi_buffer_t b) {
  if (!valid(b)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_buffer_destroy: bad handle");
  if (b->part) (void)hipFree(b->part);
  if (b->perm) (void)hipFree(b->perm);
  if (b->obs16) (void)hipFree(b->obs16);
  b->magic = 0;
  delete b;
  return GMI_OK;
}

extern "C" int collect_experience(gmi_t g, gmi_buffer_t b, int32_t t, const float* obs, const float* act,
                                  const float* logp, const float* value, const float* reward,
                                  const uint8_t* done) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "collect_experience: bad instance");
  if (!valid(b)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "collect_experience: bad buffer");
  if (t < 0 || t >= b->d.horizon) GMI_FAIL(GMI_ERR_INVALID_ARG, "collect_experience: t=%d outside [0,%d)", t, b->d.horizon);
  if (b->d.n_envs == 0) return GMI_OK;
  if (!obs || !act || !logp || !value || !reward || !done) GMI_FAIL(GMI_ERR_INVALID_ARG, "collect_experience: NULL pointer");
  const gmi_buffer_desc& d = b->d;
  const int64_t n_obs = (int64_t)d.n_envs * d.obs_dim, n_act = (int64_t)d.n_envs * d.act_dim;
  auto aligned16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  const int vec_obs = (n_obs % 4 == 0) && aligned16(obs) && aligned16(d.obs + (int64_t)t * d.ld_envs * d.obs_dim);
  const int vec_act = (n_act % 4 == 0) && aligned16(act) && aligned16(d.act + (int64_t)t * d.ld_envs * d.act_dim);
  int64_t work = (vec_obs ? n_obs / 4 : n_obs);
  int64_t grid = (work + 255) / 256;
  if (grid > 8192) grid = 8192;
  if (grid < 1) grid = 1;
  gmi::ProfScope ps(g, gmi::kClsCollect);
  ps.launch(collect_kernel, dim3((unsigned)grid), dim3(256), 0, b->d, t, obs, act, logp, value, reward, done, vec_obs, vec_act);
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}

extern "C" int gae_compute(gmi_t g, gmi_buffer_t b, const float* last_value, float gamma, float lambda,
                           int normalize) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gae_compute: bad instance");
  if (!valid(b)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gae_compute: bad buffer");
  if (b->d.n_envs == 0 || b->d.horizon == 0) return GMI_OK;
  if (!last_value) GMI_FAIL(GMI_ERR_INVALID_ARG, "gae_compute: last_value is NULL");
  gmi::ProfScope ps(g, gmi::kClsGae);
  const int n_part = launch_gae(g_gae_variant, b->d, last_value, gamma, gamma * lambda, normalize ? b->part : nullptr,
                                [&](auto kernel, int grid, size_t lds) {
                                  ps.launch(kernel, dim3(grid), dim3(256), lds, b->d, last_value, gamma, gamma * lambda,
                                            normalize ? b->part : nullptr);
                                });
  GMI_LAUNCH_CHECK();
  if (normalize) {
    const int64_t total = (int64_t)b->d.horizon * b->d.n_envs;
    int grid = (int)((total + 1023) / 1024);
    if (grid > 2048) grid = 2048;
    ps.launch(normalize_kernel, dim3(grid), dim3(256), 0, b->d, b->part, n_part);
    GMI_LAUNCH_CHECK();
  }
  return GMI_OK;
}

// ---------------------------------------------------------------------------------------------------------
// gae_compute for callers that cannot allocate: no buffer binding (a binding owns device allocations), the
// arrays as plain pointers, and the per-workgroup partial sums of the normalisation in a file-scope device array
// instead of the binding's workspace.  Same kernels, same arithmetic, same order of additions as gae_compute.
namespace {
constexpr int kStaticPartMax = 16384;                     // workgroups of 256 envs: up to 4 194 304 envs per call
static __device__ __align__(256) double scratch[2 * kStaticPartMax];      // 256 KiB on every device the library runs on

constexpr int kMaxDevices = 64;
double* g_scratch_ptr[kMaxDevices];                       // the array's address on each device (its name is only
std::once_flag g_scratch_once[kMaxDevices];               // a host-side stand-in), looked up once per device
hipError_t g_scratch_err[kMaxDevices];

// The device array's address on `device`; looked up with that device current.
double* scratch_on(int device, hipError_t* err) {
  std::call_once(g_scratch_once[device], [device]() {
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e == hipSuccess && cur != device) e = hipSetDevice(device);
    void* p = nullptr;
    if (e == hipSuccess) e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (cur >= 0 && cur != device) (void)hipSetDevice(cur);
    g_scratch_err[device] = e;
    g_scratch_ptr[device] = e == hipSuccess ? static_cast<double*>(p) : nullptr;
  });
  *err = g_scratch_err[device];
  return g_scratch_ptr[device];
}
}  // namespace

extern "C" int gae_compute_static(gmi_t g, int32_t horizon, int32_t n_envs, int32_t ld_envs, const float* rew,
                                  const float* val, const uint8_t* done, const float* last_value, float gamma,
                                  float lambda, int normalize, float* adv, float* ret) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gae_compute_static: bad instance");
  if (horizon < 0 || n_envs < 0 || ld_envs < n_envs)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "gae_compute_static: need horizon, n_envs >= 0 and ld_envs >= n_envs");
  if ((int64_t)horizon * n_envs >= (1ll << 31))
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "gae_compute_static: horizon * n_envs must be below 2^31");
  const int variant = g_gae_variant == 1 && horizon <= 64 ? 1 : 0;
  if ((n_envs + (variant ? kScanEnvs : 256) - 1) / (variant ? kScanEnvs : 256) > kStaticPartMax)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "gae_compute_static: n_envs=%d exceeds the %d envs its fixed partial-sum array covers "
             "(use gae_compute on a buffer binding)", n_envs, 256 * kStaticPartMax);
  if (n_envs == 0 || horizon == 0) return GMI_OK;
  if (!rew || !val || !done || !last_value || !adv || !ret) GMI_FAIL(GMI_ERR_INVALID_ARG, "gae_compute_static: NULL pointer");
  if (g->device < 0 || g->device >= kMaxDevices) GMI_FAIL(GMI_ERR_UNSUPPORTED, "gae_compute_static: device %d", g->device);
  hipError_t e = hipSuccess;
  double* part = scratch_on(g->device, &e);
  if (!part) GMI_FAIL(GMI_ERR_HIP, "gae_compute_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
  gmi_buffer_desc d = {};
  d.horizon = horizon; d.n_envs = n_envs; d.ld_envs = ld_envs; d.obs_dim = 1; d.act_dim = 1;
  d.rew = const_cast<float*>(rew); d.val = const_cast<float*>(val); d.done = const_cast<uint8_t*>(done);
  d.adv = adv; d.ret = ret;
  // every workgroup of gae_kernel writes its own two partials and normalize_kernel reads exactly those: nothing
  // of an earlier call is read, so nothing needs clearing
  const int n_part = launch_gae(variant, d, last_value, gamma, gamma * lambda, normalize ? part : nullptr,
                                [&](auto kernel, int grid, size_t lds) {
                                  hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), lds, g->stream, d, last_value, gamma,
                                                     gamma * lambda, normalize ? part : nullptr);
                                });
  GMI_LAUNCH_CHECK();
  if (normalize) {
    const int64_t total = (int64_t)horizon * n_envs;
    int grid = (int)((total + 1023) / 1024);
    if (grid > 2048) grid = 2048;
    hipLaunchKernelGGL(normalize_kernel, dim3(grid), dim3(256), 0, g->stream, d, (const double*)part, n_part);
    GMI_LAUNCH_CHECK();
  }
  return GMI_OK;
}

// Measurement interface: forces one of the two GAE kernels for every later gae_compute / gae_compute_static call of
// the process (0 the serial walk, the default; 1 the wavefront scan).
extern "C" int gmi_bench_gae_variant(int variant) {
  if (variant != 0 && variant != 1) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_bench_gae_variant: 0 or 1");
  g_gae_variant = variant;
  return GMI_OK;
}
