// Environment simulator role: the seeded linear-Gaussian stand-in (Section 3 of the paper describes
// the role: receive actions, return new states and rewards for hundreds or thousands of envs).
#include "internal.h"
#include "rng.h"

namespace {

// m_t[k, o] (row stride o4) = A[o, k] for k < O, B[o, k-O] for O <= k < O+A; zero padded columns.
__global__ void build_env_matrix(const float* __restrict__ a_mat, const float* __restrict__ b_mat, int O,
                                 int A, int o4, float* __restrict__ m_t) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (O + A) * o4) return;
  const int k = idx / o4, o = idx % o4;
  float v = 0.f;
  if (o < O) v = k < O ? a_mat[o * O + k] : b_mat[o * A + (k - O)];
  m_t[idx] = v;
}

// FUSED (gmi::StepFuse, internal.h): what the collection stage of a model too large for the one-launch rollout kernel
// adds to an env step -- the action decision from the policy means that the forward kernel left (the arithmetic of
// sample_kernel: same draws, same operations in the same order), the experience store of the step (copies), and the
// bf16 copy of the next state that the next step's forward kernel reads.
__device__ __forceinline__ uint32_t bf16_pair(float lo, float hi) {      // round to nearest even, as gather_kernel converts
  uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
  a += 0x7FFFu + ((a >> 16) & 1u);
  b += 0x7FFFu + ((b >> 16) & 1u);
  return (a >> 16) | (b & 0xFFFF0000u);
}

// One workgroup owns EB = G*EPT envs.  Thread (g, b): output block b (4 consecutive next-state
// elements) of envs g*EPT .. g*EPT+EPT-1.  Inputs of the workgroup's envs are staged in LDS once.
template <int EPT, bool FUSED>
__global__ __launch_bounds__(256) void env_step_kernel(
    const float* __restrict__ obs, const float* __restrict__ act, const float* __restrict__ m_t,
    uint32_t* __restrict__ episode_step, float* __restrict__ next_obs, float* __restrict__ reward,
    uint8_t* __restrict__ done, int N, int O, int A, int o4, int nb, int G, float noise_std,
    float reward_scale, uint32_t done_period, uint32_t done_threshold, uint32_t k0, uint32_t k1,
    uint32_t env_offset, uint32_t step, int vec_store, gmi::StepFuse fu) {
  extern __shared__ float smem[];
  const int OA = O + A;
  const int EB = G * EPT;
  float* s_in = smem;                          // [EB][OA]
  float* s_part = s_in + EB * OA;              // [EB][nb]
  int* s_done = (int*)(s_part + EB * nb);      // [EB]
  const int env0 = blockIdx.x * EB;
  const int tid = threadIdx.x;

  if constexpr (FUSED) {
    float* s_z = (float*)(s_done + EB);        // [EB][4 * nba] standard-normal draws of the step's actions
    const int nba = (A + 3) / 4;
    for (int idx = tid; idx < EB * O; idx += 256) {
      const int e = idx / O, k = idx % O;
      const int env = env0 + e;
      float v = 0.f;
      if (env < N) {
        v = obs[(int64_t)env * O + k];
        if (fu.b_obs) fu.b_obs[(int64_t)env * O + k] = v;
      }
      s_in[e * OA + k] = v;
    }
    for (int p = tid; p < EB * nba; p += 256) {
      const int e = p / nba, b = p % nba;
      const int env = env0 + e;
      float z[4] = {0.f, 0.f, 0.f, 0.f};
      if (env < N) gmi::normal_block(fu.a_env_offset + (uint32_t)env, step, gmi::kStreamAction, (uint32_t)b, fu.ak0, fu.ak1, z);
#pragma unroll
      for (int i = 0; i < 4; ++i) s_z[(e * nba + b) * 4 + i] = z[i];
    }
    __syncthreads();
    for (int e = tid; e < EB; e += 256) {      // one thread per env: the log-density is summed in action order
      const int env = env0 + e;
      float lp = 0.f;
      for (int j = 0; j < A; ++j) {
        float a_j = 0.f;
        if (env < N) {
          const float zj = s_z[e * nba * 4 + j];
          const float ls = fu.log_std[j];
          const float m = fu.mu[(int64_t)env * A + j];
          a_j = fmaf(expf(ls), zj, m);
          fu.b_act[(int64_t)env * A + j] = a_j;
          lp += -0.5f * zj * zj - ls - 0.918938533204672742f;
        }
        s_in[e * OA + O + j] = a_j;
      }
      if (env < N) fu.b_logp[env] = lp;
    }
  } else {
    for (int idx = tid; idx < EB * OA; idx += 256) {
      const int e = idx / OA, k = idx % OA;
      const int env = env0 + e;
      float v = 0.f;
      if (env < N) v = k < O ? obs[(int64_t)env * O + k] : act[(int64_t)env * A + (k - O)];
      s_in[idx] = v;
    }
  }
  // done flags (integer decisions): periodic counter or Bernoulli by an integer threshold
  for (int el = tid; el < EB; el += 256) {
    const int env = env0 + el;
    int d = 0;
    if (env < N) {
      const uint32_t ep = episode_step[env];
      if (done_period > 0) {
        d = ((ep + 1u) % done_period) == 0u;
      } else {
        const gmi::Words4 w = gmi::philox4x32_10(env_offset + (uint32_t)env, step, gmi::kStreamDone, 0u, k0, k1);
        d = w.w[0] < done_threshold;
      }
      episode_step[env] = d ? 0u : ep + 1u;
      done[env] = (uint8_t)d;
    }
    s_done[el] = d;
  }
  __syncthreads();

  const int b = tid % nb, g = tid / nb;
  const bool active = g < G;
  float acc[EPT][4];
#pragma unroll
  for (int i = 0; i < EPT; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  if (active) {
    const float* xin = s_in + (g * EPT) * OA;
    const float4* mrow = reinterpret_cast<const float4*>(m_t) + b;
    const int stride4 = o4 / 4;
#pragma unroll 4
    for (int k = 0; k < OA; ++k) {
      const float4 m = mrow[(int64_t)k * stride4];
#pragma unroll
      for (int i = 0; i < EPT; ++i) {
        const float x = xin[i * OA + k];
        acc[i][0] = fmaf(x, m.x, acc[i][0]);
        acc[i][1] = fmaf(x, m.y, acc[i][1]);
        acc[i][2] = fmaf(x, m.z, acc[i][2]);
        acc[i][3] = fmaf(x, m.w, acc[i][3]);
      }
    }
    // partial squared norms for the reward: this thread's 4 state elements, and its share of the action
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
      float ps = 0.f, pa = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int o = 4 * b + j;
        if (o < O) { const float x = xin[i * OA + o]; ps = fmaf(x, x, ps); }
      }
      for (int a = b; a < A; a += nb) { const float x = xin[i * OA + O + a]; pa = fmaf(x, x, pa); }
      s_part[(g * EPT + i) * nb + b] = ps + 0.01f * pa;
    }
  }
  __syncthreads();
  for (int el = tid; el < EB; el += 256) {
    if (env0 + el >= N) break;
    float s = 0.f;
    for (int j = 0; j < nb; ++j) s += s_part[el * nb + j];
    reward[env0 + el] = -reward_scale * s;
  }
  if (!active) return;
#pragma unroll
  for (int i = 0; i < EPT; ++i) {
    const int e = g * EPT + i;
    const int env = env0 + e;
    if (env >= N) continue;
    float z[4];
    float outv[4];
    if (s_done[e]) {
      gmi::normal_block(env_offset + (uint32_t)env, step, gmi::kStreamReset, (uint32_t)b, k0, k1, z);
#pragma unroll
      for (int j = 0; j < 4; ++j) outv[j] = z[j];
    } else {
      gmi::normal_block(env_offset + (uint32_t)env, step, gmi::kStreamEnv, (uint32_t)b, k0, k1, z);
#pragma unroll
      for (int j = 0; j < 4; ++j) outv[j] = fmaf(noise_std, z[j], acc[i][j]);
    }
    float* dst = next_obs + (int64_t)env * O + 4 * b;
    if (vec_store) {
      *reinterpret_cast<float4*>(dst) = make_float4(outv[0], outv[1], outv[2], outv[3]);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (4 * b + j < O) dst[j] = outv[j];
    }
    if constexpr (FUSED) {
      if (fu.x16_next) {      // rows of o_pad >= o4 two-byte elements, zero beyond O (as gather_kernel leaves them)
        const uint32_t lo = bf16_pair(4 * b + 0 < O ? outv[0] : 0.f, 4 * b + 1 < O ? outv[1] : 0.f);
        const uint32_t hi = bf16_pair(4 * b + 2 < O ? outv[2] : 0.f, 4 * b + 3 < O ? outv[3] : 0.f);
        *reinterpret_cast<uint2*>(fu.x16_next + (int64_t)env * fu.o_pad + 4 * b) = make_uint2(lo, hi);
      }
    }
  }
}

}  // namespace

extern "C" int gmi_env_bind(gmi_t g, const gmi_env_desc* d, const float* a_mat, const float* b_mat,
                            uint32_t* episode_step, gmi_env_t* out) {
  if (!out) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_env_bind: out is NULL");
  *out = nullptr;
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_env_bind: bad instance");
  if (!d || !a_mat || !b_mat || !episode_step) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_env_bind: NULL argument");
  if (d->n_envs < 0 || d->obs_dim < 1 || d->act_dim < 1 || d->obs_dim > 1024 || d->act_dim > 1024)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_env_bind: need n_envs >= 0, 1 <= obs_dim, act_dim <= 1024");
  const int O = d->obs_dim, A = d->act_dim;
  const int o4 = (O + 3) & ~3;
  float* m_t = nullptr;
  GMI_HIP(hipMalloc(&m_t, sizeof(float) * (size_t)(O + A) * o4));
  const int total = (O + A) * o4;
  build_env_matrix<<<(total + 255) / 256, 256, 0, g->stream>>>(a_mat, b_mat, O, A, o4, m_t);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipStreamSynchronize(g->stream);
  if (e != hipSuccess) {
    (void)hipFree(m_t);
    GMI_FAIL(GMI_ERR_HIP, "gmi_env_bind: building the transposed matrix failed: %s", hipGetErrorString(e));
  }
  gmi_env* env = new gmi_env();
  env->magic = gmi::kMagicEnv;
  env->d = *d;
  env->m_t = m_t;
  env->episode_step = episode_step;
  *out = env;
  return GMI_OK;
}

extern "C" int gmi_env_destroy(gmi_env_t env) {
  if (!valid(env)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_env_destroy: bad handle");
  (void)hipFree(env->m_t);
  env->magic = 0;
  delete env;
  return GMI_OK;
}

namespace gmi {
int launch_env_step(gmi_instance* g, gmi_env* env, const float* obs, const float* act, uint32_t step, float* next_obs,
                    float* reward, uint8_t* done, const StepFuse* fuse) {
  const gmi_env_desc& d = env->d;
  const int N = d.n_envs, O = d.obs_dim, A = d.act_dim;
  const int o4 = (O + 3) & ~3, nb = o4 / 4;
  const int G = 256 / nb;
  // more envs per thread once there is enough work to fill the device several times over
  int ept = 1;
  const int64_t wg1 = ((int64_t)N + G - 1) / G;
  if (wg1 >= 4096) ept = 4; else if (wg1 >= 2048) ept = 2;
  // LDS: [EB][O+A] inputs + [EB][nb] partials + [EB] flags (+ [EB][4 ceil(A/4)] action draws in the fused form)
  const int zw = fuse ? 4 * ((A + 3) / 4) : 0;
  auto lds_bytes = [&](int e) { return (size_t)(G * e) * (O + A + nb + 1 + zw) * sizeof(float); };
  while (ept > 1 && lds_bytes(ept) > 64 * 1024) ept >>= 1;
  if (lds_bytes(ept) > 64 * 1024) GMI_FAIL(GMI_ERR_UNSUPPORTED, "env_step: obs_dim + act_dim too large for the staging buffer");
  const int EB = G * ept;
  const unsigned grid = (unsigned)((N + EB - 1) / EB);
  const int vec_store = ((O & 3) == 0) && (((uintptr_t)next_obs & 15) == 0);
  const uint32_t k0 = (uint32_t)d.seed, k1 = (uint32_t)(d.seed >> 32);
  const StepFuse fu = fuse ? *fuse : StepFuse{};
  gmi::ProfScope ps(g, gmi::kClsEnvStep);
#define GMI_ENV_LAUNCH(E, F)                                                                       \
  ps.launch(env_step_kernel<E, F>, dim3(grid), dim3(256), lds_bytes(E),                                    \
      obs, act, env->m_t, env->episode_step, next_obs, reward, done, N, O, A, o4, nb, G,          \
      d.noise_std, d.reward_scale, d.done_period, d.done_threshold, k0, k1, d.env_offset, step, vec_store, fu)
  if (fuse) {
    if (ept == 4) GMI_ENV_LAUNCH(4, true); else if (ept == 2) GMI_ENV_LAUNCH(2, true); else GMI_ENV_LAUNCH(1, true);
  } else {
    if (ept == 4) GMI_ENV_LAUNCH(4, false); else if (ept == 2) GMI_ENV_LAUNCH(2, false); else GMI_ENV_LAUNCH(1, false);
  }
#undef GMI_ENV_LAUNCH
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}
}  // namespace gmi

extern "C" int env_step(gmi_t g, gmi_env_t env, const float* obs, const float* act, uint32_t step,
                        float* next_obs, float* reward, uint8_t* done) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "env_step: bad instance");
  if (!valid(env)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "env_step: bad env");
  if (env->d.n_envs == 0) return GMI_OK;
  if (!obs || !act || !next_obs || !reward || !done) GMI_FAIL(GMI_ERR_INVALID_ARG, "env_step: NULL pointer");
  if (obs == next_obs) GMI_FAIL(GMI_ERR_INVALID_ARG, "env_step: next_obs must not alias obs");
  return gmi::launch_env_step(g, env, obs, act, step, next_obs, reward, done, nullptr);
}
