// Policy / value model: parameter layout, bf16 shadow, workspace, forward driver, and the agent role's
// action decision (Section 3 of the paper, "DRL Agent"; model shapes as in its Table 6).
#include "internal.h"
#include "rng.h"


int build_layout(const gmi_model_desc* d, ModelLayout* L) {
  if (!d) GMI_FAIL(GMI_ERR_INVALID_ARG, "model desc is NULL");
  if (d->obs_dim < 1 || d->act_dim < 1 || d->n_hidden < 1 || d->n_hidden > GMI_MAX_HIDDEN)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "model desc: need obs_dim, act_dim >= 1 and 1 <= n_hidden <= %d", GMI_MAX_HIDDEN);
  if (d->dtype != GMI_DTYPE_F32 && d->dtype != GMI_DTYPE_BF16)
    GMI_FAIL(GMI_ERR_UNSUPPORTED, "model desc: dtype %d not supported", d->dtype);
  if (d->act_dim > 1024 || d->obs_dim > 65536) GMI_FAIL(GMI_ERR_BAD_SHAPE, "model desc: act_dim <= 1024, obs_dim <= 65536");
  for (int i = 0; i < d->n_hidden; ++i)
    if (d->hidden[i] < 1 || d->hidden[i] > 65536) GMI_FAIL(GMI_ERR_BAD_SHAPE, "model desc: hidden[%d] = %d", i, d->hidden[i]);
  L->obs_dim = d->obs_dim;
  L->act_dim = d->act_dim;
  L->n_hidden = d->n_hidden;
  L->n_layers = d->n_hidden + 1;
  L->dtype = d->dtype;
  int64_t off = 0, sh = 0, wbytes = 0;
  int maxw = gmi::pad32(d->obs_dim);
  for (int net = 0; net < 2; ++net) {
    L->net[net].clear();
    int prev = d->obs_dim;
    for (int l = 0; l < L->n_layers; ++l) {
      LayerInfo li;
      li.in = prev;
      li.head = (l == L->n_layers - 1);
      li.out = li.head ? (net == 0 ? d->act_dim : 1) : d->hidden[l];
      li.in_pad = gmi::pad32(li.in);
      li.out_pad = gmi::pad32(li.out);
      li.w_off = off; off += (int64_t)li.in * li.out;
      li.b_off = off; off += li.out;
      li.sh_w = sh;  sh += gmi::align_up((int64_t)li.out_pad * li.in_pad * 2, 256);
      li.sh_wt = sh; sh += gmi::align_up((int64_t)li.out_pad * li.in_pad * 2, 256);
      li.sh_wf = sh; sh += gmi::align_up((int64_t)li.out_pad * li.in_pad * 2, 256);
      wbytes += (int64_t)li.out_pad * li.in_pad * 2;
      li.sh_b = sh;  sh += gmi::align_up((int64_t)li.out_pad * 4, 256);
      if (li.out_pad > maxw) maxw = li.out_pad;
      L->net[net].push_back(li);
      prev = li.out;
    }
  }
  L->logstd_off = off;
  off += d->act_dim;
  L->sh_logstd = sh;
  sh += gmi::align_up((int64_t)d->act_dim * 4, 256);
  L->n_params = off;
  L->weight_bytes = wbytes;
  L->max_width_pad = maxw;
  // the register-chained trainer kernel's weight streams (one per net), after everything else
  L->sh_chain_bytes = gmi::chain_stream_bytes(*L);
  for (int net = 0; net < 2; ++net) {
    L->sh_chain[net] = sh;
    sh += gmi::align_up(L->sh_chain_bytes, 256);
  }
  L->shadow_bytes = d->dtype == GMI_DTYPE_BF16 ? sh : 0;
  return GMI_OK;
}

extern "C" int64_t gmi_model_param_count(const gmi_model_desc* d) {
  ModelLayout L;
  const int rc = build_layout(d, &L);
  return rc == GMI_OK ? L.n_params : (int64_t)rc;
}

extern "C" int64_t gmi_model_shadow_bytes(const gmi_model_desc* d) {
  ModelLayout L;
  const int rc = build_layout(d, &L);
  return rc == GMI_OK ? L.shadow_bytes : (int64_t)rc;
}

namespace {

__device__ __forceinline__ uint16_t f_to_bf16_dev(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// One thread per parameter: writes its bf16 copies (W, W^T and fragment-major layouts) or fp32 bias / log_std copy.
// Padding entries of the shadow are zeroed by gmi_model_refresh_shadow and never written otherwise.
__global__ void refresh_shadow_kernel(gmi::ShadowTable tab, const float* __restrict__ params, char* __restrict__ shadow) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= tab.n_params) return;
  const float v = params[p];
  if (p >= tab.logstd_off) {
    reinterpret_cast<float*>(shadow + tab.sh_logstd)[p - tab.logstd_off] = v;
    return;
  }
  int li = 0;
  while (li + 1 < tab.n && p >= tab.l[li + 1].w_off) ++li;
  const gmi::ShadowLayer& L = tab.l[li];
  if (p >= L.b_off) {
    reinterpret_cast<float*>(shadow + L.sh_b)[p - L.b_off] = v;
  } else {
    const int64_t q = p - L.w_off;
    const int o = (int)(q / L.in), i = (int)(q % L.in);
    const uint16_t b = f_to_bf16_dev(v);
    reinterpret_cast<uint16_t*>(shadow + L.sh_w)[(int64_t)o * L.in_pad + i] = b;
    reinterpret_cast<uint16_t*>(shadow + L.sh_wt)[(int64_t)i * L.out_pad + o] = b;
    reinterpret_cast<uint16_t*>(shadow + L.sh_wf)[gmi::wfrag_index(o, i, L.in_pad)] = b;
  }
}

// Gather / convert: tpr threads share one row.  Each takes 4 consecutive observation columns per pass
// (one 16-byte load when VEC: obs_dim % 4 == 0 and a 16-byte aligned base), converts them to the model's
// element type and stores them as one 8- or 16-byte piece of x0 (zero padded to o_pad); the same threads
// then copy the row's act[A], logp, adv, ret if extras are asked for.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void gather_kernel(const float* __restrict__ obs, int n_envs, int ld_envs, int O,
                                                     int o_pad, const int32_t* __restrict__ idx, int rows,
                                                     T* __restrict__ x0, int A, const float* __restrict__ b_act,
                                                     const float* __restrict__ b_logp, const float* __restrict__ b_adv,
                                                     const float* __restrict__ b_ret, float* __restrict__ m_act,
                                                     float* __restrict__ m_logp, float* __restrict__ m_adv,
                                                     float* __restrict__ m_ret, int tpr) {
  const int tr = threadIdx.x / tpr, tc = threadIdx.x - tr * tpr;
  const int r = blockIdx.x * (256 / tpr) + tr;
  if (r >= rows) return;
  const int s = idx ? idx[r] : r;
  const int64_t slot = (int64_t)(s / n_envs) * ld_envs + (s % n_envs);
  const float* __restrict__ src = obs + slot * O;
  for (int c = tc * 4; c < o_pad; c += tpr * 4) {
    float4 v;
    if (VEC && c + 4 <= O) {
      v = *reinterpret_cast<const float4*>(src + c);
    } else {
      v.x = c + 0 < O ? src[c + 0] : 0.f;
      v.y = c + 1 < O ? src[c + 1] : 0.f;
      v.z = c + 2 < O ? src[c + 2] : 0.f;
      v.w = c + 3 < O ? src[c + 3] : 0.f;
    }
    if constexpr (sizeof(T) == 2) {
      uint2 o;
      o.x = (uint32_t)f_to_bf16_dev(v.x) | ((uint32_t)f_to_bf16_dev(v.y) << 16);
      o.y = (uint32_t)f_to_bf16_dev(v.z) | ((uint32_t)f_to_bf16_dev(v.w) << 16);
      *reinterpret_cast<uint2*>(x0 + (int64_t)r * o_pad + c) = o;
    } else {
      *reinterpret_cast<float4*>(x0 + (int64_t)r * o_pad + c) = v;
    }
  }
  if (b_act) {
    for (int j = tc; j < A + 3; j += tpr) {
      if (j < A) m_act[(int64_t)r * A + j] = b_act[slot * A + j];
      else if (j == A) m_logp[r] = b_logp[slot];
      else if (j == A + 1) m_adv[r] = b_adv[slot];
      else m_ret[r] = b_ret[slot];
    }
  }
}

// act = mu + exp(log_std) * eps; logp = sum_j [-eps_j^2/2 - log_std_j - ln(2 pi)/2]; one thread per env.
__global__ void sample_kernel(const float* __restrict__ mu, const float* __restrict__ log_std, int n, int A,
                              uint32_t k0, uint32_t k1, uint32_t step, uint32_t env_offset,
                              float* __restrict__ act, float* __restrict__ logp, float* __restrict__ mu_out) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n) return;
  float lp = 0.f;
  const int nb = (A + 3) / 4;
  for (int b = 0; b < nb; ++b) {
    float z[4];
    gmi::normal_block(env_offset + (uint32_t)e, step, gmi::kStreamAction, (uint32_t)b, k0, k1, z);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = 4 * b + i;
      if (j < A) {
        const float ls = log_std[j];
        const float m = mu[(int64_t)e * A + j];
        act[(int64_t)e * A + j] = fmaf(expf(ls), z[i], m);
        if (mu_out) mu_out[(int64_t)e * A + j] = m;
        lp += -0.5f * z[i] * z[i] - ls - 0.918938533204672742f;
      }
    }
  }
  logp[e] = lp;
}

}  // namespace

namespace gmi {

int launch_sample(gmi_instance* g, const float* mu, const float* log_std, int n_rows, int act_dim, uint64_t seed,
                  uint32_t step, uint32_t env_offset, float* act, float* logp, float* mu_out) {
  ProfScope ps(g, kClsSample);
  ps.launch(sample_kernel, dim3((n_rows + 127) / 128), dim3(128), 0, mu, log_std, n_rows, act_dim, (uint32_t)seed,
            (uint32_t)(seed >> 32), step, env_offset, act, logp, mu_out);
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}

int rollout_stepwise(gmi_instance* g, gmi_model* m, gmi_env* env, gmi_buffer* b, float* obs, uint64_t seed,
                     uint32_t step0, uint32_t env_offset, float* last_value) {
  const ModelLayout& L = m->L;
  const gmi_buffer_desc& bd = b->d;
  const int n = bd.n_envs, T = bd.horizon, O = L.obs_dim, A = L.act_dim;
  // obs_t lives in slot t of the experience arrays (step t - 1 writes its next state there), obs_T in the caller's
  // array; with a horizon of one the step would read and write the caller's array
  if (T < 2 || n > m->max_rows || !g->fusion) return GMI_ERR_UNSUPPORTED;
  const int64_t ld = bd.ld_envs;
  const int o_pad = gmi::pad32(O);
  for (int t = 0; t < T; ++t) {
    const float* cur = t == 0 ? obs : bd.obs + (int64_t)t * ld * O;
    float* nxt = t == T - 1 ? obs : bd.obs + (int64_t)(t + 1) * ld * O;
    // policy means into the model's workspace, values straight into slot t
    int rc = launch_forward_chain(g, m, cur, n, m->mu, bd.val + t * ld, t > 0 && forward_chain_reads_x0(m, cur));
    if (rc != GMI_OK) return rc;      // before anything has run if this model has no forward-only kernel (t == 0)
    StepFuse fu;
    fu.mu = m->mu;
    fu.log_std = reinterpret_cast<const float*>(m->shadow + L.sh_logstd);
    fu.ak0 = (uint32_t)seed; fu.ak1 = (uint32_t)(seed >> 32); fu.a_env_offset = env_offset;
    fu.b_obs = t == 0 ? bd.obs : nullptr;
    fu.b_act = bd.act + (int64_t)t * ld * A;
    fu.b_logp = bd.logp + t * ld;
    fu.x16_next = forward_chain_reads_x0(m, nxt) ? reinterpret_cast<uint16_t*>(m->x0) : nullptr;
    fu.o_pad = o_pad;
    rc = launch_env_step(g, env, cur, nullptr, step0 + (uint32_t)t, nxt, bd.rew + t * ld, bd.done + t * ld, &fu);
    if (rc != GMI_OK) return rc;
  }
  return launch_forward_chain(g, m, obs, n, nullptr, last_value, forward_chain_reads_x0(m, obs));
}

int launch_gather(gmi_instance* g, gmi_model* m, const float* obs, int n_envs, int ld_envs,
                  const int32_t* idx, int rows, const gmi_buffer_desc* ex) {
  return launch_gather_to(g, m, obs, n_envs, ld_envs, idx, rows, ex, m->x0);
}

int launch_gather_to(gmi_instance* g, gmi_model* m, const float* obs, int n_envs, int ld_envs,
                     const int32_t* idx, int rows, const gmi_buffer_desc* ex, void* x_out) {
  if (rows <= 0) return GMI_OK;
  ProfScope ps(g, kClsGather);
  const int O = m->L.obs_dim, A = m->L.act_dim, o_pad = gmi::pad32(O);
  int tpr = 8;                                   // threads per row: a power of two covering o_pad / 4, at most 64
  while (tpr < 64 && tpr * 4 < o_pad) tpr <<= 1;
  const unsigned grid = (unsigned)((rows + 256 / tpr - 1) / (256 / tpr));
  const bool vec = (O % 4 == 0) && (((uintptr_t)obs & 15) == 0);
  const float* e_act = ex ? ex->act : nullptr;
  const float* e_logp = ex ? ex->logp : nullptr;
  const float* e_adv = ex ? ex->adv : nullptr;
  const float* e_ret = ex ? ex->ret : nullptr;
#define GMI_GATHER(T, V)                                                                                     \
  ps.launch(gather_kernel<T, V>, dim3(grid), dim3(256), 0, obs, n_envs, ld_envs, O, o_pad, idx, rows, (T*)x_out, A, \
            e_act, e_logp, e_adv, e_ret, m->mb_act, m->mb_logp, m->mb_adv, m->mb_ret, tpr)
  if (m->L.dtype == GMI_DTYPE_BF16) {
    if (vec) GMI_GATHER(uint16_t, true); else GMI_GATHER(uint16_t, false);
  } else {
    if (vec) GMI_GATHER(float, true); else GMI_GATHER(float, false);
  }
#undef GMI_GATHER
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}

// Layer l maps h[l] (input, width in_pad) to h[l+1]; the head writes mu / val in fp32.
int forward_nets(gmi_instance* g, gmi_model* m, int rows, bool policy, bool value, float* mu_dst,
                 float* val_dst) {
  const ModelLayout& L = m->L;
  const bool bf = L.dtype == GMI_DTYPE_BF16;
  for (int l = 0; l < L.n_layers; ++l) {
    LinearBatch b;
    b.n = 0;
    for (int net = 0; net < 2; ++net) {
      if ((net == 0 && !policy) || (net == 1 && !value)) continue;
      const LayerInfo& li = L.net[net][l];
      LinearProblem& p = b.p[b.n++];
      p.x = l == 0 ? m->x0 : m->h[net][l];
      p.ldx = li.in_pad;
      if (bf) {
        p.w = m->shadow + li.sh_w; p.ldw = li.in_pad; p.wsf = li.in_pad; p.wsk = 1;
        p.bias = reinterpret_cast<const float*>(m->shadow + li.sh_b);
        p.K = li.in_pad; p.F = li.out_pad;
      } else {
        p.w = m->params + li.w_off; p.ldw = li.in; p.wsf = li.in; p.wsk = 1;
        p.bias = m->params + li.b_off;
        p.K = li.in; p.F = li.out;
      }
      p.K_log = li.in; p.F_log = li.out;
      p.h = nullptr; p.ldh = 0;
      if (li.head) {
        p.y = net == 0 ? (void*)mu_dst : (void*)val_dst;
        p.ldy = li.out;
        p.F_store = li.out;
      } else {
        p.y = m->h[net][l + 1];
        p.ldy = li.out_pad;
        p.F_store = p.F;
      }
    }
    const int rc = launch_linear(g, L.dtype, l == L.n_layers - 1 ? kEpiBiasHead : kEpiBiasElu, rows, b);
    if (rc != GMI_OK) return rc;
  }
  return GMI_OK;
}

}  // namespace gmi

extern "C" int gmi_model_bind(gmi_t g, const gmi_model_desc* d, float* params, void* shadow, float* adam_m,
                              float* adam_v, gmi_model_t* out) {
  if (!out) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_model_bind: out is NULL");
  *out = nullptr;
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_model_bind: bad instance");
  ModelLayout L;
  const int rc = build_layout(d, &L);
  if (rc != GMI_OK) return rc;
  if (!params) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_model_bind: params is NULL");
  if (L.dtype == GMI_DTYPE_BF16 && !shadow) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_model_bind: BF16 needs a shadow buffer");
  if (L.dtype == GMI_DTYPE_BF16 && ((uintptr_t)shadow & 255)) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_model_bind: shadow must be 256-byte aligned");
  if ((adam_m == nullptr) != (adam_v == nullptr)) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_model_bind: give both Adam moments or neither");
  if (d->max_rows < 1) GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_model_bind: max_rows must be >= 1");

  gmi_model* m = new gmi_model();
  m->magic = gmi::kMagicModel;
  m->device = g->device;
  m->L = L;
  m->max_rows = d->max_rows;
  m->params = params;
  m->shadow = (char*)shadow;
  m->adam_m = adam_m;
  m->adam_v = adam_v;
  {
    int n_tiles = 0;
    for (int net = 0; net < 2; ++net)
      for (int l = 0; l < L.n_layers; ++l)
        n_tiles += ((L.net[net][l].out_pad + 127) / 128) * ((L.net[net][l].in_pad + 127) / 128);
    m->n_split_max = gmi::wgrad_split_limit(n_tiles);
  }

  const int64_t rows = d->max_rows;
  const size_t es = gmi::elem_size(L.dtype);
  const int A = L.act_dim;
  // first pass sizes, second pass pointers
  for (int pass = 0; pass < 2; ++pass) {
    int64_t off = 0;
    char* base = (char*)m->ws_base;
    auto take = [&](int64_t bytes) -> void* {
      void* p = pass ? (void*)(base + off) : nullptr;
      off += gmi::align_up(bytes, 256);
      return p;
    };
    // activation arrays hold a whole number of 256-row tiles: the register-chained trainer kernel stores
    // (and loads) the ragged last tile without bounds checks; rows past the batch are never used
    const int64_t arows = (rows + 255) / 256 * 256;
    m->x0 = take(arows * gmi::pad32(L.obs_dim) * es);
    m->x0b = take(arows * gmi::pad32(L.obs_dim) * es);      // the same rows in the row-tile trainer kernel's block layout
    for (int net = 0; net < 2; ++net) {
      m->h[net][0] = m->x0;
      for (int l = 0; l < L.n_layers; ++l) {
        const LayerInfo& li = L.net[net][l];
        if (!li.head) m->h[net][l + 1] = take(arows * li.out_pad * es);
        m->dz[net][l] = take(arows * li.out_pad * es);
      }
    }
    m->mu = (float*)take(rows * A * 4);
    m->val = (float*)take(rows * 4);
    m->mb_act = (float*)take(rows * A * 4);
    m->mb_logp = (float*)take(rows * 4);
    m->mb_adv = (float*)take(rows * 4);
    m->mb_ret = (float*)take(rows * 4);
    m->grad_part = (float*)take((int64_t)m->n_split_max * L.n_params * 4);
    m->stat_part = (float*)take((int64_t)(gmi::kLossBlocksMax + 1) * (gmi::kStatStride + A) * 4);
    if (pass == 0) {
      m->ws_bytes = (size_t)off;
      hipError_t e = hipMalloc(&m->ws_base, m->ws_bytes);
      if (e != hipSuccess) {
        delete m;
        GMI_FAIL(GMI_ERR_HIP, "gmi_model_bind: hipMalloc(%zu) failed: %s", (size_t)off, hipGetErrorString(e));
      }
    }
  }
  hipError_t e = hipMemsetAsync(m->ws_base, 0, m->ws_bytes, g->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(g->stream);
  if (e != hipSuccess) {
    (void)hipFree(m->ws_base);
    delete m;
    GMI_FAIL(GMI_ERR_HIP, "gmi_model_bind: clearing the workspace failed: %s", hipGetErrorString(e));
  }
  *out = m;
  return GMI_OK;
}

extern "C" int gmi_model_destroy(gmi_model_t m) {
  if (!valid(m)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_model_destroy: bad handle");
  (void)hipFree(m->ws_base);
  m->magic = 0;
  delete m;
  return GMI_OK;
}

extern "C" int gmi_model_refresh_shadow(gmi_t g, gmi_model_t m) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_model_refresh_shadow: bad instance");
  if (!valid(m)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_model_refresh_shadow: bad model");
  if (m->L.dtype != GMI_DTYPE_BF16) return GMI_OK;
  GMI_HIP(hipMemsetAsync(m->shadow, 0, (size_t)m->L.shadow_bytes, g->stream));
  const gmi::ShadowTable tab = gmi::make_shadow_table(m->L);
  refresh_shadow_kernel<<<(unsigned)((m->L.n_params + 255) / 256), 256, 0, g->stream>>>(tab, m->params, m->shadow);
  GMI_LAUNCH_CHECK();
  return gmi::launch_chain_pack(g, m);
}

static int check_rows(const char* fn, gmi_model_t m, int n_rows) {
  if (n_rows < 0) GMI_FAIL(GMI_ERR_BAD_SHAPE, "%s: negative n_rows", fn);
  if (n_rows > m->max_rows) GMI_FAIL(GMI_ERR_BAD_SHAPE, "%s: n_rows=%d exceeds the binding's max_rows=%d", fn, n_rows, m->max_rows);
  return GMI_OK;
}

extern "C" int agent_act(gmi_t g, gmi_model_t m, const float* obs, int32_t n_rows, uint64_t seed, uint32_t step,
                         uint32_t env_offset, float* act, float* logp, float* value, float* mu) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "agent_act: bad instance");
  if (!valid(m)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "agent_act: bad model");
  int rc = check_rows("agent_act", m, n_rows);
  if (rc != GMI_OK) return rc;
  if (n_rows == 0) return GMI_OK;
  if (!obs || !act || !logp || !value) GMI_FAIL(GMI_ERR_INVALID_ARG, "agent_act: NULL pointer");
  if (g->fusion) {
    rc = gmi::launch_agent_fused(g, m, obs, n_rows, seed, step, env_offset, act, logp, value, mu, true);
    if (rc != GMI_ERR_UNSUPPORTED) return rc;
  }
  rc = g->fusion ? gmi::launch_forward_chain(g, m, obs, n_rows, m->mu, value) : GMI_ERR_UNSUPPORTED;
  if (rc == GMI_ERR_UNSUPPORTED) {
    rc = gmi::launch_gather(g, m, obs, n_rows, n_rows, nullptr, n_rows, nullptr);
    if (rc != GMI_OK) return rc;
    rc = gmi::forward_nets(g, m, n_rows, true, true, m->mu, value);
  }
  if (rc != GMI_OK) return rc;
  const float* log_std = m->L.dtype == GMI_DTYPE_BF16 ? reinterpret_cast<const float*>(m->shadow + m->L.sh_logstd)
                                                      : m->params + m->L.logstd_off;
  return gmi::launch_sample(g, m->mu, log_std, n_rows, m->L.act_dim, seed, step, env_offset, act, logp, mu);
}

extern "C" int agent_value(gmi_t g, gmi_model_t m, const float* obs, int32_t n_rows, float* value) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "agent_value: bad instance");
  if (!valid(m)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "agent_value: bad model");
  int rc = check_rows("agent_value", m, n_rows);
  if (rc != GMI_OK) return rc;
  if (n_rows == 0) return GMI_OK;
  if (!obs || !value) GMI_FAIL(GMI_ERR_INVALID_ARG, "agent_value: NULL pointer");
  if (g->fusion) {
    rc = gmi::launch_agent_fused(g, m, obs, n_rows, 0, 0, 0, nullptr, nullptr, value, nullptr, false);
    if (rc != GMI_ERR_UNSUPPORTED) return rc;
  }
  rc = g->fusion ? gmi::launch_forward_chain(g, m, obs, n_rows, nullptr, value) : GMI_ERR_UNSUPPORTED;
  if (rc != GMI_ERR_UNSUPPORTED) return rc;
  rc = gmi::launch_gather(g, m, obs, n_rows, n_rows, nullptr, n_rows, nullptr);
  if (rc != GMI_OK) return rc;
  rc = gmi::forward_nets(g, m, n_rows, false, true, nullptr, value);
  return rc;
}
