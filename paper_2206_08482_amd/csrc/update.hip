// Trainer role (Section 3 of the paper, "DRL Trainer"; stage (ii) of Section 5.1): clipped-surrogate
// loss, exact backward through both MLPs, Adam on the fp32 master parameters, shadow refresh.
#include <math.h>

#include "internal.h"

namespace {

__device__ __forceinline__ uint16_t f_to_bf16_u(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ void store_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(uint16_t* p, float v) { *p = f_to_bf16_u(v); }

__device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}

// One thread per sample (grid-stride).  Per workgroup partial sums go to
//   stat_part[blk][0..4] = sum policy term, sum value term, entropy (workgroup 0 only), sum kl, sum clipped
//   stat_part[blk][kStatStride + j] = partial dL/dlog_std_j (without the entropy term)
// and, if want_grad, dL/dmu and dL/dv rows are written for the backward products.
template <typename T>
__global__ __launch_bounds__(256) void loss_kernel(int rows, int A, const float* __restrict__ mu,
                                                   const float* __restrict__ val, const float* __restrict__ act,
                                                   const float* __restrict__ logp_old, const float* __restrict__ adv,
                                                   const float* __restrict__ ret, const float* __restrict__ log_std,
                                                   float clip, float c_v, int want_grad, T* __restrict__ dmu,
                                                   int ld_dmu, T* __restrict__ dv, int ld_dv,
                                                   float* __restrict__ stat_part) {
  extern __shared__ float sh[];            // [4][A] log_std partials, then [4][4] stats
  float* s_dls = sh;
  float* s_st = sh + 4 * A;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 4 * A + 16; i += 256) sh[i] = 0.f;
  __syncthreads();
  const float inv_m = 1.0f / (float)rows;
  float s_pl = 0.f, s_vl = 0.f, s_kl = 0.f, s_cf = 0.f;
  const int n_iter = (rows + gridDim.x * 256 - 1) / (gridDim.x * 256);
  for (int it = 0; it < n_iter; ++it) {
    const int r = (it * gridDim.x + blockIdx.x) * 256 + tid;
    const bool ok = r < rows;
    float lp = 0.f;
    if (ok) {
      for (int j = 0; j < A; ++j) {
        const float ls = log_std[j];
        const float z = (act[(int64_t)r * A + j] - mu[(int64_t)r * A + j]) * expf(-ls);
        lp += -0.5f * z * z - ls - 0.918938533204672742f;
      }
    }
    float g_lp = 0.f;
    if (ok) {
      const float lo = logp_old[r], a = adv[r];
      const float ratio = expf(lp - lo);
      const float s1 = ratio * a;
      const float s2 = fminf(fmaxf(ratio, 1.0f - clip), 1.0f + clip) * a;
      s_pl += -fminf(s1, s2);
      s_kl += lo - lp;
      s_cf += fabsf(ratio - 1.0f) > clip ? 1.f : 0.f;
      g_lp = (s1 <= s2) ? -(a * ratio) * inv_m : 0.f;
      const float dvv = val[r] - ret[r];
      s_vl += dvv * dvv;
      if (want_grad) store_elem(dv + (int64_t)r * ld_dv, 2.0f * c_v * dvv * inv_m);
    }
    // dL/dmu_j = g_lp * z_j / sigma_j ;  dL/dlog_std_j += g_lp * (z_j^2 - 1)   (wave reduction per j)
    for (int j = 0; j < A; ++j) {
      float c = 0.f;
      if (ok) {
        const float inv_sigma = expf(-log_std[j]);
        const float z = (act[(int64_t)r * A + j] - mu[(int64_t)r * A + j]) * inv_sigma;
        if (want_grad) store_elem(dmu + (int64_t)r * ld_dmu + j, g_lp * z * inv_sigma);
        c = g_lp * (z * z - 1.0f);
      }
      c = wave_sum_f(c);
      if (lane == 0) s_dls[wave * A + j] += c;
    }
  }
  s_pl = wave_sum_f(s_pl); s_vl = wave_sum_f(s_vl); s_kl = wave_sum_f(s_kl); s_cf = wave_sum_f(s_cf);
  if (lane == 0) { s_st[wave * 4 + 0] = s_pl; s_st[wave * 4 + 1] = s_vl; s_st[wave * 4 + 2] = s_kl; s_st[wave * 4 + 3] = s_cf; }
  __syncthreads();
  float* out = stat_part + (int64_t)blockIdx.x * (gmi::kStatStride + A);
  if (tid < 4) {
    const float v = s_st[tid] + s_st[4 + tid] + s_st[8 + tid] + s_st[12 + tid];
    const int slot = tid == 0 ? 0 : (tid == 1 ? 1 : (tid == 2 ? 3 : 4));
    out[slot] = v;
  }
  if (tid == 4) {
    float ent = 0.f;
    if (blockIdx.x == 0)
      for (int j = 0; j < A; ++j) ent += log_std[j] + 1.418938533204672742f;
    out[2] = ent;
  }
  for (int j = tid; j < A; j += 256)
    out[gmi::kStatStride + j] = s_dls[j] + s_dls[A + j] + s_dls[2 * A + j] + s_dls[3 * A + j];
}

struct AdamScalars {
  float lr, b1, b2, eps, c1, c2;   // c1 = 1 - b1^k, c2 = 1 - b2^k
};

// Adam step of one parameter given its gradient (Adam as in the PPO trainer of Section 2: bias-corrected
// moments, epsilon outside the square root).
__device__ __forceinline__ float adam_one(float g, float* __restrict__ params, float* __restrict__ am,
                                          float* __restrict__ av, int64_t p, const AdamScalars& hs) {
  const float m = hs.b1 * am[p] + (1.0f - hs.b1) * g;
  const float v = hs.b2 * av[p] + (1.0f - hs.b2) * g * g;
  am[p] = m;
  av[p] = v;
  const float w = params[p] - hs.lr * (m / hs.c1) / (sqrtf(v / hs.c2) + hs.eps);
  params[p] = w;
  return w;
}

// Gradient partials of the trainer instances whose replicas are reduced into one update (one entry for an
// ordinary single-instance update): per instance [n_split, part_stride] weight partials and the loss
// kernel's [n_loss_blocks, kStatStride + A] statistics partials.
constexpr int kMaxGroup = 16;
struct PartSet {
  int n;
  const float* part[kMaxGroup];
  const float* stat[kMaxGroup];
};

// One thread per weight / bias: reduce the gradient partials, Adam, and (BF16) refresh the bias and the
// [out_pad, in_pad] weight shadow (the transposed shadow is rebuilt by shadow_transpose_kernel).
// grad(p) = (1/n) sum_i sum_s part_i[s * part_stride + p]: the in-memory mean over the n replicas
// (Section 4.1's gradient reduction for instances that share one address space), fixed summation order.
// The last workgroup instead finalises the minibatch statistics and owns log_std, whose gradient is the sum
// of the loss kernel's per-workgroup partials minus the entropy coefficient; it reduces the
// [n_loss_blocks, kStatStride + A] partials cooperatively (a serial walk by one thread per column costs
// one memory round trip per loss workgroup).
__global__ __launch_bounds__(256) void adam_kernel(gmi::ShadowTable tab, int write_shadow, float* __restrict__ params,
                                                   float* __restrict__ am, float* __restrict__ av,
                                                   PartSet ps, int n_split, int64_t part_stride,
                                                   int n_loss_blocks, int A,
                                                   float c_e, float inv_rows, AdamScalars hs, char* __restrict__ shadow,
                                                   float* __restrict__ stats_out, float* __restrict__ grad_out,
                                                   int do_update) {
  if (blockIdx.x == gridDim.x - 1) {
    __shared__ float s_col[256];
    const int C = gmi::kStatStride + A;              // columns of a statistics row
    const int tid = threadIdx.x;
    // up to 256 columns per pass; narrow rows are walked by 256 / C row groups in parallel
    const int width = C < 256 ? C : 256;
    const int groups = 256 / width;
    const bool have_stat = ps.stat[0] != nullptr;
    const float inv_n = 1.0f / (float)ps.n;
    for (int cbase = 0; cbase < C; cbase += 256) {
      const int col = cbase + tid % width, grp = tid / width;
      float s = 0.f;
      if (have_stat && grp < groups && col < C)
        for (int i = 0; i < ps.n; ++i) {
          // rows grp, grp + groups, ...: eight loads in flight, fixed order of additions
          const float* q = ps.stat[i] + col;
          int b = grp;
          for (; b + 7 * groups < n_loss_blocks; b += 8 * groups) {
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = q[(int64_t)(b + u * groups) * C];
            s += ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
          }
          for (; b < n_loss_blocks; b += groups) s += q[(int64_t)b * C];
        }
      s_col[tid] = s;
      __syncthreads();
      const int c = cbase + tid;
      if (tid < width && c < C) {
        float t = 0.f;
        for (int q = 0; q < groups; ++q) t += s_col[q * width + tid];
        t *= inv_n;                                   // mean over the replicas (exact for one)
        if (have_stat && stats_out && c < 5) stats_out[c] = c == 2 ? t : t * inv_rows;
        if (c >= gmi::kStatStride) {
          const int j = c - gmi::kStatStride;
          const int64_t p = tab.logstd_off + j;
          // without loss partials (a caller-supplied gradient) log_std takes the split sums like any weight
          float g = 0.f;
          if (have_stat) g = t - c_e;
          else for (int q = 0; q < n_split; ++q) g += ps.part[0][(int64_t)q * part_stride + p];
          if (grad_out) grad_out[p] = g;
          if (do_update) {
            const float w = adam_one(g, params, am, av, p, hs);
            if (write_shadow) reinterpret_cast<float*>(shadow + tab.sh_logstd)[j] = w;
          }
        }
      }
      __syncthreads();
    }
    return;
  }
  const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (p >= tab.logstd_off) return;
  // the moments and the parameter are fetched ahead of the partials (their latency would otherwise follow the sum's)
  float m0 = 0.f, v0 = 0.f, w0 = 0.f;
  if (do_update) { m0 = am[p]; v0 = av[p]; w0 = params[p]; }
  float g = 0.f;
  for (int i = 0; i < ps.n; ++i) {
    const float* q = ps.part[i] + p;
    int sidx = 0;
    // fixed order of additions, 16 (then 8) loads in flight
    for (; sidx + 16 <= n_split; sidx += 16) {
      float t[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) t[u] = q[(int64_t)(sidx + u) * part_stride];
#pragma unroll
      for (int u = 0; u < 16; ++u) g += t[u];
    }
    for (; sidx + 8 <= n_split; sidx += 8) {
      float t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = q[(int64_t)(sidx + u) * part_stride];
#pragma unroll
      for (int u = 0; u < 8; ++u) g += t[u];
    }
    for (; sidx < n_split; ++sidx) g += q[(int64_t)sidx * part_stride];
  }
  g *= 1.0f / (float)ps.n;
  if (grad_out) grad_out[p] = g;
  if (!do_update) return;
  // same expressions as adam_one
  const float mn = hs.b1 * m0 + (1.0f - hs.b1) * g;
  const float vn = hs.b2 * v0 + (1.0f - hs.b2) * g * g;
  am[p] = mn;
  av[p] = vn;
  const float w = w0 - hs.lr * (mn / hs.c1) / (sqrtf(vn / hs.c2) + hs.eps);
  params[p] = w;
  if (!write_shadow) return;
  int li = 0;
  while (li + 1 < tab.n && p >= tab.l[li + 1].w_off) ++li;
  const gmi::ShadowLayer& L = tab.l[li];
  if (p >= L.b_off) {
    reinterpret_cast<float*>(shadow + L.sh_b)[p - L.b_off] = w;
  } else {
    const int64_t q = p - L.w_off;
    const int o = (int)(q / L.in), i = (int)(q % L.in);
    reinterpret_cast<uint16_t*>(shadow + L.sh_w)[(int64_t)o * L.in_pad + i] = f_to_bf16_u(w);
  }
}

// Rebuilds the transposed weight shadows [in_pad, out_pad] and the fragment-major ones from the
// [out_pad, in_pad] ones through 64x64 LDS tiles, so that all sides move whole 16-byte pieces (one 2-byte
// store per weight into the transposed copy touched a different memory line for every thread of a wave).
struct TransposeTiles {
  int n;
  int start[gmi::kMaxWgradProblems + 1];
};
// Index of block (feature tile ft, k step ks) inside a chain-stream segment of nft tiles and nks k steps whose
// tiles are grouped gm, .., gm, (2), (1): groups one after the other, a group's blocks k step major.
__device__ __forceinline__ int chain_block_index(int nft, int nks, int gm, int ft, int ks) {
  const int full = nft / gm;
  int base, gs, t;
  if (ft < gm * full) {
    const int gi = ft / gm;
    base = gi * gm * nks; gs = gm; t = ft - gi * gm;
  } else {
    base = full * gm * nks;
    const int r = ft - gm * full;
    if ((nft % gm) >= 2) {
      if (r < 2) { gs = 2; t = r; }
      else { base += 2 * nks; gs = 1; t = 0; }
    } else {
      gs = 1; t = 0;
    }
  }
  return base + ks * gs + t;
}

__global__ __launch_bounds__(256) void shadow_transpose_kernel(gmi::ShadowTable tab, TransposeTiles tt, gmi::ChainEmit ce,
                                                               char* __restrict__ shadow) {
  __shared__ __attribute__((aligned(16))) uint16_t s_t[64][72];
  int li = 0;
  while (li + 1 < tt.n && (int)blockIdx.x >= tt.start[li + 1]) ++li;
  const gmi::ShadowLayer& L = tab.l[li];
  const int local = blockIdx.x - tt.start[li];
  const int n_ti = (L.in_pad + 63) / 64;
  const int o0 = (local / n_ti) * 64, i0 = (local % n_ti) * 64;
  const uint16_t* __restrict__ w = reinterpret_cast<const uint16_t*>(shadow + L.sh_w);
  uint16_t* __restrict__ wt = reinterpret_cast<uint16_t*>(shadow + L.sh_wt);
  uint16_t* __restrict__ wf = reinterpret_cast<uint16_t*>(shadow + L.sh_wf);
  const int tid = threadIdx.x, c8 = (tid & 7) * 8, r = tid >> 3;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int o = o0 + r + 32 * k, i = i0 + c8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (o < L.out_pad && i < L.in_pad) v = *reinterpret_cast<const uint4*>(w + (int64_t)o * L.in_pad + i);
    *reinterpret_cast<uint4*>(&s_t[r + 32 * k][c8]) = v;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int i = i0 + r + 32 * k, o = o0 + c8;
    if (i < L.in_pad && o < L.out_pad) {
      uint16_t e[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) e[j] = s_t[c8 + j][r + 32 * k];
      uint4 v;
      v.x = e[0] | ((uint32_t)e[1] << 16); v.y = e[2] | ((uint32_t)e[3] << 16);
      v.z = e[4] | ((uint32_t)e[5] << 16); v.w = e[6] | ((uint32_t)e[7] << 16);
      *reinterpret_cast<uint4*>(wt + (int64_t)i * L.out_pad + o) = v;
    }
  }
  // the tile holds 2 feature tiles x 4 k steps = 8 fragment blocks of 64 lanes x 16 bytes
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int idx = tid + 256 * k, blk = idx >> 6, lane = idx & 63;
    const int ol = (blk >> 2) * 32 + (lane & 31), il = (blk & 3) * 16 + (lane >> 5) * 8;
    if (o0 + ol < L.out_pad && i0 + il < L.in_pad)
      *reinterpret_cast<uint4*>(wf + gmi::wfrag_index(o0 + ol, i0 + il, L.in_pad)) =
          *reinterpret_cast<const uint4*>(&s_t[ol][il]);
  }
  // the same 8 + 8 blocks in the order and with the k permutation of the chained trainer kernel's streams:
  // lane (s, h) of a block holds, for its row, the k indices 16 ks + 8 (j / 4) + 4 h + j % 4, j = 0..7 (natural
  // order 8 h + j in the first forward layer)
  if (ce.gmax == 0) return;
  uint4* __restrict__ cs = reinterpret_cast<uint4*>(shadow + ce.out[li / ce.n_layers]);
  const gmi::ChainEmitLayer& E = ce.l[li];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int idx = tid + 256 * k, blk = idx >> 6, lane = idx & 63, h = lane >> 5;
    {   // forward segment: rows = output features, k = input features
      const int ol = (blk >> 2) * 32 + (lane & 31), il = (blk & 3) * 16;
      if (o0 + ol < L.out_pad && i0 + il < L.in_pad) {
        uint4 v;
        if (E.natural) {
          v = *reinterpret_cast<const uint4*>(&s_t[ol][il + 8 * h]);
        } else {
          const uint2 a = *reinterpret_cast<const uint2*>(&s_t[ol][il + 4 * h]);
          const uint2 b = *reinterpret_cast<const uint2*>(&s_t[ol][il + 8 + 4 * h]);
          v = make_uint4(a.x, a.y, b.x, b.y);
        }
        const int dst = E.fwd_blk + chain_block_index(L.out_pad >> 5, L.in_pad >> 4, ce.gmax, (o0 + ol) >> 5, (i0 + il) >> 4);
        cs[(int64_t)dst * 64 + lane] = v;
      }
    }
    if (E.bwd_blk >= 0) {   // input-gradient segment: rows = input features, k = output features
      const int il = (blk >> 2) * 32 + (lane & 31), ol = (blk & 3) * 16;
      if (i0 + il < L.in_pad && o0 + ol < L.out_pad) {
        uint16_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = s_t[ol + 8 * (j >> 2) + 4 * h + (j & 3)][il];
        uint4 v;
        v.x = e[0] | ((uint32_t)e[1] << 16); v.y = e[2] | ((uint32_t)e[3] << 16);
        v.z = e[4] | ((uint32_t)e[5] << 16); v.w = e[6] | ((uint32_t)e[7] << 16);
        const int dst = E.bwd_blk + chain_block_index(L.in_pad >> 5, L.out_pad >> 4, ce.gmax, (i0 + il) >> 5, (o0 + ol) >> 4);
        cs[(int64_t)dst * 64 + lane] = v;
      }
    }
  }
}

AdamScalars adam_scalars(const gmi_ppo_hparams* hp, uint32_t k) {
  AdamScalars s;
  s.lr = hp->lr; s.b1 = hp->beta1; s.b2 = hp->beta2; s.eps = hp->adam_eps;
  s.c1 = (float)(1.0 - pow((double)hp->beta1, (double)k));
  s.c2 = (float)(1.0 - pow((double)hp->beta2, (double)k));
  return s;
}

int check_hp(const char* fn, const gmi_ppo_hparams* hp) {
  if (!hp) GMI_FAIL(GMI_ERR_INVALID_ARG, "%s: hparams is NULL", fn);
  if (!(hp->clip >= 0.f) || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f))
    GMI_FAIL(GMI_ERR_INVALID_ARG, "%s: need clip >= 0 and betas in [0,1)", fn);
  return GMI_OK;
}

int check_model_buffer(const char* fn, gmi_model_t m, gmi_buffer_t b) {
  if (m->L.obs_dim != b->d.obs_dim || m->L.act_dim != b->d.act_dim)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "%s: model (obs %d, act %d) and buffer (obs %d, act %d) disagree", fn, m->L.obs_dim,
             m->L.act_dim, b->d.obs_dim, b->d.act_dim);
  return GMI_OK;
}

// The per-layer form of a minibatch pass: gather, forward of every layer, loss, and (want_grad) the input-gradient
// products, one launch each.  Leaves h, dz and one statistics row per loss workgroup (*n_loss_blocks_out rows).
int layers_pass(gmi_instance* g, gmi_model* m, gmi_buffer* b, const gmi_ppo_hparams* hp, const int32_t* idx, int rows,
                bool want_grad, int* n_loss_blocks_out) {
  const ModelLayout& L = m->L;
  const bool bf = L.dtype == GMI_DTYPE_BF16;
  const int A = L.act_dim;
  int rc = gmi::launch_gather(g, m, b->d.obs, b->d.n_envs, b->d.ld_envs, idx, rows, &b->d);
  if (rc != GMI_OK) return rc;
  rc = gmi::forward_nets(g, m, rows, true, true, m->mu, m->val);
  if (rc != GMI_OK) return rc;
  int nlb = (rows + 255) / 256;
  if (nlb > gmi::kLossBlocksMax) nlb = gmi::kLossBlocksMax;
  *n_loss_blocks_out = nlb;
  const float* log_std = bf ? reinterpret_cast<const float*>(m->shadow + L.sh_logstd) : m->params + L.logstd_off;
  const int head = L.n_layers - 1;
  const size_t lds = sizeof(float) * (4 * A + 16);
  {
    gmi::ProfScope ps(g, gmi::kClsLoss);
    if (bf)
      ps.launch(loss_kernel<uint16_t>, dim3(nlb), dim3(256), lds, rows, A, m->mu, m->val, m->mb_act, m->mb_logp, m->mb_adv, m->mb_ret,
                                                log_std, hp->clip, hp->c_v, want_grad ? 1 : 0,
                                                (uint16_t*)m->dz[0][head], L.net[0][head].out_pad,
                                                (uint16_t*)m->dz[1][head], L.net[1][head].out_pad, m->stat_part);
    else
      ps.launch(loss_kernel<float>, dim3(nlb), dim3(256), lds, rows, A, m->mu, m->val, m->mb_act, m->mb_logp, m->mb_adv, m->mb_ret,
                                             log_std, hp->clip, hp->c_v, want_grad ? 1 : 0, (float*)m->dz[0][head],
                                             L.net[0][head].out_pad, (float*)m->dz[1][head], L.net[1][head].out_pad,
                                             m->stat_part);
  }
  GMI_LAUNCH_CHECK();
  if (!want_grad) return GMI_OK;

  // input gradients, head to first hidden layer: dz[l-1] = (dz[l] W_l) * ELU'(h[l])
  for (int l = L.n_layers - 1; l >= 1; --l) {
    gmi::LinearBatch lb;
    lb.n = 2;
    for (int net = 0; net < 2; ++net) {
      const LayerInfo& li = L.net[net][l];
      gmi::LinearProblem& p = lb.p[net];
      p.x = m->dz[net][l]; p.ldx = li.out_pad;
      if (bf) {
        p.w = m->shadow + li.sh_wt; p.ldw = li.out_pad; p.wsf = li.out_pad; p.wsk = 1;
        p.K = li.out_pad; p.F = li.in_pad;
      } else {
        p.w = m->params + li.w_off; p.ldw = li.in; p.wsf = 1; p.wsk = li.in;
        p.K = li.out; p.F = li.in;
      }
      p.bias = nullptr;
      p.h = m->h[net][l]; p.ldh = li.in_pad;
      p.y = m->dz[net][l - 1]; p.ldy = li.in_pad;
      p.F_store = p.F;
      p.K_log = li.out; p.F_log = li.in;
    }
    rc = gmi::launch_linear(g, L.dtype, gmi::kEpiEluGrad, rows, lb);
    if (rc != GMI_OK) return rc;
  }
  return GMI_OK;
}

// Forward + loss (+ backward products) of the `rows` samples idx[0..rows) of the buffer.
// Leaves gradient partials in m->grad_part / m->stat_part.  Returns the split count through n_split.
int minibatch_pass(gmi_instance* g, gmi_model* m, gmi_buffer* b, const gmi_ppo_hparams* hp, const int32_t* idx,
                   int rows, bool want_grad, int* n_split_out, int* n_loss_blocks_out, bool obs16_ready = false) {
  const ModelLayout& L = m->L;
  const bool bf = L.dtype == GMI_DTYPE_BF16;
  int rc = GMI_ERR_UNSUPPORTED;
  bool blocks = false;
  if (rc == GMI_ERR_UNSUPPORTED && g->fusion >= 1 && want_grad && bf) {
    // register-chained kernel (gather + forward + loss + input gradients in one launch) where this shape has one
    rc = gmi::launch_train_chain(g, m, b, hp, idx, rows, n_loss_blocks_out, obs16_ready, &blocks);
  }
  if (rc == GMI_ERR_UNSUPPORTED) rc = layers_pass(g, m, b, hp, idx, rows, want_grad, n_loss_blocks_out);
  if (rc != GMI_OK || !want_grad) return rc;
  // weight / bias gradients of every layer of both nets in one launch
  int n_split = (rows + 63) / 64;
  if (n_split > m->n_split_max) n_split = m->n_split_max;
  if (n_split < 1) n_split = 1;
  int chunk = (rows + n_split - 1) / n_split;
  chunk = (chunk + 63) / 64 * 64;
  *n_split_out = n_split;
  gmi::WgradBatch wb;
  wb.n = 0;
  for (int net = 0; net < 2; ++net)
    for (int l = 0; l < L.n_layers; ++l) {
      const LayerInfo& li = L.net[net][l];
      gmi::WgradProblem& p = wb.p[wb.n++];
      p.dz = m->dz[net][l]; p.lddz = li.out_pad;
      p.x = m->h[net][l]; p.ldx = li.in_pad;
      p.out = li.out; p.in = li.in; p.out_pad = li.out_pad; p.in_pad = li.in_pad;
      p.w_off = li.w_off; p.b_off = li.b_off;
      // the row-tile kernel leaves every activation and every gradient in its block layout
      if (blocks && l == 0) p.x = m->x0b;
      p.x_blocks = blocks ? (l == 0 ? 2 : 1) : 0;
      p.dz_blocks = blocks ? 1 : 0;
    }
  return gmi::launch_wgrad(g, L.dtype, rows, n_split, chunk, wb, m->grad_part, L.n_params);
}

// Reduces the partials of the n bindings ms[0..n) (replicas of one model: same parameter arrays, own
// workspaces) and applies one Adam step through ms[0]; launched on instance g.
int launch_adam(gmi_instance* g, gmi_model* const* ms, int n, int n_split, int n_loss_blocks,
                const gmi_ppo_hparams* hp, int rows, uint32_t k, float* stats_out, float* grad_out, bool do_update) {
  gmi_model* m = ms[0];
  const gmi::ShadowTable tab = gmi::make_shadow_table(m->L);
  gmi::ProfScope ps(g, gmi::kClsAdam);
  // one workgroup per 256 weights / biases plus one for the statistics and log_std
  const unsigned grid = (unsigned)((m->L.logstd_off + 255) / 256) + 1;
  PartSet set;
  set.n = n;
  for (int i = 0; i < kMaxGroup; ++i) {
    set.part[i] = i < n ? ms[i]->grad_part : nullptr;
    set.stat[i] = i < n ? ms[i]->stat_part : nullptr;
  }
  const bool bf = m->L.dtype == GMI_DTYPE_BF16;
  ps.launch(adam_kernel, dim3(grid), dim3(256), 0, tab, bf ? 1 : 0, m->params, m->adam_m, m->adam_v, set, n_split,
            m->L.n_params, n_loss_blocks, m->L.act_dim, hp->c_e, 1.0f / (float)rows, adam_scalars(hp, k), m->shadow,
            stats_out, grad_out, do_update ? 1 : 0);
  GMI_LAUNCH_CHECK();
  if (bf && do_update) {
    TransposeTiles tt;
    tt.n = tab.n;
    int total = 0;
    for (int i = 0; i < tab.n; ++i) {
      tt.start[i] = total;
      total += ((tab.l[i].out_pad + 63) / 64) * ((tab.l[i].in_pad + 63) / 64);
    }
    tt.start[tab.n] = total;
    gmi::ProfScope ps2(g, gmi::kClsShadowTranspose);
    gmi::ChainEmit ce;
    gmi::fill_chain_emit(m->L, &ce);
    ps2.launch(shadow_transpose_kernel, dim3(total), dim3(256), 0, tab, tt, ce, m->shadow);
    GMI_LAUNCH_CHECK();
    return GMI_OK;
  }
  return GMI_OK;
}

}  // namespace

extern "C" int ppo_update(gmi_t g, gmi_model_t m, gmi_buffer_t b, const gmi_ppo_hparams* hp, float* stats_out) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "ppo_update: bad instance");
  if (!valid(m)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "ppo_update: bad model");
  if (!valid(b)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "ppo_update: bad buffer");
  int rc = check_hp("ppo_update", hp);
  if (rc != GMI_OK) return rc;
  rc = check_model_buffer("ppo_update", m, b);
  if (rc != GMI_OK) return rc;
  if (!m->adam_m) GMI_FAIL(GMI_ERR_INVALID_ARG, "ppo_update: the model binding has no Adam state");
  const int64_t B = (int64_t)b->d.horizon * b->d.n_envs;
  if (hp->epochs < 0 || hp->minibatch < 1) GMI_FAIL(GMI_ERR_INVALID_ARG, "ppo_update: epochs >= 0 and minibatch >= 1");
  if (B == 0 || hp->epochs == 0) return GMI_OK;
  if (B % hp->minibatch != 0)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "ppo_update: minibatch %d does not divide T*N = %lld", hp->minibatch, (long long)B);
  if (hp->minibatch > m->max_rows)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "ppo_update: minibatch %d exceeds the binding's max_rows %d", hp->minibatch, m->max_rows);
  const int nmb = (int)(B / hp->minibatch);
  uint32_t k = hp->adam_step0;
  bool obs16 = false;
  rc = gmi::prepare_obs16(g, m, b, &obs16);
  if (rc != GMI_OK) return rc;
  for (int e = 0; e < hp->epochs; ++e) {
    // the shuffles of up to kPermEpochs epochs in one launch (each launch of this small kernel is mostly latency)
    const int32_t* perm = b->perm + (int64_t)(e % gmi::kPermEpochs) * B;
    if (e % gmi::kPermEpochs == 0) {
      const int ne = hp->epochs - e < gmi::kPermEpochs ? hp->epochs - e : gmi::kPermEpochs;
      rc = gmi::launch_permutation(g, (int)B, hp->seed, hp->iteration, (uint32_t)e, ne, b->perm);
      if (rc != GMI_OK) return rc;
    }
    for (int j = 0; j < nmb; ++j) {
      int n_split = 1, nlb = 1;
      rc = minibatch_pass(g, m, b, hp, perm + (int64_t)j * hp->minibatch, hp->minibatch, true, &n_split, &nlb, obs16);
      if (rc != GMI_OK) return rc;
      ++k;
      rc = launch_adam(g, &m, 1, n_split, nlb, hp, hp->minibatch, k,
                       stats_out ? stats_out + 5 * ((int64_t)e * nmb + j) : nullptr, nullptr, true);
      if (rc != GMI_OK) return rc;
    }
  }
  return GMI_OK;
}

extern "C" int ppo_update_group(const gmi_t* gs, const gmi_model_t* ms, const gmi_buffer_t* bs, int32_t n,
                                const gmi_ppo_hparams* hp, float* stats_out) {
  if (n < 1 || n > kMaxGroup) GMI_FAIL(GMI_ERR_INVALID_ARG, "ppo_update_group: 1 <= n <= %d instances", kMaxGroup);
  if (!gs || !ms || !bs) GMI_FAIL(GMI_ERR_INVALID_ARG, "ppo_update_group: NULL handle array");
  int rc = check_hp("ppo_update_group", hp);
  if (rc != GMI_OK) return rc;
  for (int i = 0; i < n; ++i) {
    if (!valid(gs[i])) GMI_FAIL(GMI_ERR_BAD_HANDLE, "ppo_update_group: bad instance %d", i);
    if (!valid(ms[i])) GMI_FAIL(GMI_ERR_BAD_HANDLE, "ppo_update_group: bad model %d", i);
    if (!valid(bs[i])) GMI_FAIL(GMI_ERR_BAD_HANDLE, "ppo_update_group: bad buffer %d", i);
    rc = check_model_buffer("ppo_update_group", ms[i], bs[i]);
    if (rc != GMI_OK) return rc;
    for (int j = 0; j < i; ++j)
      if (gs[j] == gs[i] || ms[j] == ms[i] || bs[j] == bs[i])
        GMI_FAIL(GMI_ERR_INVALID_ARG, "ppo_update_group: entries %d and %d share a handle", j, i);
    // replicas of one model: same arrays, own workspaces
    if (ms[i]->params != ms[0]->params || ms[i]->adam_m != ms[0]->adam_m || ms[i]->adam_v != ms[0]->adam_v ||
        ms[i]->shadow != ms[0]->shadow || ms[i]->L.n_params != ms[0]->L.n_params || ms[i]->L.dtype != ms[0]->L.dtype ||
        ms[i]->n_split_max != ms[0]->n_split_max)
      GMI_FAIL(GMI_ERR_INVALID_ARG, "ppo_update_group: model %d is not a binding of model 0's parameter arrays", i);
    if (bs[i]->d.horizon != bs[0]->d.horizon || bs[i]->d.n_envs != bs[0]->d.n_envs)
      GMI_FAIL(GMI_ERR_BAD_SHAPE, "ppo_update_group: buffer %d has another size than buffer 0", i);
    if (gs[i]->device != gs[0]->device) GMI_FAIL(GMI_ERR_INVALID_ARG, "ppo_update_group: instances on different devices");
  }
  if (!ms[0]->adam_m) GMI_FAIL(GMI_ERR_INVALID_ARG, "ppo_update_group: the model bindings have no Adam state");
  const int64_t B = (int64_t)bs[0]->d.horizon * bs[0]->d.n_envs;
  if (hp->epochs < 0 || hp->minibatch < 1) GMI_FAIL(GMI_ERR_INVALID_ARG, "ppo_update_group: epochs >= 0 and minibatch >= 1");
  if (B == 0 || hp->epochs == 0) return GMI_OK;
  if (B % hp->minibatch != 0)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "ppo_update_group: minibatch %d does not divide T*N = %lld", hp->minibatch, (long long)B);
  for (int i = 0; i < n; ++i)
    if (hp->minibatch > ms[i]->max_rows)
      GMI_FAIL(GMI_ERR_BAD_SHAPE, "ppo_update_group: minibatch %d exceeds binding %d's max_rows %d", hp->minibatch, i,
               ms[i]->max_rows);
  const int nmb = (int)(B / hp->minibatch);
  uint32_t k = hp->adam_step0;
  gmi_instance* g0 = gs[0];
  gmi_model* models[kMaxGroup];
  for (int i = 0; i < n; ++i) models[i] = ms[i];
  // instance 0's stream also reads what the other instances' earlier calls left (e.g. their buffers are
  // theirs alone, but the shared parameters were last written on stream 0): nothing to order before the loop.
  bool obs16[kMaxGroup];
  for (int i = 0; i < n; ++i) {
    rc = gmi::prepare_obs16(gs[i], ms[i], bs[i], &obs16[i]);
    if (rc != GMI_OK) return rc;
  }
  for (int e = 0; e < hp->epochs; ++e) {
    if (e % gmi::kPermEpochs == 0) {
      const int ne = hp->epochs - e < gmi::kPermEpochs ? hp->epochs - e : gmi::kPermEpochs;
      for (int i = 0; i < n; ++i) {
        rc = gmi::launch_permutation(gs[i], (int)B, hp->seed + (uint64_t)i, hp->iteration, (uint32_t)e, ne, bs[i]->perm);
        if (rc != GMI_OK) return rc;
      }
    }
    const int64_t perm_off = (int64_t)(e % gmi::kPermEpochs) * B;
    for (int j = 0; j < nmb; ++j) {
      int n_split = 1, nlb = 1;
      for (int i = 0; i < n; ++i) {
        int ns_i = 1, nlb_i = 1;
        rc = minibatch_pass(gs[i], ms[i], bs[i], hp, bs[i]->perm + perm_off + (int64_t)j * hp->minibatch, hp->minibatch, true,
                            &ns_i, &nlb_i, obs16[i]);
        if (rc != GMI_OK) return rc;
        if (i == 0) { n_split = ns_i; nlb = nlb_i; }
        // replica i's partials are complete: let instance 0 see them
        if (i > 0) {
          GMI_HIP(hipEventRecord(gs[i]->event, gs[i]->stream));
          GMI_HIP(hipStreamWaitEvent(g0->stream, gs[i]->event, 0));
        }
      }
      ++k;
      rc = launch_adam(g0, models, n, n_split, nlb, hp, hp->minibatch, k,
                       stats_out ? stats_out + 5 * ((int64_t)e * nmb + j) : nullptr, nullptr, true);
      if (rc != GMI_OK) return rc;
      // the updated parameters are complete: the other instances may start their next forward pass
      if (n > 1) {
        GMI_HIP(hipEventRecord(g0->event, g0->stream));
        for (int i = 1; i < n; ++i) GMI_HIP(hipStreamWaitEvent(gs[i]->stream, g0->event, 0));
      }
    }
  }
  return GMI_OK;
}

static int check_idx_call(const char* fn, gmi_t g, gmi_model_t m, gmi_buffer_t b, const gmi_ppo_hparams* hp,
                          const int32_t* idx, int32_t n) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "%s: bad instance", fn);
  if (!valid(m)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "%s: bad model", fn);
  if (!valid(b)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "%s: bad buffer", fn);
  int rc = check_hp(fn, hp);
  if (rc != GMI_OK) return rc;
  rc = check_model_buffer(fn, m, b);
  if (rc != GMI_OK) return rc;
  if (n < 1 || n > m->max_rows) GMI_FAIL(GMI_ERR_BAD_SHAPE, "%s: n=%d outside [1, max_rows=%d]", fn, n, m->max_rows);
  if (!idx) GMI_FAIL(GMI_ERR_INVALID_ARG, "%s: idx is NULL", fn);
  return GMI_OK;
}

extern "C" int ppo_evaluate(gmi_t g, gmi_model_t m, gmi_buffer_t b, const gmi_ppo_hparams* hp, const int32_t* idx,
                            int32_t n, float* stats_out) {
  int rc = check_idx_call("ppo_evaluate", g, m, b, hp, idx, n);
  if (rc != GMI_OK) return rc;
  if (!stats_out) GMI_FAIL(GMI_ERR_INVALID_ARG, "ppo_evaluate: stats_out is NULL");
  int n_split = 0, nlb = 1;
  rc = minibatch_pass(g, m, b, hp, idx, n, false, &n_split, &nlb);
  if (rc != GMI_OK) return rc;
  return launch_adam(g, &m, 1, 0, nlb, hp, n, 1, stats_out, nullptr, false);
}

extern "C" int ppo_gradient(gmi_t g, gmi_model_t m, gmi_buffer_t b, const gmi_ppo_hparams* hp, const int32_t* idx,
                            int32_t n, float* grad_out, float* stats_out) {
  int rc = check_idx_call("ppo_gradient", g, m, b, hp, idx, n);
  if (rc != GMI_OK) return rc;
  if (!grad_out) GMI_FAIL(GMI_ERR_INVALID_ARG, "ppo_gradient: grad_out is NULL");
  int n_split = 1, nlb = 1;
  rc = minibatch_pass(g, m, b, hp, idx, n, true, &n_split, &nlb);
  if (rc != GMI_OK) return rc;
  return launch_adam(g, &m, 1, n_split, nlb, hp, n, 1, stats_out, grad_out, false);
}

extern "C" int adam_update(gmi_t g, float* params, float* adam_m, float* adam_v, const float* grad, int64_t n,
                           const gmi_ppo_hparams* hp, uint32_t step) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "adam_update: bad instance");
  int rc = check_hp("adam_update", hp);
  if (rc != GMI_OK) return rc;
  if (n < 0) GMI_FAIL(GMI_ERR_BAD_SHAPE, "adam_update: negative n");
  if (n == 0) return GMI_OK;
  if (step < 1) GMI_FAIL(GMI_ERR_INVALID_ARG, "adam_update: step is 1-based");
  if (!params || !adam_m || !adam_v || !grad) GMI_FAIL(GMI_ERR_INVALID_ARG, "adam_update: NULL pointer");
  gmi::ShadowTable tab;
  tab.n = 0;
  tab.logstd_off = n;
  tab.sh_logstd = 0;
  tab.act_dim = 0;
  tab.n_params = n;
  gmi::ProfScope ps(g, gmi::kClsAdam);
  PartSet set;
  set.n = 1;
  for (int i = 0; i < kMaxGroup; ++i) set.part[i] = set.stat[i] = nullptr;
  set.part[0] = grad;
  ps.launch(adam_kernel, dim3((unsigned)((n + 255) / 256) + 1), dim3(256), 0, tab, 0, params, adam_m, adam_v, set, 1, n,
            0, 0, 0.f, 1.f, adam_scalars(hp, step), nullptr, nullptr, nullptr, 1);
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}
