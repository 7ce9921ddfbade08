// Row-tile fused MLP kernels: a workgroup owns a tile of R samples (envs), keeps the activations of the
// tile in LDS (bf16) from layer to layer, and streams each layer's bf16 weights from L2 straight into the
// matrix cores' weight operand.  One launch replaces the per-layer launches of the agent's action decision
// (Section 3 of the paper, "DRL Agent"): observation conversion, every layer of both nets, and the Gaussian
// sampling epilogue.
#include "internal.h"
#include "rng.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef float float2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float elu_f(float z) {
  // The [0, 1] clamp (an output modifier of the exponential, no instruction of its own) makes the exponential term
  // 0 for z > 0, so that one maximum replaces the compare and select; for z <= 0, e^z - 1 >= z, and where rounding
  // puts the computed difference below z (|z| < 1e-7) z is the closer value anyway.
  const float e = __builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(z * 1.44269504f), 0.f, 1.f);
  return __builtin_fmaxf(z, e - 1.0f);
}
// ELU'(z) from the stored output h = ELU(z) >= -1: 1 if h > 0 else h + 1, as one add with the [0, 1] clamp
__device__ __forceinline__ float elu_grad_f(float h) { return __builtin_amdgcn_fmed3f(h + 1.0f, 0.f, 1.f); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  float2v v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2v));
}
__device__ __forceinline__ float bf16_to_f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

struct FusedNet {
  const uint16_t* w[GMI_MAX_HIDDEN + 1];     // bf16, fragment-major copy of W [out_pad, in_pad]
  const float* bias[GMI_MAX_HIDDEN + 1];     // fp32 [out_pad]
  int in_pad[GMI_MAX_HIDDEN + 1], out_pad[GMI_MAX_HIDDEN + 1];
  int bias_off[GMI_MAX_HIDDEN + 1];          // offset (floats) of the layer's bias inside a net's LDS bias block
  int bias_total;                            // floats of that block
  int n_layers;
  int out_store;                             // logical outputs of the head
};

enum { kFEpiElu = 0, kFEpiHead = 1, kFEpiEluGrad = 2 };

// One layer for the workgroup's tile: s_out[r, f] = epi(sum_k s_in[r, k] W[f, k] + bias[f]).
// Feature tiles of 32 are dealt to the 4 waves; a wave walks its (tile, 64-wide k chunk) pairs in one
// flat loop through a ring of 4 register buffers, so the weight fragments of the next three pairs are in
// flight while one is multiplied: an L2 round trip (~1 us measured here) costs far more than a chunk's
// products, and with only one pair ahead every chunk waited for it.  The bias comes from LDS (s_bias).
// FRAG: W is the fragment-major copy (wfrag_index) instead of row-major [out_pad, in_pad].
template <int RT, int EPI, bool FRAG = true>
__device__ __forceinline__ void fused_layer(const uint16_t* __restrict__ W, const float* s_bias,
                                            int in_pad, int out_pad, const uint16_t* s_in, int stride_in,
                                            uint16_t* s_out, int stride_out, float* s_head, int head_stride,
                                            int out_store, const uint16_t* s_h = nullptr, int stride_hh = 0,
                                            int wave_id = -1) {
  // wave_id: this wave's index among the 4 that share the layer (default: a 256-thread workgroup's own);
  // made wave-uniform for the compiler: tile loops and operand addresses then run on the scalar unit
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = wave_id >= 0 ? wave_id : __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_ft = out_pad >> 5;
  const int n_my = (n_ft - wave + 3) >> 2;                 // tiles wave, wave+4, ...
  const int nchunk = (in_pad + 63) >> 6;
  const int nq = n_my > 0 ? n_my * nchunk : 0;
  const int khalf = (lane >> 5) * 8;
  floatx16 acc[RT];
  bf16x8 A0[4], A1[4], A2[4], A3[4];

  auto load_chunk = [&](bf16x8* A, int q) {
    if (q >= nq) return;
    const int tile = q / nchunk, ch = q - tile * nchunk;
    if (FRAG) {
      // k steps past the ragged end repeat the last one (never multiplied)
      const int nks = in_pad >> 4;
      const uint16_t* p = W + ((int64_t)(wave + 4 * tile) * nks) * 512 + lane * 8;
#pragma unroll
      for (int s = 0; s < 4; ++s) A[s] = *reinterpret_cast<const bf16x8*>(p + (int64_t)min(ch * 4 + s, nks - 1) * 512);
    } else {
      const int frow = (wave + 4 * tile) * 32 + (lane & 31);
      const uint16_t* p = W + (int64_t)frow * in_pad;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const int k = min(ch * 64 + s * 16 + khalf, in_pad - 8);
        A[s] = *reinterpret_cast<const bf16x8*>(p + k);
      }
    }
  };
  auto compute_chunk = [&](const bf16x8* A, int q) {
    if (q >= nq) return;
    const int tile = q / nchunk, ch = q - tile * nchunk;
    if (ch == 0) {
#pragma unroll
      for (int j = 0; j < RT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    }
    // widths are multiples of 32: a chunk holds 4 k-steps of 16, or 2 at the ragged end.  All activation
    // fragments of the chunk are read from LDS before the first product, so the reads overlap each other.
    const uint16_t* xrow = s_in + (lane & 31) * stride_in + ch * 64 + khalf;
    if (ch * 64 + 64 <= in_pad) {
      bf16x8 b[RT][4];
#pragma unroll
      for (int j = 0; j < RT; ++j)
#pragma unroll
        for (int s = 0; s < 4; ++s) b[j][s] = *reinterpret_cast<const bf16x8*>(xrow + j * 32 * stride_in + s * 16);
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int j = 0; j < RT; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[s], b[j][s], acc[j], 0, 0, 0);
    } else {
      bf16x8 b[RT][2];
#pragma unroll
      for (int j = 0; j < RT; ++j)
#pragma unroll
        for (int s = 0; s < 2; ++s) b[j][s] = *reinterpret_cast<const bf16x8*>(xrow + j * 32 * stride_in + s * 16);
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int j = 0; j < RT; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[s], b[j][s], acc[j], 0, 0, 0);
    }
    if (ch == nchunk - 1) {
      const int fb = (wave + 4 * tile) * 32;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int f = fb + g * 8 + (lane >> 5) * 4;
        float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (EPI != kFEpiEluGrad) bv = *reinterpret_cast<const float4*>(s_bias + f);
#pragma unroll
        for (int j = 0; j < RT; ++j) {
          const int r = j * 32 + (lane & 31);
          float o0 = acc[j][g * 4 + 0] + bv.x, o1 = acc[j][g * 4 + 1] + bv.y;
          float o2 = acc[j][g * 4 + 2] + bv.z, o3 = acc[j][g * 4 + 3] + bv.w;
          if (EPI == kFEpiEluGrad) {
            // times ELU'(z) expressed through the stored output h = ELU(z): 1 if h > 0 else h + 1
            const uint2 hv = *reinterpret_cast<const uint2*>(&s_h[r * stride_hh + f]);
            const float h0 = bf16_to_f((uint16_t)(hv.x & 0xFFFF)), h1 = bf16_to_f((uint16_t)(hv.x >> 16));
            const float h2 = bf16_to_f((uint16_t)(hv.y & 0xFFFF)), h3 = bf16_to_f((uint16_t)(hv.y >> 16));
            o0 *= elu_grad_f(h0); o1 *= elu_grad_f(h1);
            o2 *= elu_grad_f(h2); o3 *= elu_grad_f(h3);
            *reinterpret_cast<uint2*>(&s_out[r * stride_out + f]) = make_uint2(pack_bf16(o0, o1), pack_bf16(o2, o3));
          } else if (EPI == kFEpiElu) {
            *reinterpret_cast<uint2*>(&s_out[r * stride_out + f]) =
                make_uint2(pack_bf16(elu_f(o0), elu_f(o1)), pack_bf16(elu_f(o2), elu_f(o3)));
          } else {
            float* d = s_head + r * head_stride + f;
            if (f + 0 < out_store) d[0] = o0;
            if (f + 1 < out_store) d[1] = o1;
            if (f + 2 < out_store) d[2] = o2;
            if (f + 3 < out_store) d[3] = o3;
          }
        }
      }
    }
  };

  load_chunk(A0, 0);
  load_chunk(A1, 1);
  load_chunk(A2, 2);
  for (int q = 0; q < nq; q += 4) {
    load_chunk(A3, q + 3);
    compute_chunk(A0, q);
    load_chunk(A0, q + 4);
    compute_chunk(A1, q + 1);
    load_chunk(A1, q + 5);
    compute_chunk(A2, q + 2);
    load_chunk(A2, q + 6);
    compute_chunk(A3, q + 3);
  }
}

// Copies the biases of all layers of a net into LDS (dst[bias_off[l] + f]); the caller synchronises.
__device__ __forceinline__ void stage_biases(const FusedNet& N, float* dst, int tid0, int nthreads) {
  for (int l = 0; l < N.n_layers; ++l)
    for (int f = tid0; f < N.out_pad[l]; f += nthreads) dst[N.bias_off[l] + f] = N.bias[l][f];
}

// Runs all layers of one net on the tile whose input sits in s_x0; hidden activations ping-pong between
// s_a and s_b; the head's fp32 outputs go to s_head[r * head_stride + j].
template <int RT>
__device__ __forceinline__ void fused_net_forward(const FusedNet& N, const float* s_bias, const uint16_t* s_x0,
                                                  int stride_x0, uint16_t* s_a, uint16_t* s_b, int stride_h,
                                                  float* s_head, int head_stride) {
  const uint16_t* in = s_x0;
  int stride_in = stride_x0;
  uint16_t* out = s_a;
  for (int l = 0; l < N.n_layers - 1; ++l) {
    fused_layer<RT, kFEpiElu>(N.w[l], s_bias + N.bias_off[l], N.in_pad[l], N.out_pad[l], in, stride_in, out, stride_h,
                              nullptr, 0, 0);
    __syncthreads();
    in = out;
    stride_in = stride_h;
    out = (out == s_a) ? s_b : s_a;
  }
  const int l = N.n_layers - 1;
  fused_layer<RT, kFEpiHead>(N.w[l], s_bias + N.bias_off[l], N.in_pad[l], N.out_pad[l], in, stride_in, nullptr, 0,
                             s_head, head_stride, N.out_store);
  __syncthreads();
}

struct AgentArgs {
  FusedNet net[2];
  const float* log_std;
  const float* obs;
  int n, obs_dim, obs_pad, act_dim, max_h;
  int do_policy;
  uint32_t k0, k1, step, env_offset;
  float* act; float* logp; float* value; float* mu_out;
};

template <int RT>
__global__ __launch_bounds__(256) void agent_fused_kernel(AgentArgs a) {
  constexpr int R = RT * 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  const int stride_x0 = a.obs_pad + 8, stride_h = a.max_h + 8;
  uint16_t* s_x0 = reinterpret_cast<uint16_t*>(smem_raw);
  uint16_t* s_a = s_x0 + R * stride_x0;
  uint16_t* s_b = s_a + R * stride_h;
  float* s_mu = reinterpret_cast<float*>(s_b + R * stride_h);       // [R][act_dim]
  float* s_val = s_mu + R * a.act_dim;                              // [R]
  float* s_lp = s_val + R;                                          // [R][nb] log-prob partials
  float* s_bias = s_lp + R * ((a.act_dim + 3) >> 2);                // biases of the policy net, then the value net
  const int tid = threadIdx.x;
  const int r0 = blockIdx.x * R;

  if (a.do_policy) stage_biases(a.net[0], s_bias, tid, 256);
  stage_biases(a.net[1], s_bias + a.net[0].bias_total, tid, 256);
  // observations -> bf16 tile (zero padded columns, zero rows past the end)
  for (int idx = tid; idx < R * a.obs_pad; idx += 256) {
    const int r = idx / a.obs_pad, k = idx - r * a.obs_pad;
    float v = 0.f;
    if (r0 + r < a.n && k < a.obs_dim) v = a.obs[(int64_t)(r0 + r) * a.obs_dim + k];
    s_x0[r * stride_x0 + k] = (uint16_t)(pack_bf16(v, 0.f) & 0xFFFFu);
  }
  __syncthreads();
  if (a.do_policy) fused_net_forward<RT>(a.net[0], s_bias, s_x0, stride_x0, s_a, s_b, stride_h, s_mu, a.act_dim);
  fused_net_forward<RT>(a.net[1], s_bias + a.net[0].bias_total, s_x0, stride_x0, s_a, s_b, stride_h, s_val, 1);

  for (int r = tid; r < R; r += 256)
    if (r0 + r < a.n) a.value[r0 + r] = s_val[r];
  if (!a.do_policy) return;

  // act = mu + exp(log_std) * eps; log-prob partial per block of 4 action elements
  const int A = a.act_dim, nb = (A + 3) >> 2;
  for (int item = tid; item < R * nb; item += 256) {
    const int r = item / nb, b = item - r * nb;
    const int e = r0 + r;
    float lp = 0.f;
    if (e < a.n) {
      float z[4];
      gmi::normal_block(a.env_offset + (uint32_t)e, a.step, gmi::kStreamAction, (uint32_t)b, a.k0, a.k1, z);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = 4 * b + i;
        if (j < A) {
          const float ls = a.log_std[j];
          const float m = s_mu[r * A + j];
          a.act[(int64_t)e * A + j] = fmaf(expf(ls), z[i], m);
          if (a.mu_out) a.mu_out[(int64_t)e * A + j] = m;
          lp += -0.5f * z[i] * z[i] - ls - 0.918938533204672742f;
        }
      }
    }
    s_lp[r * nb + b] = lp;
  }
  __syncthreads();
  for (int r = tid; r < R; r += 256) {
    if (r0 + r >= a.n) continue;
    float lp = 0.f;
    for (int b = 0; b < nb; ++b) lp += s_lp[r * nb + b];
    a.logp[r0 + r] = lp;
  }
}


// ------------------------------------------------------------------------------------------------
// Experience collection of a whole horizon in one launch (Section 5.1, stage (i), with the simulator and
// the agent co-located in one instance as in Section 3): envs are independent of each other, so a workgroup
// can own R envs for all T steps and keep their state in LDS: per step it decides the actions (both nets +
// Gaussian sampling), records the experience slot, and advances the linear-Gaussian simulator; after the last
// step it evaluates the bootstrap value of the final state.  Arithmetic and Philox counters are those of
// agent_act / env_step / collect_experience called step by step.
struct RolloutArgs {
  FusedNet net[2];
  const float* log_std;
  float* obs_state;                 // [n, O]: in = state before the first step, out = state after the last
  const float* m_t;                 // [(O + A), o4] transposed env matrices
  uint32_t* episode_step;           // [n]
  int n, obs_dim, obs_pad, act_dim, max_h, o4, T, ld_envs;
  int rows_per_wg;                  // envs owned by a workgroup: the tile height, or half of it
  int n_tiles;                      // ceil(n / rows_per_wg); the grid may be smaller (workgroups loop)
  float noise_std, reward_scale;
  uint32_t done_period, done_threshold;
  uint32_t ak0, ak1, a_env_offset;  // agent's Philox key and env offset
  uint32_t ek0, ek1, e_env_offset;  // simulator's
  uint32_t step0;
  int mt_lds;                       // m_t: 2 = LDS copy kept for the whole launch, 1 = LDS copy made at every
                                    // step in the (then idle) hidden-activation space, 0 = read from global
  int obs_vec;                      // 1 = observation rows are whole 16-byte pieces in the buffer and in the LDS tile
  int noise_ahead;                  // 1 = the waves without simulator items make step t+1's random draws while the
                                    // others run step t's simulator (two buffers at byte ahead_off of the LDS)
  int ahead_off;
  float* b_obs; float* b_act; float* b_logp; float* b_val; float* b_rew; uint8_t* b_done;
  float* last_value;
};

// Simulator step for the tile: items (group of EPT envs, block of 4 state elements).  mt points at the
// transposed matrices (LDS copy or global), row stride nbo float4.
template <int EPT>
__device__ __forceinline__ void sim_items(const RolloutArgs& a, int R, int r0, uint32_t step, const float* s_in,
                                          const float4* mt, float* s_part, float* s_next, const int* s_done,
                                          const float4* s_noise, int npr, int nba) {
  const int O = a.obs_dim, A = a.act_dim, OA = O + A, o4 = a.o4, nbo = o4 >> 2;
  for (int item = threadIdx.x; item < (R / EPT) * nbo; item += blockDim.x) {
    const int g = item / nbo, b = item - g * nbo;
    const float* xin = s_in + (g * EPT) * OA;
    const float4* mrow = mt + b;
    float acc[EPT][4];
#pragma unroll
    for (int i = 0; i < EPT; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    // eight matrix rows (and state elements) are fetched before the first of their products: left to the
    // compiler under this kernel's register pressure, every k waited a full LDS round trip for its row
    int k = 0;
    for (; k + 8 <= OA; k += 8) {
      float4 m[8];
      float xv[EPT][8];
#pragma unroll
      for (int u = 0; u < 8; ++u) m[u] = mrow[(k + u) * nbo];
#pragma unroll
      for (int i = 0; i < EPT; ++i)
#pragma unroll
        for (int u = 0; u < 8; ++u) xv[i][u] = xin[i * OA + k + u];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
          acc[i][0] = fmaf(xv[i][u], m[u].x, acc[i][0]);
          acc[i][1] = fmaf(xv[i][u], m[u].y, acc[i][1]);
          acc[i][2] = fmaf(xv[i][u], m[u].z, acc[i][2]);
          acc[i][3] = fmaf(xv[i][u], m[u].w, acc[i][3]);
        }
    }
    for (; k < OA; ++k) {
      const float4 m = mrow[k * nbo];
#pragma unroll
      for (int i = 0; i < EPT; ++i) {
        const float x = xin[i * OA + k];
        acc[i][0] = fmaf(x, m.x, acc[i][0]);
        acc[i][1] = fmaf(x, m.y, acc[i][1]);
        acc[i][2] = fmaf(x, m.z, acc[i][2]);
        acc[i][3] = fmaf(x, m.w, acc[i][3]);
      }
    }
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
      const int r = g * EPT + i;
      float ps = 0.f, pa = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int o = 4 * b + j;
        if (o < O) { const float x = xin[i * OA + o]; ps = fmaf(x, x, ps); }
      }
      for (int q = b; q < A; q += nbo) { const float x = xin[i * OA + O + q]; pa = fmaf(x, x, pa); }
      s_part[r * nbo + b] = ps + 0.01f * pa;
      const int e = r0 + r;
      float z[4] = {0.f, 0.f, 0.f, 0.f};
      float outv[4];
      if (s_done[r]) {
        if (e < a.n) gmi::normal_block(a.e_env_offset + (uint32_t)e, step, gmi::kStreamReset, (uint32_t)b, a.ek0, a.ek1, z);
#pragma unroll
        for (int j = 0; j < 4; ++j) outv[j] = z[j];
      } else {
        const float4 zn = s_noise[r * npr + nba + b];       // drawn at the top of the step
        z[0] = zn.x; z[1] = zn.y; z[2] = zn.z; z[3] = zn.w;
#pragma unroll
        for (int j = 0; j < 4; ++j) outv[j] = fmaf(a.noise_std, z[j], acc[i][j]);
      }
      *reinterpret_cast<float4*>(&s_next[r * o4 + 4 * b]) = make_float4(outv[0], outv[1], outv[2], outv[3]);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Weight-stationary form of the layers, for model shapes whose share of the weights fits a wave's registers:
// the one-launch rollout runs the same layers T + 1 times, so each wave fetches the operand blocks of ITS
// feature tiles once, at kernel start, and keeps them in registers for all steps (streamed from L2 they cost
// ~2000 cycles of latency per layer and step).  Same products in the same order as fused_layer: results are
// bit-identical.  DIMS = padded widths d[0..NL] (input, hidden..., head).
template <class WS> struct WsFrags { static constexpr int value = WS::n_frags(); };
template <> struct WsFrags<void> { static constexpr int value = 1; };

// Layers LDSL.. keep their operand blocks in LDS instead (one copy per net, fragment-major as in global memory):
// with every layer in registers the kernel needed more than the 256 registers two waves per SIMD leave and the
// compiler parked values in scratch memory, whose reloads sat in every phase of every step.
template <int LDSL, int... DIMS>
struct WsShape {
  static constexpr int NL = (int)sizeof...(DIMS) - 1;
  static constexpr int lds_from = LDSL;
  static constexpr int dim(int i) {
    constexpr int d[] = {DIMS...};
    return d[i];
  }
  static constexpr int max_tiles(int l) { return (dim(l + 1) / 32 + 3) / 4; }      // feature tiles of one wave
  static constexpr int frag_base(int l) {
    int n = 0;
    for (int i = 0; i < l && i < LDSL; ++i) n += max_tiles(i) * (dim(i) / 16);
    return n;
  }
  static constexpr int n_frags() { return frag_base(NL) > 0 ? frag_base(NL) : 1; }
  // the 16-env form (16x16x32 products): 16-feature tiles of one wave, and its register fragments before layer l
  static constexpr int max_tiles16(int l) { return (dim(l + 1) / 16 + 3) / 4; }
  static constexpr int frag_base16(int l) {
    int n = 0;
    for (int i = 0; i < l && i < LDSL; ++i) n += max_tiles16(i) * (dim(i) / 32);
    return n;
  }
  // bf16 elements of the LDS-resident layers before layer l / of all of them (one net)
  static constexpr int lds_base(int l) {
    int n = 0;
    for (int i = LDSL; i < l; ++i) n += (dim(i + 1) / 32) * (dim(i) / 16) * 512;
    return n;
  }
  static constexpr int lds_elems() { return lds_base(NL); }
};

template <class WS, int L>
__device__ __forceinline__ void ws_load(bf16x8* wreg, const FusedNet& N, int wave, int lane) {
  if constexpr (L < WS::NL && L < WS::lds_from) {
    constexpr int nks = WS::dim(L) / 16, nft = WS::dim(L + 1) / 32, base = WS::frag_base(L);
#pragma unroll
    for (int i = 0; i < WS::max_tiles(L); ++i) {
      const int tile = wave + 4 * i;
      const int tc = tile < nft ? tile : nft - 1;       // a wave without an i-th tile loads a valid block it never uses
      const uint16_t* p = N.w[L] + ((int64_t)tc * nks) * 512 + lane * 8;
#pragma unroll
      for (int ks = 0; ks < nks; ++ks) wreg[base + i * nks + ks] = *reinterpret_cast<const bf16x8*>(p + (int64_t)ks * 512);
    }
    ws_load<WS, L + 1>(wreg, N, wave, lane);
  }
}

// Copies the operand blocks of the LDS-resident layers of one net into s_w (all threads of the workgroup).
template <class WS, int L>
__device__ __forceinline__ void ws_stage(uint16_t* s_w, const FusedNet& N, int tid, int nthreads) {
  if constexpr (L < WS::NL) {
    if constexpr (L >= WS::lds_from) {
      constexpr int n16 = (WS::dim(L + 1) / 32) * (WS::dim(L) / 16) * 64;       // 16-byte pieces
      const uint4* src = reinterpret_cast<const uint4*>(N.w[L]);
      uint4* dst = reinterpret_cast<uint4*>(s_w + WS::lds_base(L));
      for (int i = tid; i < n16; i += nthreads) dst[i] = src[i];
    }
    ws_stage<WS, L + 1>(s_w, N, tid, nthreads);
  }
}

template <class WS, int L, int RT, int EPI>
__device__ __forceinline__ void ws_layer(const bf16x8* wreg, const uint16_t* s_w, const float* s_bias, const uint16_t* s_in, int stride_in,
                                         uint16_t* s_out, int stride_out, float* s_head, int head_stride,
                                         int out_store, int wave, int lane) {
  constexpr int nks = WS::dim(L) / 16, nft = WS::dim(L + 1) / 32, base = WS::frag_base(L);
  const int khalf = (lane >> 5) * 8;
  const uint16_t* xrow = s_in + (lane & 31) * stride_in + khalf;
#pragma unroll
  for (int i = 0; i < WS::max_tiles(L); ++i) {
    const int tile = wave + 4 * i;
    if (tile < nft) {                                   // wave-uniform
      floatx16 acc[RT];
#pragma unroll
      for (int j = 0; j < RT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < nks; ++ks)
#pragma unroll
        for (int j = 0; j < RT; ++j) {
          const bf16x8 b = *reinterpret_cast<const bf16x8*>(xrow + j * 32 * stride_in + ks * 16);
          bf16x8 w;
          if constexpr (L < WS::lds_from) w = wreg[base + i * nks + ks];
          else w = *reinterpret_cast<const bf16x8*>(s_w + WS::lds_base(L) + (tile * nks + ks) * 512 + lane * 8);
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w, b, acc[j], 0, 0, 0);
        }
      const int fb = tile * 32;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int f = fb + g * 8 + (lane >> 5) * 4;
        const float4 bv = *reinterpret_cast<const float4*>(s_bias + f);
#pragma unroll
        for (int j = 0; j < RT; ++j) {
          const int r = j * 32 + (lane & 31);
          const float o0 = acc[j][g * 4 + 0] + bv.x, o1 = acc[j][g * 4 + 1] + bv.y;
          const float o2 = acc[j][g * 4 + 2] + bv.z, o3 = acc[j][g * 4 + 3] + bv.w;
          if (EPI == kFEpiElu) {
            *reinterpret_cast<uint2*>(&s_out[r * stride_out + f]) =
                make_uint2(pack_bf16(elu_f(o0), elu_f(o1)), pack_bf16(elu_f(o2), elu_f(o3)));
          } else {
            float* d = s_head + r * head_stride + f;
            if (f + 0 < out_store) d[0] = o0;
            if (f + 1 < out_store) d[1] = o1;
            if (f + 2 < out_store) d[2] = o2;
            if (f + 3 < out_store) d[3] = o3;
          }
        }
      }
    }
  }
}

// ---- The 16-env form of the weight-stationary nets (a workgroup that owns 16 envs): 16x16x32 products on
// 16-feature tiles, so that no row of a tile is padding -- half the matrix-instruction passes and half the epilogue
// arithmetic of the 32-row tiles.  The sums are bit-identical to those of the 32x32x16 products over the same k order
// (checked on the device over 256000 outputs of mixed magnitudes before this form was written), so the rollout stays
// bit-identical to the per-step kernels.
// Element offset, inside a layer's fragment-major array, of the 8 consecutive k values from k0 (a multiple of 8) of
// feature f: block (f / 32, k0 / 16), lane f % 32 + 32 * ((k0 / 8) % 2) of the 32x32x16 layout.
__device__ __forceinline__ int wfrag16_off(int f, int k0, int nks16) {
  return ((((f >> 5) * nks16 + (k0 >> 4)) * 64) + (f & 31) + 32 * ((k0 >> 3) & 1)) * 8;
}

// The streaming layer (fused_layer) for a 16-env tile: the same 32-feature tiles, 64-wide k chunks and ring of 4
// register buffers, but every chunk's weights fetched as the operands of 16x16x32 products (two 16-feature halves x
// two k steps of 32, from the same fragment-major copy) -- half the instruction passes and half the epilogue
// arithmetic; k runs in the same order, so the sums are those of fused_layer bit for bit.
template <int EPI>
__device__ __forceinline__ void fused_layer16(const uint16_t* __restrict__ W, const float* s_bias, int in_pad, int out_pad,
                                              const uint16_t* s_in, int stride_in, uint16_t* s_out, int stride_out,
                                              float* s_head, int head_stride, int out_store, int wave) {
  const int lane = threadIdx.x & 63, q = lane >> 4, n = lane & 15;
  const int n_ft = out_pad >> 5;
  const int n_my = (n_ft - wave + 3) >> 2;                 // tiles wave, wave+4, ...
  const int nchunk = (in_pad + 63) >> 6;
  const int nq = n_my > 0 ? n_my * nchunk : 0;
  const int nks16 = in_pad >> 4;
  floatx4 acc[2];
  bf16x8 A0[4], A1[4], A2[4], A3[4];

  auto load_chunk = [&](bf16x8* A, int qq) {
    if (qq >= nq) return;
    const int tile = qq / nchunk, ch = qq - tile * nchunk;
#pragma unroll
    for (int fh = 0; fh < 2; ++fh)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        // a k step past the ragged end repeats the last one (never multiplied)
        const int k0 = min(ch * 64 + ks * 32, in_pad - 32);
        A[fh * 2 + ks] = *reinterpret_cast<const bf16x8*>(W + wfrag16_off((wave + 4 * tile) * 32 + fh * 16 + n, k0 + q * 8, nks16));
      }
  };
  auto compute_chunk = [&](const bf16x8* A, int qq) {
    if (qq >= nq) return;
    const int tile = qq / nchunk, ch = qq - tile * nchunk;
    if (ch == 0) {
      acc[0] = floatx4{0.f, 0.f, 0.f, 0.f};
      acc[1] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    const uint16_t* xrow = s_in + n * stride_in + ch * 64 + q * 8;
    const bf16x8 b0 = *reinterpret_cast<const bf16x8*>(xrow);
    if (ch * 64 + 64 <= in_pad) {
      const bf16x8 b1 = *reinterpret_cast<const bf16x8*>(xrow + 32);
      acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[0], b0, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[2], b0, acc[1], 0, 0, 0);
      acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[1], b1, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[3], b1, acc[1], 0, 0, 0);
    } else {                                              // widths are multiples of 32: one k step at the ragged end
      acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[0], b0, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[2], b0, acc[1], 0, 0, 0);
    }
    if (ch == nchunk - 1) {
#pragma unroll
      for (int fh = 0; fh < 2; ++fh) {
        const int f = (wave + 4 * tile) * 32 + fh * 16 + 4 * q;
        const float4 bv = *reinterpret_cast<const float4*>(s_bias + f);
        const float o0 = acc[fh][0] + bv.x, o1 = acc[fh][1] + bv.y, o2 = acc[fh][2] + bv.z, o3 = acc[fh][3] + bv.w;
        if (EPI == kFEpiElu) {
          *reinterpret_cast<uint2*>(&s_out[n * stride_out + f]) =
              make_uint2(pack_bf16(elu_f(o0), elu_f(o1)), pack_bf16(elu_f(o2), elu_f(o3)));
        } else {
          float* d = s_head + n * head_stride + f;
          if (f + 0 < out_store) d[0] = o0;
          if (f + 1 < out_store) d[1] = o1;
          if (f + 2 < out_store) d[2] = o2;
          if (f + 3 < out_store) d[3] = o3;
        }
      }
    }
  };

  load_chunk(A0, 0);
  load_chunk(A1, 1);
  load_chunk(A2, 2);
  for (int qq = 0; qq < nq; qq += 4) {
    load_chunk(A3, qq + 3);
    compute_chunk(A0, qq);
    load_chunk(A0, qq + 4);
    compute_chunk(A1, qq + 1);
    load_chunk(A1, qq + 5);
    compute_chunk(A2, qq + 2);
    load_chunk(A2, qq + 6);
    compute_chunk(A3, qq + 3);
  }
}

template <class WS, int L>
__device__ __forceinline__ void ws_load16(bf16x8* wreg, const FusedNet& N, int wave, int lane) {
  if constexpr (L < WS::NL && L < WS::lds_from) {
    constexpr int nks = WS::dim(L) / 32, nks16 = WS::dim(L) / 16, nft = WS::dim(L + 1) / 16, base = WS::frag_base16(L);
    static_assert(WS::frag_base16(L + 1) <= WS::n_frags(), "the 16-env form fits the register fragments of the 32-env form");
#pragma unroll
    for (int i = 0; i < WS::max_tiles16(L); ++i) {
      const int tile = wave + 4 * i;
      const int tc = tile < nft ? tile : nft - 1;       // a wave without an i-th tile loads a valid block it never uses
      const int f = tc * 16 + (lane & 15);
#pragma unroll
      for (int ks = 0; ks < nks; ++ks)
        wreg[base + i * nks + ks] =
            *reinterpret_cast<const bf16x8*>(N.w[L] + wfrag16_off(f, ks * 32 + (lane >> 4) * 8, nks16));
    }
    ws_load16<WS, L + 1>(wreg, N, wave, lane);
  }
}

template <class WS, int L, int EPI>
__device__ __forceinline__ void ws_layer16(const bf16x8* wreg, const uint16_t* s_w, const float* s_bias, const uint16_t* s_in,
                                           int stride_in, uint16_t* s_out, int stride_out, float* s_head, int head_stride,
                                           int out_store, int wave, int lane) {
  constexpr int nks = WS::dim(L) / 32, nks16 = WS::dim(L) / 16, nft = WS::dim(L + 1) / 16, base = WS::frag_base16(L);
  const int q = lane >> 4, n = lane & 15;               // lane (n, q): env n, k values 8 q .. + 7 of a k step, features 4 q .. + 3 of a tile
  const uint16_t* xrow = s_in + n * stride_in + q * 8;
#pragma unroll
  for (int i = 0; i < WS::max_tiles16(L); ++i) {
    const int tile = wave + 4 * i;
    if (tile < nft) {                                   // wave-uniform
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < nks; ++ks) {
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(xrow + ks * 32);
        bf16x8 w;
        if constexpr (L < WS::lds_from) w = wreg[base + i * nks + ks];
        else w = *reinterpret_cast<const bf16x8*>(s_w + WS::lds_base(L) + wfrag16_off(tile * 16 + n, ks * 32 + q * 8, nks16));
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w, b, acc, 0, 0, 0);
      }
      const int f = tile * 16 + 4 * q;
      const float4 bv = *reinterpret_cast<const float4*>(s_bias + f);
      const float o0 = acc[0] + bv.x, o1 = acc[1] + bv.y, o2 = acc[2] + bv.z, o3 = acc[3] + bv.w;
      if (EPI == kFEpiElu) {
        *reinterpret_cast<uint2*>(&s_out[n * stride_out + f]) =
            make_uint2(pack_bf16(elu_f(o0), elu_f(o1)), pack_bf16(elu_f(o2), elu_f(o3)));
      } else {
        float* d = s_head + n * head_stride + f;
        if (f + 0 < out_store) d[0] = o0;
        if (f + 1 < out_store) d[1] = o1;
        if (f + 2 < out_store) d[2] = o2;
        if (f + 3 < out_store) d[3] = o3;
      }
    }
  }
}

template <class WS, int L>
__device__ __forceinline__ void ws_net16(const bf16x8* wreg, const uint16_t* s_w, const FusedNet& N, const float* s_nb,
                                         const uint16_t* in, int stride_in, uint16_t* s_a, uint16_t* s_b, int stride_h,
                                         float* s_head, int head_stride, bool run, int wave, int lane) {
  if constexpr (L < WS::NL - 1) {
    uint16_t* out = (L & 1) ? s_b : s_a;
    if (run)
      ws_layer16<WS, L, kFEpiElu>(wreg, s_w, s_nb + N.bias_off[L], in, stride_in, out, stride_h, nullptr, 0, 0, wave, lane);
    __syncthreads();
    ws_net16<WS, L + 1>(wreg, s_w, N, s_nb, out, stride_h, s_a, s_b, stride_h, s_head, head_stride, run, wave, lane);
  } else {
    if (run)
      ws_layer16<WS, L, kFEpiHead>(wreg, s_w, s_nb + N.bias_off[L], in, stride_in, nullptr, 0, s_head, head_stride,
                                   N.out_store, wave, lane);
    __syncthreads();
  }
}

// All layers of one net from layer L on, hidden activations ping-ponging between s_a and s_b as in the
// streaming form; every layer ends with a workgroup barrier.
template <class WS, int L, int RT>
__device__ __forceinline__ void ws_net(const bf16x8* wreg, const uint16_t* s_w, const FusedNet& N, const float* s_nb, const uint16_t* in,
                                       int stride_in, uint16_t* s_a, uint16_t* s_b, int stride_h, float* s_head,
                                       int head_stride, bool run, int wave, int lane) {
  if constexpr (L < WS::NL - 1) {
    uint16_t* out = (L & 1) ? s_b : s_a;
    if (run)
      ws_layer<WS, L, RT, kFEpiElu>(wreg, s_w, s_nb + N.bias_off[L], in, stride_in, out, stride_h, nullptr, 0, 0, wave, lane);
    __syncthreads();
    ws_net<WS, L + 1, RT>(wreg, s_w, N, s_nb, out, stride_h, s_a, s_b, stride_h, s_head, head_stride, run, wave, lane);
  } else {
    if (run)
      ws_layer<WS, L, RT, kFEpiHead>(wreg, s_w, s_nb + N.bias_off[L], in, stride_in, nullptr, 0, s_head, head_stride,
                                     N.out_store, wave, lane);
    __syncthreads();
  }
}

// Shapes with a weight-stationary rollout: the first two layers in registers (24 operand blocks = 96 registers per
// wave), the last two in LDS (20 KiB per net).
using WsAnt = WsShape<2, 64, 256, 128, 64, 32>;         // 60:256:128:64:8 (benchmark workload C2), 48:256:128:64:12
using WsSmallObs = WsShape<2, 32, 256, 128, 64, 32>;    // 24:256:128:64:3, 23:256:128:64:9

template <class WS>
bool ws_matches(const ModelLayout& L) {
  if (L.n_layers != WS::NL) return false;
  for (int net = 0; net < 2; ++net)
    for (int l = 0; l < WS::NL; ++l)
      if (L.net[net][l].in_pad != WS::dim(l) || L.net[net][l].out_pad != WS::dim(l + 1)) return false;
  return true;
}

// Random blocks first, first + stride, ... of one step of a tile, one float4 per (env, block): nba action-noise
// blocks, nbo env-noise blocks, then the done draw (raw word in .x).
__device__ __forceinline__ void draw_items(const RolloutArgs& a, float4* dst, uint32_t stp, int Rv, int r0, int npr, int nba,
                                           int nbo, int first, int stride) {
  for (int item = first; item < Rv * npr; item += stride) {
    const int r = item / npr, q = item - r * npr;
    const uint32_t e = (uint32_t)(r0 + r < a.n ? r0 + r : a.n - 1);
    const bool is_act = q < nba, is_env = q >= nba && q < nba + nbo;
    const uint32_t strm = is_act ? gmi::kStreamAction : (is_env ? gmi::kStreamEnv : gmi::kStreamDone);
    const uint32_t blk = is_act ? (uint32_t)q : (is_env ? (uint32_t)(q - nba) : 0u);
    const gmi::Words4 w = gmi::philox4x32_10((is_act ? a.a_env_offset : a.e_env_offset) + e, stp, strm, blk,
                                             is_act ? a.ak0 : a.ek0, is_act ? a.ak1 : a.ek1);
    float z0, z1, z2, z3;
    gmi::normal_pair(w.w[0], w.w[1], z0, z1);
    gmi::normal_pair(w.w[2], w.w[3], z2, z3);
    dst[item] = (is_act || is_env) ? make_float4(z0, z1, z2, z3) : make_float4(__uint_as_float(w.w[0]), 0.f, 0.f, 0.f);
  }
}

// 512 threads: waves 0-3 run the policy net and waves 4-7 the value net at the same time (the two nets
// have the same hidden widths, so their layers finish together and share the barriers); every other phase
// uses all 8 waves.
// WS: a WsShape whose widths the model has (weights held in registers for the whole launch), or void (weights
// streamed from L2 at every step).
// R16: the 16-env form of the weight-stationary nets (rows_per_wg == 16).
template <int RT, class WS = void, bool R16 = false>
__global__ __launch_bounds__(512) void rollout_fused_kernel(RolloutArgs a) {
  constexpr int R = RT * 32;
  constexpr int NT = 512;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  const int O = a.obs_dim, A = a.act_dim, OA = O + A, o4 = a.o4, nbo = o4 >> 2, nba = (A + 3) >> 2;
  const int stride_x0 = a.obs_pad + 8, stride_h = a.max_h + 8;
  // hidden activations (bf16, ping-pong, one pair per net) share their space with the next-state tile
  // (after the nets: next-state tile, then this step's random draws, then the staged simulator matrix)
  const int npr = nba + nbo + 1;                     // random blocks per env and step: action, env noise, done
  const size_t hid_bytes = 4 * (size_t)R * stride_h * 2, next_bytes = ((size_t)R * o4 * 4 + 15) & ~(size_t)15;
  const size_t noise_bytes = (size_t)R * npr * 16;
  const size_t region = ((hid_bytes > next_bytes + noise_bytes ? hid_bytes : next_bytes + noise_bytes) + 15) & ~(size_t)15;
  float* s_in = reinterpret_cast<float*>(smem_raw);                                  // [R][O + A] state | action
  uint16_t* s_x0 = reinterpret_cast<uint16_t*>(s_in + ((R * OA + 3) & ~3));          // [R][obs_pad + 8]
  unsigned char* s_reg = reinterpret_cast<unsigned char*>(s_x0 + R * stride_x0);
  uint16_t* s_hid = reinterpret_cast<uint16_t*>(s_reg);                              // [2 nets][2][R][stride_h]
  float* s_next = reinterpret_cast<float*>(s_reg);                                   // [R][o4]
  float* s_mu = reinterpret_cast<float*>(s_reg + region);                            // [R][A]
  float* s_val = s_mu + R * A;                                                       // [R]
  float* s_lp = s_val + R;                                                           // [R][nba]
  float* s_part = s_lp + R * nba;                                                    // [R][nbo]
  int* s_done = reinterpret_cast<int*>(s_part + R * nbo);                            // [R]
  float* s_bias = reinterpret_cast<float*>(s_done + ((R + 3) & ~3));                 // policy biases, value biases
  // this step's random draws, one float4 per (env, block): nba action-noise blocks, nbo env-noise blocks, then
  // the done draw (raw word in .x); in the hidden-activation space, which is idle once the heads are done
  float4* s_noise_inplace = reinterpret_cast<float4*>(s_reg + next_bytes);
  float* s_mt = s_bias + ((a.net[0].bias_total + a.net[1].bias_total + 3) & ~3);     // [O + A][o4] when mt_lds == 2
  // weight-stationary form: operand blocks of the LDS-resident layers, policy net then value net
  uint16_t* s_wl = reinterpret_cast<uint16_t*>(s_mt + (a.mt_lds == 2 ? OA * o4 : 0));
  float4* s_ahead = reinterpret_cast<float4*>(smem_raw + a.ahead_off);                // [2][Rv][npr] when noise_ahead
  const int tid = threadIdx.x;
  // wave-uniform values, so that the per-net kernel arguments are fetched by scalar loads
  const int half = __builtin_amdgcn_readfirstlane(tid >> 8), wave4 = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);
  // Rv <= R envs are owned by this workgroup (a half-filled tile doubles the workgroups of a small batch);
  // rows Rv..R-1 of the tile go through the matrix products but are never read or stored
  const int Rv = a.rows_per_wg;
  // first thread of the first wave without a simulator item (rollout_sim_threads on the host)
  const int ahead_tid0 = ((((Rv / 4) * nbo >= 192 ? (Rv / 4) * nbo : Rv * nbo) + 63) & ~63);
  // the observation stores go to the waves without action items when those are at least half of the workgroup
  // (in the simulator phase the idle waves have no time to spare: measured, the next step's draws fill it)
  const int act_waves_end = (Rv * nba * 4 + 63) & ~63;
  const int obs_tid0 = act_waves_end <= NT / 2 ? act_waves_end : 0;
  for (int idx = tid; idx < (R - Rv) * stride_x0; idx += NT) s_x0[Rv * stride_x0 + idx] = 0;
  stage_biases(a.net[0], s_bias, tid, NT);
  stage_biases(a.net[1], s_bias + a.net[0].bias_total, tid, NT);
  if (a.mt_lds == 2)
    for (int idx = tid; idx < OA * nbo; idx += NT)
      reinterpret_cast<float4*>(s_mt)[idx] = reinterpret_cast<const float4*>(a.m_t)[idx];
  float4* s_stage = reinterpret_cast<float4*>(s_reg + next_bytes + noise_bytes);
  // the simulator matrix as an LDS pointer (resident copy or per-step staging) or as a global pointer: kept apart,
  // because one pointer that may be either makes every access a flat load (measured: the 68-step matrix-vector
  // loop of a 60-dimensional env took 8600 cycles through flat loads)
  const float4* mt_lds_ptr = a.mt_lds == 2 ? reinterpret_cast<const float4*>(s_mt) : s_stage;
  const float4* mt_glb_ptr = reinterpret_cast<const float4*>(a.m_t);
  const FusedNet& N = a.net[half];
  uint16_t* s_a = s_hid + (size_t)half * 2 * R * stride_h;
  uint16_t* s_b = s_a + R * stride_h;
  float* s_head = half ? s_val : s_mu;
  const int head_stride = half ? 1 : A;
  const float* s_nb = s_bias + (half ? a.net[0].bias_total : 0);
  constexpr bool kStationary = !std::is_void<WS>::value;
  // this wave's weight operands, fetched once (a dummy single entry in the streaming form)
  bf16x8 wreg[WsFrags<WS>::value];
  const uint16_t* s_w = s_wl;
  if constexpr (kStationary) {
    if constexpr (R16) ws_load16<WS, 0>(wreg, N, wave4, tid & 63);
    else ws_load<WS, 0>(wreg, N, wave4, tid & 63);
    ws_stage<WS, 0>(s_wl, a.net[0], tid, NT);
    ws_stage<WS, 0>(s_wl + WS::lds_elems(), a.net[1], tid, NT);
    s_w = s_wl + (half ? WS::lds_elems() : 0);
  }

  // The grid never exceeds what the instance's compute units hold at once: a workgroup takes the tiles
  // blockIdx.x, blockIdx.x + gridDim.x, ... one after the other, each through all T steps.  (Workgroups
  // that wait for a free compute unit would keep the dispatcher from placing other instances' kernels.)
  for (int tile = blockIdx.x; tile < a.n_tiles; tile += gridDim.x) {
  const int r0 = tile * Rv;
  for (int idx = tid; idx < Rv * O; idx += NT) {
    const int r = idx / O, k = idx - r * O;
    s_in[r * OA + k] = (r0 + r < a.n) ? a.obs_state[(int64_t)(r0 + r) * O + k] : 0.f;
  }
  // thread NT - 64 + r (r < Rv; the last wave, which has no action items and gets an observation-store item last of
  // all: on the fifth wave the done flags came after an observation store and that wave ended the sampling phase
  // 1000 cycles after the others) carries env r's episode counter and makes its done flag
  const int dtid = tid - (NT - 64);
  uint32_t ep = 0;
  if (dtid >= 0 && dtid < Rv && r0 + dtid < a.n) ep = a.episode_step[r0 + dtid];
  if (a.noise_ahead) draw_items(a, s_ahead, a.step0, Rv, r0, npr, nba, nbo, tid, NT);
  __syncthreads();
  // the nets' bf16 copy of the state, zero padded; every later step refreshes it together with the state itself
  for (int idx = tid; idx < Rv * a.obs_pad; idx += NT) {
    const int r = idx / a.obs_pad, k = idx - r * a.obs_pad;
    const float v = k < O ? s_in[r * OA + k] : 0.f;
    s_x0[r * stride_x0 + k] = (uint16_t)(pack_bf16(v, 0.f) & 0xFFFFu);
  }
  __syncthreads();

  for (int t = 0; t <= a.T; ++t) {
    // both nets, layer by layer; after the last step only the value net (bootstrap value)
    const bool run = half == 1 || t < a.T;
    if constexpr (kStationary) {
      if constexpr (R16)
        ws_net16<WS, 0>(wreg, s_w, N, s_nb, s_x0, stride_x0, s_a, s_b, stride_h, s_head, head_stride, run, wave4, tid & 63);
      else
        ws_net<WS, 0, RT>(wreg, s_w, N, s_nb, s_x0, stride_x0, s_a, s_b, stride_h, s_head, head_stride, run, wave4, tid & 63);
    } else {
      const uint16_t* in = s_x0;
      int stride_in = stride_x0;
      uint16_t* out = s_a;
      for (int l = 0; l < N.n_layers - 1; ++l) {
        if (run) {
          if constexpr (R16)
            fused_layer16<kFEpiElu>(N.w[l], s_nb + N.bias_off[l], N.in_pad[l], N.out_pad[l], in, stride_in, out, stride_h,
                                    nullptr, 0, 0, wave4);
          else
            fused_layer<RT, kFEpiElu>(N.w[l], s_nb + N.bias_off[l], N.in_pad[l], N.out_pad[l], in, stride_in, out, stride_h,
                                      nullptr, 0, 0, nullptr, 0, wave4);
        }
        __syncthreads();
        in = out;
        stride_in = stride_h;
        out = (out == s_a) ? s_b : s_a;
      }
      const int l = N.n_layers - 1;
      if (run) {
        if constexpr (R16)
          fused_layer16<kFEpiHead>(N.w[l], s_nb + N.bias_off[l], N.in_pad[l], N.out_pad[l], in, stride_in, nullptr, 0,
                                   s_head, head_stride, N.out_store, wave4);
        else
          fused_layer<RT, kFEpiHead>(N.w[l], s_nb + N.bias_off[l], N.in_pad[l], N.out_pad[l], in, stride_in, nullptr, 0,
                                     s_head, head_stride, N.out_store, nullptr, 0, wave4);
      }
      __syncthreads();
    }
    if (t == a.T) {
      if (tid < Rv && r0 + tid < a.n) a.last_value[r0 + tid] = s_val[tid];
      break;
    }

    // All random draws of this step, one block per thread and the same instructions for every kind of block
    // (left where they are used, they ran on the few threads of the sampling phase and inside the simulator's
    // matrix product).  With noise_ahead they were made during the previous step's simulator phase.
    float4* s_noise = a.noise_ahead ? s_ahead + (size_t)(t & 1) * Rv * npr : s_noise_inplace;
    if (!a.noise_ahead) {
      draw_items(a, s_noise, a.step0 + (uint32_t)t, Rv, r0, npr, nba, nbo, tid, NT);
      __syncthreads();
    }
    const uint32_t step = a.step0 + (uint32_t)t;
    const int64_t slot0 = (int64_t)t * a.ld_envs + r0;
    // action = mu + exp(log_std) * eps, log-prob partials per block of 4 action elements: one thread per element;
    // the four terms of a block are added in index order through lane exchanges (((t0 + t1) + t2) + t3, the order
    // of a single accumulator), so that one thread per block no longer walks its four elements one after the other
    for (int item = tid; item < Rv * nba * 4; item += NT) {
      const int blk = item >> 2, i = item & 3;
      const int r = blk / nba, b = blk - r * nba;
      const int e = r0 + r, j = 4 * b + i;
      float term = 0.f;
      if (j < A) {
        float act = 0.f;
        if (e < a.n) {
          const float z = reinterpret_cast<const float*>(s_noise + r * npr + b)[i];
          const float ls = a.log_std[j];
          act = fmaf(expf(ls), z, s_mu[r * A + j]);
          a.b_act[(slot0 + r) * A + j] = act;
          term = -0.5f * z * z - ls - 0.918938533204672742f;
        }
        s_in[r * OA + O + j] = act;
      }
      float lp = term;
      lp += __shfl_down(term, 1, 64);
      lp += __shfl_down(term, 2, 64);
      lp += __shfl_down(term, 3, 64);
      if (i == 0) s_lp[blk] = lp;
    }
    // this step's observations to the buffer, by the waves without action items
    if (tid >= obs_tid0) {
      if (a.obs_vec) {          // rows of whole 16-byte pieces on both sides: a quarter of the stores
        const int o4n = O >> 2;
        for (int idx = tid - obs_tid0; idx < Rv * o4n; idx += NT - obs_tid0) {
          const int r = idx / o4n, c = idx - r * o4n;
          const float4 v = *reinterpret_cast<const float4*>(s_in + r * OA + 4 * c);
          if (r0 + r < a.n) *reinterpret_cast<float4*>(a.b_obs + (slot0 + r) * O + 4 * c) = v;
        }
      } else {
        for (int idx = tid - obs_tid0; idx < Rv * O; idx += NT - obs_tid0) {
          const int r = idx / O, k = idx - r * O;
          if (r0 + r < a.n) a.b_obs[(slot0 + r) * O + k] = s_in[r * OA + k];
        }
      }
    }
    if (dtid >= 0 && dtid < Rv) {
      const int e = r0 + dtid;
      int d = 0;
      if (e < a.n) {
        if (a.done_period > 0) {
          d = ((ep + 1u) % a.done_period) == 0u;
        } else {
          d = __float_as_uint(s_noise[dtid * npr + nba + nbo].x) < a.done_threshold;
        }
        ep = d ? 0u : ep + 1u;
        a.b_done[slot0 + dtid] = (uint8_t)d;
        a.b_val[slot0 + dtid] = s_val[dtid];
      }
      s_done[dtid] = d;
    }
    __syncthreads();
    if (tid < Rv && r0 + tid < a.n) {
      float lp = 0.f;
      for (int b = 0; b < nba; ++b) lp += s_lp[tid * nba + b];
      a.b_logp[slot0 + tid] = lp;
    }
    // simulator: next = A s + B act + noise_std * eps (or a fresh N(0,1) state after a done); as many envs
    // per item as still leaves an item for every thread
    if (a.mt_lds == 1) {
      for (int idx = tid; idx < OA * nbo; idx += NT) s_stage[idx] = reinterpret_cast<const float4*>(a.m_t)[idx];
      __syncthreads();
    }
    // the next step's draws, by the waves that have no simulator item
    if (a.noise_ahead && t + 1 < a.T && tid >= ahead_tid0)
      draw_items(a, s_ahead + (size_t)((t + 1) & 1) * Rv * npr, step + 1u, Rv, r0, npr, nba, nbo, tid - ahead_tid0, NT - ahead_tid0);
    if (a.mt_lds != 0) {
      if ((Rv / 4) * nbo >= 192) sim_items<4>(a, Rv, r0, step, s_in, mt_lds_ptr, s_part, s_next, s_done, s_noise, npr, nba);
      else sim_items<1>(a, Rv, r0, step, s_in, mt_lds_ptr, s_part, s_next, s_done, s_noise, npr, nba);
    } else {
      if ((Rv / 4) * nbo >= 192) sim_items<4>(a, Rv, r0, step, s_in, mt_glb_ptr, s_part, s_next, s_done, s_noise, npr, nba);
      else sim_items<1>(a, Rv, r0, step, s_in, mt_glb_ptr, s_part, s_next, s_done, s_noise, npr, nba);
    }
    __syncthreads();
    // the reward on the last wave (the state update below starts with the first threads)
    const int rt = tid - (NT - 64);
    if (rt >= 0 && rt < Rv && r0 + rt < a.n) {
      // same order of additions as one by one, eight LDS reads in flight
      const float* q = s_part + rt * nbo;
      float sum = 0.f;
      int j = 0;
      for (; j + 8 <= nbo; j += 8) {
        float t8[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t8[u] = q[j + u];
#pragma unroll
        for (int u = 0; u < 8; ++u) sum += t8[u];
      }
      for (; j < nbo; ++j) sum += q[j];
      a.b_rew[slot0 + rt] = -a.reward_scale * sum;
    }
    // the new state, in fp32 for the simulator and the stores and in bf16 for the next step's nets (one pass and
    // one barrier instead of two)
    if (a.obs_vec) {            // four elements per thread (O, O + A and the padded width are multiples of 4)
      const int p4 = a.obs_pad >> 2;
      for (int idx = tid; idx < Rv * p4; idx += NT) {
        const int r = idx / p4, k = 4 * (idx - r * p4);
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k < O && r0 + r < a.n) v = *reinterpret_cast<const float4*>(s_next + r * o4 + k);
        if (k < O) *reinterpret_cast<float4*>(s_in + r * OA + k) = v;
        *reinterpret_cast<uint2*>(s_x0 + r * stride_x0 + k) = make_uint2(pack_bf16(v.x, v.y), pack_bf16(v.z, v.w));
      }
    } else {
      for (int idx = tid; idx < Rv * a.obs_pad; idx += NT) {
        const int r = idx / a.obs_pad, k = idx - r * a.obs_pad;
        const float v = (k < O && r0 + r < a.n) ? s_next[r * o4 + k] : 0.f;
        if (k < O) s_in[r * OA + k] = v;
        s_x0[r * stride_x0 + k] = (uint16_t)(pack_bf16(v, 0.f) & 0xFFFFu);
      }
    }
    __syncthreads();
  }
  // the loop ends right after the bootstrap value; s_in still holds the final state
  for (int idx = tid; idx < Rv * O; idx += NT) {
    const int r = idx / O, k = idx - r * O;
    if (r0 + r < a.n) a.obs_state[(int64_t)(r0 + r) * O + k] = s_in[r * OA + k];
  }
  if (dtid >= 0 && dtid < Rv && r0 + dtid < a.n) a.episode_step[r0 + dtid] = ep;
  __syncthreads();                                   // the next tile overwrites the state rows
  }
}

// floats of one net's LDS bias block (the two nets have the same padded widths except for the head,
// whose padded width is at least as large for the policy net)
size_t bias_floats(const gmi_model* m, int net) {
  size_t n = 0;
  for (int l = 0; l < m->L.n_layers; ++l) n += m->L.net[net][l].out_pad;
  return n;
}

void fill_net(const gmi_model* m, int net, FusedNet* N) {
  const ModelLayout& L = m->L;
  N->n_layers = L.n_layers;
  for (int l = 0; l < L.n_layers; ++l) {
    const LayerInfo& li = L.net[net][l];
    N->w[l] = reinterpret_cast<const uint16_t*>(m->shadow + li.sh_wf);
    N->bias[l] = reinterpret_cast<const float*>(m->shadow + li.sh_b);
    N->in_pad[l] = li.in_pad;
    N->out_pad[l] = li.out_pad;
    N->bias_off[l] = l ? N->bias_off[l - 1] + N->out_pad[l - 1] : 0;
  }
  N->bias_total = N->bias_off[L.n_layers - 1] + N->out_pad[L.n_layers - 1];
  N->out_store = L.net[net][L.n_layers - 1].out;
}

size_t agent_lds_bytes(const gmi_model* m, int R) {
  const ModelLayout& L = m->L;
  int max_h = 32;
  for (int l = 0; l < L.n_hidden; ++l) max_h = L.net[0][l].out_pad > max_h ? L.net[0][l].out_pad : max_h;
  const int nb = (L.act_dim + 3) / 4;
  return (size_t)R * (gmi::pad32(L.obs_dim) + 8) * 2 + 2 * (size_t)R * (max_h + 8) * 2 +
         ((size_t)R * (L.act_dim + 1 + nb) + bias_floats(m, 0) + bias_floats(m, 1)) * 4;
}

// Bytes of one step's random draws for a tile of R envs (one float4 per block).
size_t rollout_noise_bytes(const gmi_model* m, int R) {
  const int O = m->L.obs_dim, A = m->L.act_dim, o4 = (O + 3) & ~3;
  return (size_t)R * ((A + 3) / 4 + o4 / 4 + 1) * 16;
}

// Bytes of the hidden-activation space left over beside the next-state tile and the random draws while the
// simulator runs.
size_t rollout_stage_room(const gmi_model* m, int R) {
  const ModelLayout& L = m->L;
  int max_h = 32;
  for (int l = 0; l < L.n_hidden; ++l) max_h = L.net[0][l].out_pad > max_h ? L.net[0][l].out_pad : max_h;
  const int o4 = (L.obs_dim + 3) & ~3;
  const size_t hid = 4 * (size_t)R * (max_h + 8) * 2, used = (((size_t)R * o4 * 4 + 15) & ~(size_t)15) + rollout_noise_bytes(m, R);
  return hid > used ? hid - used : 0;
}

// LDS of the operand blocks that the weight-stationary form keeps there (both nets); 0 for other shapes.
size_t rollout_ws_lds_bytes(const ModelLayout& L) {
  if (ws_matches<WsAnt>(L)) return 2 * (size_t)WsAnt::lds_elems() * 2;
  if (ws_matches<WsSmallObs>(L)) return 2 * (size_t)WsSmallObs::lds_elems() * 2;
  return 0;
}

size_t rollout_lds_bytes(const gmi_model* m, int R, bool mt_lds) {
  const ModelLayout& L = m->L;
  int max_h = 32;
  for (int l = 0; l < L.n_hidden; ++l) max_h = L.net[0][l].out_pad > max_h ? L.net[0][l].out_pad : max_h;
  const int O = L.obs_dim, A = L.act_dim, o4 = (O + 3) & ~3;
  const size_t hid = 4 * (size_t)R * (max_h + 8) * 2, used = (((size_t)R * o4 * 4 + 15) & ~(size_t)15) + rollout_noise_bytes(m, R);
  const size_t region = ((hid > used ? hid : used) + 15) & ~(size_t)15;
  return (size_t)((R * (O + A) + 3) & ~3) * 4 + (size_t)R * (gmi::pad32(O) + 8) * 2 + region +
         (size_t)(R * (A + 1 + (A + 3) / 4 + o4 / 4) + ((R + 3) & ~3)) * 4 +
         ((bias_floats(m, 0) + bias_floats(m, 1) + 3) & ~(size_t)3) * 4 +
         (mt_lds ? (size_t)(O + A) * o4 * 4 : 0) + rollout_ws_lds_bytes(L);
}

}  // namespace

namespace gmi {

// Returns GMI_OK if the fused kernel was launched, GMI_ERR_UNSUPPORTED (without setting an error
// message the caller must report) if the model does not fit the fused kernel and the per-layer path
// has to be used instead.
int launch_agent_fused(gmi_instance* g, gmi_model* m, const float* obs, int n, uint64_t seed, uint32_t step,
                       uint32_t env_offset, float* act, float* logp, float* value, float* mu_out, bool do_policy) {
  if (m->L.dtype != GMI_DTYPE_BF16) return GMI_ERR_UNSUPPORTED;
  // every row tile streams all weights from L2 once: beyond ~1 MB of bf16 weights the per-layer
  // large-tile kernels are faster (measured on a
  // [512,512,256,128] model: 180 us fused against ~140 us per-layer for 16384 rows)
  if (m->L.weight_bytes > (1 << 20)) return GMI_ERR_UNSUPPORTED;
  constexpr size_t kLdsMax = 160 * 1024;
  int R = 64;
  if (agent_lds_bytes(m, R) > kLdsMax) R = 32;
  if (agent_lds_bytes(m, R) > kLdsMax) return GMI_ERR_UNSUPPORTED;
  // small batches: 32-row tiles give twice the workgroups
  if (R == 64 && (n + 63) / 64 < g->cu_count / 2) R = 32;
  AgentArgs a;
  fill_net(m, 0, &a.net[0]);
  fill_net(m, 1, &a.net[1]);
  a.log_std = reinterpret_cast<const float*>(m->shadow + m->L.sh_logstd);
  a.obs = obs;
  a.n = n;
  a.obs_dim = m->L.obs_dim;
  a.obs_pad = pad32(m->L.obs_dim);
  a.act_dim = m->L.act_dim;
  a.max_h = 32;
  for (int l = 0; l < m->L.n_hidden; ++l) a.max_h = m->L.net[0][l].out_pad > a.max_h ? m->L.net[0][l].out_pad : a.max_h;
  a.do_policy = do_policy ? 1 : 0;
  a.k0 = (uint32_t)seed; a.k1 = (uint32_t)(seed >> 32); a.step = step; a.env_offset = env_offset;
  a.act = act; a.logp = logp; a.value = value; a.mu_out = mu_out;
  const size_t lds = agent_lds_bytes(m, R);
  ProfScope ps(g, kClsFusedAgent);
  if (R == 64) {
    static bool attr64 = false;
    if (!attr64) {
      GMI_HIP(hipFuncSetAttribute((const void*)agent_fused_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax));
      attr64 = true;
    }
    ps.launch(agent_fused_kernel<2>, dim3((n + 63) / 64), dim3(256), lds, a);
  } else {
    static bool attr32 = false;
    if (!attr32) {
      GMI_HIP(hipFuncSetAttribute((const void*)agent_fused_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax));
      attr32 = true;
    }
    ps.launch(agent_fused_kernel<1>, dim3((n + 31) / 32), dim3(256), lds, a);
  }
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}

}  // namespace gmi


extern "C" int rollout_collect(gmi_t g, gmi_model_t m, gmi_env_t env, gmi_buffer_t b, float* obs, uint64_t seed,
                               uint32_t step0, uint32_t env_offset, float* last_value) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "rollout_collect: bad instance");
  if (!valid(m)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "rollout_collect: bad model");
  if (!valid(env)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "rollout_collect: bad env");
  if (!valid(b)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "rollout_collect: bad buffer");
  const ModelLayout& L = m->L;
  const gmi_env_desc& ed = env->d;
  const gmi_buffer_desc& bd = b->d;
  if (ed.obs_dim != L.obs_dim || ed.act_dim != L.act_dim || bd.obs_dim != L.obs_dim || bd.act_dim != L.act_dim)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "rollout_collect: model, env and buffer disagree on obs_dim / act_dim");
  if (ed.n_envs != bd.n_envs)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "rollout_collect: env has %d envs, buffer %d", ed.n_envs, bd.n_envs);
  if (bd.n_envs == 0 || bd.horizon == 0) return GMI_OK;
  if (!obs || !last_value) GMI_FAIL(GMI_ERR_INVALID_ARG, "rollout_collect: NULL pointer");
  if (L.dtype != GMI_DTYPE_BF16)
    GMI_FAIL(GMI_ERR_UNSUPPORTED, "rollout_collect: BF16 models only; use agent_act / env_step / collect_experience");
  // as for the fused agent kernel: every tile streams all weights from L2 at every step, which loses to the
  // per-layer large-tile kernels beyond ~1 MB of bf16 weights (measured on a [512,512,256,128] model with
  // 16384 envs and 16 steps: 4.1 ms in one launch against 3.3 ms step by step)
  if (L.weight_bytes > (1 << 20)) {
    // ... where the model has a forward-only kernel of its own, the stage is two launches per step instead
    const int rc = gmi::rollout_stepwise(g, m, env, b, obs, seed, step0, env_offset, last_value);
    if (rc != GMI_ERR_UNSUPPORTED) return rc;
  }
  if (L.weight_bytes > (1 << 20))
    GMI_FAIL(GMI_ERR_UNSUPPORTED, "rollout_collect: model too large for the one-launch kernel (%lld bytes of bf16 "
             "weights, limit %d); use agent_act / env_step / collect_experience", (long long)L.weight_bytes, 1 << 20);
  constexpr size_t kLdsMax = 160 * 1024;
  const int n = bd.n_envs;
  int R = 64;
  if (rollout_lds_bytes(m, R, false) > kLdsMax || (n + 63) / 64 < g->cu_count) R = 32;
  if (rollout_lds_bytes(m, R, false) > kLdsMax)
    GMI_FAIL(GMI_ERR_UNSUPPORTED, "rollout_collect: a 32-env tile of this model needs %zu bytes of LDS (limit %zu); "
             "use agent_act / env_step / collect_experience", rollout_lds_bytes(m, R, false), kLdsMax);
  const size_t mt_bytes = (size_t)(L.obs_dim + L.act_dim) * ((L.obs_dim + 3) & ~3) * 4;
  const bool mt_lds = rollout_lds_bytes(m, R, true) <= kLdsMax;
  const int mt_mode = mt_lds ? 2 : (rollout_stage_room(m, R) >= mt_bytes ? 1 : 0);
  RolloutArgs a;
  fill_net(m, 0, &a.net[0]);
  fill_net(m, 1, &a.net[1]);
  a.log_std = reinterpret_cast<const float*>(m->shadow + L.sh_logstd);
  a.obs_state = obs;
  a.m_t = env->m_t;
  a.episode_step = env->episode_step;
  a.n = n; a.obs_dim = L.obs_dim; a.obs_pad = gmi::pad32(L.obs_dim); a.act_dim = L.act_dim;
  a.max_h = 32;
  for (int l = 0; l < L.n_hidden; ++l) a.max_h = L.net[0][l].out_pad > a.max_h ? L.net[0][l].out_pad : a.max_h;
  a.o4 = (L.obs_dim + 3) & ~3;
  a.T = bd.horizon; a.ld_envs = bd.ld_envs;
  a.noise_std = ed.noise_std; a.reward_scale = ed.reward_scale;
  a.done_period = ed.done_period; a.done_threshold = ed.done_threshold;
  a.ak0 = (uint32_t)seed; a.ak1 = (uint32_t)(seed >> 32); a.a_env_offset = env_offset;
  a.ek0 = (uint32_t)ed.seed; a.ek1 = (uint32_t)(ed.seed >> 32); a.e_env_offset = ed.env_offset;
  a.step0 = step0;
  a.mt_lds = mt_mode;
  a.obs_vec = (L.obs_dim % 4 == 0 && (L.obs_dim + L.act_dim) % 4 == 0 && ((uintptr_t)bd.obs & 15) == 0) ? 1 : 0;
  a.b_obs = bd.obs; a.b_act = bd.act; a.b_logp = bd.logp; a.b_val = bd.val; a.b_rew = bd.rew; a.b_done = bd.done;
  a.last_value = last_value;
  size_t lds = rollout_lds_bytes(m, R, mt_lds);
  // fewer 32-env tiles than compute units: 16 envs per workgroup use twice as many of them
  const int rows_per_wg = (R == 32 && (n + 31) / 32 < g->cu_count && n > 16) ? 16 : R;
  a.rows_per_wg = rows_per_wg;
  // Draws one step ahead: when the simulator's items leave enough whole waves idle to make a step's draws in two
  // rounds at most, and two buffers of them still fit
  {
    const int nbo = a.o4 / 4, nba = (L.act_dim + 3) / 4, npr = nba + nbo + 1;
    const int sim_items = (rows_per_wg / 4) * nbo >= 192 ? (rows_per_wg / 4) * nbo : rows_per_wg * nbo;
    const int idle = 512 - ((sim_items + 63) & ~63);
    const size_t off = (lds + 15) & ~(size_t)15, need = off + 2 * (size_t)rows_per_wg * npr * 16;
    a.noise_ahead = (idle > 0 && idle * 2 >= rows_per_wg * npr && need <= kLdsMax) ? 1 : 0;
    a.ahead_off = (int)off;
    if (a.noise_ahead) lds = need;
  }
  a.n_tiles = (n + rows_per_wg - 1) / rows_per_wg;
  // weight-stationary variant where this model's padded widths have one (both nets share them)
  typedef void (*rollout_fn)(RolloutArgs);
  rollout_fn kfn = R == 64 ? rollout_fused_kernel<2> : rollout_fused_kernel<1>;
  int variant = R == 64 ? 1 : 0;
  if (ws_matches<WsAnt>(L)) { kfn = R == 64 ? rollout_fused_kernel<2, WsAnt> : rollout_fused_kernel<1, WsAnt>; variant += 2; }
  else if (ws_matches<WsSmallObs>(L)) { kfn = R == 64 ? rollout_fused_kernel<2, WsSmallObs> : rollout_fused_kernel<1, WsSmallObs>; variant += 4; }
  // 16 envs per workgroup: the weight-stationary nets on 16-row products
  if (rows_per_wg == 16 && variant == 2) { kfn = rollout_fused_kernel<1, WsAnt, true>; variant = 6; }
  else if (rows_per_wg == 16 && variant == 4) { kfn = rollout_fused_kernel<1, WsSmallObs, true>; variant = 7; }
  else if (rows_per_wg == 16 && variant == 0) { kfn = rollout_fused_kernel<1, void, true>; variant = 8; }
  static bool attr_set[9] = {false, false, false, false, false, false, false, false, false};
  if (!attr_set[variant]) {
    GMI_HIP(hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax));
    attr_set[variant] = true;
  }
  // no more workgroups than the instance's compute units hold at once; the rest of the tiles are taken
  // by the same workgroups in turn
  int per_cu = 0;
  GMI_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)kfn, 512, lds));
  if (per_cu < 1) per_cu = 1;
  const int64_t resident = (int64_t)per_cu * g->cu_count;
  const int grid = (int)(a.n_tiles < resident ? a.n_tiles : resident);
  gmi::ProfScope ps(g, gmi::kClsFusedRollout);
  ps.launch(kfn, dim3(grid), dim3(512), lds, a);
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}
