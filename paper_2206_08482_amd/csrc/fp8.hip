// Inference-only agents in 8-bit floating point (the agent role of Section 3 of the paper needs the forward pass
// alone): weights of every layer as E4M3 with one power-of-two scale per layer, the observation and the hidden
// activations as unscaled E4M3 (saturating), products on the 64-deep fp8 matrix instruction with fp32 accumulation,
// scale, bias and ELU in fp32, the heads' outputs in fp32.  The action is then drawn exactly as agent_act draws it.
//
// A workgroup of 4 waves owns 128 rows of one net (64 where the activation buffers of 128 rows would leave room for
// only one workgroup per compute unit).  Activations live in LDS as bytes [row][k] (row stride K + 16
// bytes), two buffers that swap roles from layer to layer.  Wave w computes a quarter of the feature tiles (32 features
// each) for all its 32-row tiles, so a weight block is fetched once per workgroup; weights are read straight from
// their packed array in operand order: for feature tile ft and k-step ks (64 deep), lane (f = lane % 32,
// kh = lane / 32) holds the 32 bytes k = 64 ks + 32 kh + 0..31 of feature 32 ft + f, stored as two 16-byte halves
// [block][half][lane] so that each load instruction reads 1 KiB contiguously.  Activations are read with the same
// (kh, byte) -> k rule, which is all the dot product needs: how the instruction orders k inside a lane pair does
// not matter as long as both operands use one rule.  Layer widths are padded to 64 (heads to 32) with zero weights.
//
// The fp8 matrix instructions do not add their products exactly: a product more than 2^13 times smaller than the
// largest one of the instruction is dropped (measured on the 16-deep form: 1*1 + 2^-13 is exact, 1*1 + 2^-14 gives
// 1).  Results therefore follow an exact-sum model of the same roundings to ~1e-4 per activation, not to fp32
// rounding.
#include "internal.h"

#include <vector>

struct gmi_fp8 {
  uint32_t magic;
  int device;
  ModelLayout L;
  int max_rows;
  int rows;                                // rows of a workgroup, 128 or 64
  int buf_bytes;                           // one activation buffer of the kernel
  size_t lds_bytes;                        // both buffers and the biases
  char* base;                              // everything below, one allocation
  size_t bytes;
  std::vector<int64_t> w_off[2];           // packed E4M3 weights of (net, layer), byte offsets
  std::vector<int64_t> b_off[2];           // fp32 bias [F], zero padded
  int64_t scale_off, max_off, logstd_off, mu_off;   // fp32 [2 * n_layers], u32 [2 * n_layers], fp32 [A], fp32 [max_rows, A]
};

namespace {
constexpr uint32_t kMagicFp8 = 0x474d4938;   // "GMI8"
bool valid(gmi_fp8_t w) { return w && w->magic == kMagicFp8; }
int pad64(int x) { return (x + 63) & ~63; }
constexpr int kMaxLayers = GMI_MAX_HIDDEN + 1;

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef int intx8 __attribute__((ext_vector_type(8)));
constexpr int kFp8LdsTwo = 80 * 1024;   // two workgroups of at most this much LDS fit a compute unit

struct Fp8Layer {
  const float* w;          // fp32 [out, in] of the parameter vector
  const float* b;          // fp32 [out]
  uint32_t* packed;        // E4M3 bytes in operand order, as words
  float* bias;             // fp32 [F]
  int in, out, K, F;       // K = in padded to 64; F = out padded to 64 (hidden) or 32 (head)
};
struct Fp8Table {
  Fp8Layer l[2 * kMaxLayers];
  int n;                   // layers of both nets
  uint32_t* maxbits;       // [n] bit patterns of max|w| (non-negative floats order like their bit patterns)
  float* scale;            // [n]
  const float* log_std;
  float* log_std_out;
  int act_dim;
};

__global__ void fp8_clear_kernel(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

__global__ void fp8_absmax_kernel(Fp8Table t) {
  const Fp8Layer& L = t.l[blockIdx.y];
  const int64_t n = (int64_t)L.in * L.out;
  float m = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    m = fmaxf(m, fabsf(L.w[i]));
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  if ((threadIdx.x & 63) == 0 && m > 0.f) atomicMax(t.maxbits + blockIdx.y, __float_as_uint(m));
}

// The smallest power of two s with m <= 448 s, from m's exponent and mantissa: m = f 2^e with 0.5 <= f < 1 and
// 448 = 0.875 * 2^9, so s = 2^(e - 9) if f <= 0.875, else 2^(e - 8).  1 for m = 0.
__device__ float scale_for(uint32_t maxbits) {
  if (maxbits == 0u) return 1.0f;
  int e;
  const float f = frexpf(__uint_as_float(maxbits), &e);
  return ldexpf(1.0f, f <= 0.875f ? e - 9 : e - 8);
}

__device__ __forceinline__ uint32_t to_e4m3x4(float a, float b, float c, float d) {
  // the conversion rounds to nearest even; its inputs are kept within the format's range, so it never overflows
  a = __builtin_amdgcn_fmed3f(a, -448.f, 448.f); b = __builtin_amdgcn_fmed3f(b, -448.f, 448.f);
  c = __builtin_amdgcn_fmed3f(c, -448.f, 448.f); d = __builtin_amdgcn_fmed3f(d, -448.f, 448.f);
  int v = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
  v = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, v, true);
  return (uint32_t)v;
}

// One thread per packed word (4 consecutive k of one feature); also the scales, the padded biases and log_std.
__global__ void fp8_pack_kernel(Fp8Table t) {
  const Fp8Layer& L = t.l[blockIdx.y];
  const float s = scale_for(t.maxbits[blockIdx.y]);
  const float inv = 1.0f / s;                 // a power of two: exact
  const int nks = L.K / 64;
  const int64_t words = (int64_t)L.F * L.K / 4;
  for (int64_t wd = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; wd < words; wd += (int64_t)gridDim.x * blockDim.x) {
    const int q = (int)(wd & 3);              // word within the 16-byte piece
    const int lane = (int)((wd >> 2) & 63);
    const int half = (int)((wd >> 8) & 1);
    const int64_t blk = wd >> 9;              // ft * nks + ks
    const int ks = (int)(blk % nks), ft = (int)(blk / nks);
    const int f = 32 * ft + (lane & 31);
    const int k = 64 * ks + 32 * (lane >> 5) + 16 * half + 4 * q;
    float v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = (f < L.out && k + j < L.in) ? L.w[(int64_t)f * L.in + k + j] * inv : 0.f;
    L.packed[wd] = to_e4m3x4(v[0], v[1], v[2], v[3]);
  }
  if (blockIdx.x == 0) {
    for (int i = threadIdx.x; i < L.F; i += blockDim.x) L.bias[i] = i < L.out ? L.b[i] : 0.f;
    if (threadIdx.x == 0) t.scale[blockIdx.y] = s;
    if (blockIdx.y == 0)
      for (int i = threadIdx.x; i < t.act_dim; i += blockDim.x) t.log_std_out[i] = t.log_std[i];
  }
}

struct Fp8Net {
  const uint4* packed[kMaxLayers];
  const float* bias[kMaxLayers];
  int K[kMaxLayers], F[kMaxLayers];
  int scale0;              // index of this net's first layer in the scale array
  int out;                 // act_dim or 1
  float* dst;              // mu [N, A] or value [N]
};
struct Fp8Args {
  Fp8Net net[2];
  const float* scale;
  const float* obs;
  int n_rows, obs_dim, n_layers, buf_bytes;   // buf_bytes: size of one of the two activation buffers
};


// ELU as max(z, min(e^z, 1) - 1) on the hardware exponential (the [0, 1] clamp is an output modifier): its error of
// ~1e-7 is far below the matrix instruction's own (above); expm1f measured the same parity and 2x the kernel time.
__device__ __forceinline__ float elu32(float z) {
  const float e = __builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(z * 1.44269504f), 0.f, 1.f);
  return __builtin_fmaxf(z, e - 1.0f);
}

__device__ __forceinline__ intx8 join(const uint4& a, const uint4& b) {
  intx8 r;
  r[0] = (int)a.x; r[1] = (int)a.y; r[2] = (int)a.z; r[3] = (int)a.w;
  r[4] = (int)b.x; r[5] = (int)b.y; r[6] = (int)b.z; r[7] = (int)b.w;
  return r;
}

// The observation rows of a workgroup, rounded to E4M3, zero beyond obs_dim and beyond the last row.  BATCH groups of
// four values per thread and round (8 covers observations up to 64 wide in one round, 16 up to 128; more would push the kernel past 256
// registers, and models narrow enough for two workgroups per compute unit would lose the second one), all loads of a
// round issued before the first is used; an element outside the matrix is read from a clamped (valid) address and
// replaced by zero, so that no load sits behind a branch.
template <int BATCH>
__device__ __forceinline__ void fp8_gather(const float* __restrict__ obs, int n_rows, int obs_dim, int K0, int row0,
                                           int rows, int tid, unsigned char* cur) {
  const int kg = K0 / 4, S = K0 + 16, groups = rows * kg;
  const int64_t last = (int64_t)n_rows * obs_dim - 1;
  for (int i0 = tid; i0 < groups; i0 += 256 * BATCH) {
    float v[BATCH][4];
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int i = i0 + 256 * u, r = i / kg, k = 4 * (i % kg);
      const int64_t e = (int64_t)(row0 + r) * obs_dim + k;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int64_t ej = e + j < last ? e + j : last;
        const float x = obs[ej];
        v[u][j] = (i < groups && row0 + r < n_rows && k + j < obs_dim) ? x : 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int i = i0 + 256 * u, r = i / kg, k = 4 * (i % kg);
      if (i < groups) *reinterpret_cast<uint32_t*>(cur + r * S + k) = to_e4m3x4(v[u][0], v[u][1], v[u][2], v[u][3]);
    }
  }
}

// One layer for one wave: the feature tiles [wave * per, (wave + 1) * per) for the workgroup's four 32-row tiles.
// NKS = K / 64 is a compile-time constant so that the k loop unrolls: the wave holds all NKS weight blocks of the
// tile in use and, requested when that tile starts, those of the next tile (one wave per SIMD: nothing else hides
// the latency of the loads; a whole tile's products lie between a request and its use).  Activations for k-step
// ks + 1 are read from LDS while the products of step ks run.  No load sits behind a branch: after the last tile
// its own blocks are requested again.
template <int NKS, int RT>
__device__ __forceinline__ void fp8_layer(const uint4* __restrict__ packed, const float* bias, float s,
                                          const unsigned char* cur, unsigned char* nxt, int K, int F, bool head,
                                          int wave, int lane, int row0, int n_rows, int n_out, float* __restrict__ dst) {
  const int r32 = lane & 31, kh = lane >> 5;
  const int S = K + 16, So = F + 16;
  const int nt = F / 32, per = (nt + 3) / 4;
  const int t0 = wave * per, t1 = (t0 + per < nt) ? t0 + per : nt;
  if (t0 >= t1) return;
  const unsigned char* xrow = cur + r32 * S + 32 * kh;
  uint4 wc[NKS][2], wn[NKS][2];
  {
    const uint4* p = packed + (int64_t)t0 * NKS * 128 + lane;
#pragma unroll
    for (int k = 0; k < NKS; ++k) { wc[k][0] = p[k * 128]; wc[k][1] = p[k * 128 + 64]; }
  }
  for (int ft = t0; ft < t1; ++ft) {
    {
      const int fn = ft + 1 < t1 ? ft + 1 : ft;
      const uint4* p = packed + (int64_t)fn * NKS * 128 + lane;
#pragma unroll
      for (int k = 0; k < NKS; ++k) { wn[k][0] = p[k * 128]; wn[k][1] = p[k * 128 + 64]; }
    }
    floatx16 acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rt][i] = 0.f;
    uint4 x[2][RT][2];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      x[0][rt][0] = *reinterpret_cast<const uint4*>(xrow + rt * 32 * S);
      x[0][rt][1] = *reinterpret_cast<const uint4*>(xrow + rt * 32 * S + 16);
    }
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      const intx8 wa = join(wc[ks][0], wc[ks][1]);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        if (ks + 1 < NKS) {
          x[(ks + 1) & 1][rt][0] = *reinterpret_cast<const uint4*>(xrow + rt * 32 * S + 64 * (ks + 1));
          x[(ks + 1) & 1][rt][1] = *reinterpret_cast<const uint4*>(xrow + rt * 32 * S + 64 * (ks + 1) + 16);
        }
        acc[rt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wa, join(x[ks & 1][rt][0], x[ks & 1][rt][1]), acc[rt],
                                                                   0, 0, 0, 0, 0, 0);
      }
    }
    // result register i of this lane: feature 32 ft + 8 (i / 4) + 4 kh + i % 4 of row 32 rt + r32
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int f0 = 32 * ft + 8 * q + 4 * kh;
      const float4 b = *reinterpret_cast<const float4*>(bias + f0);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const int r = 32 * rt + r32;
        const float z0 = fmaf(acc[rt][4 * q + 0], s, b.x), z1 = fmaf(acc[rt][4 * q + 1], s, b.y);
        const float z2 = fmaf(acc[rt][4 * q + 2], s, b.z), z3 = fmaf(acc[rt][4 * q + 3], s, b.w);
        if (!head) {
          *reinterpret_cast<uint32_t*>(nxt + r * So + f0) = to_e4m3x4(elu32(z0), elu32(z1), elu32(z2), elu32(z3));
        } else if (row0 + r < n_rows) {
          const float z[4] = {z0, z1, z2, z3};
#pragma unroll
          for (int jj = 0; jj < 4; ++jj)
            if (f0 + jj < n_out) dst[(int64_t)(row0 + r) * n_out + f0 + jj] = z[jj];
        }
      }
    }
#pragma unroll
    for (int k = 0; k < NKS; ++k) { wc[k][0] = wn[k][0]; wc[k][1] = wn[k][1]; }
  }
}

template <int ROWS>
__global__ __launch_bounds__(256) void agent_fp8_kernel(Fp8Args a) {
  extern __shared__ __align__(16) unsigned char lds[];
  const Fp8Net& N = a.net[blockIdx.y];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int row0 = blockIdx.x * ROWS;
  unsigned char* cur = lds;
  unsigned char* nxt = lds + a.buf_bytes;
  // the biases of all layers, one after the other, behind the two activation buffers (the layer loop reads them from
  // LDS: a global load in its epilogue would make the wait for it drain the weight requests in flight)
  float* bias_all = reinterpret_cast<float*>(lds + 2 * a.buf_bytes);
  {
    int off = 0;
    for (int l = 0; l < a.n_layers; ++l) {
      for (int i = tid; i < N.F[l]; i += 256) bias_all[off + i] = N.bias[l][i];
      off += N.F[l];
    }
  }
  const float* bias = bias_all;
  if (ROWS * (N.K[0] / 4) <= 256 * 8) fp8_gather<8>(a.obs, a.n_rows, a.obs_dim, N.K[0], row0, ROWS, tid, cur);
  else fp8_gather<16>(a.obs, a.n_rows, a.obs_dim, N.K[0], row0, ROWS, tid, cur);
  __syncthreads();
  for (int l = 0; l < a.n_layers; ++l) {
    const int K = N.K[l], F = N.F[l], nks = K / 64;
    const bool head = l == a.n_layers - 1;
    const float s = a.scale[N.scale0 + l];
    switch (nks) {
      case 1: fp8_layer<1, ROWS / 32>(N.packed[l], bias, s, cur, nxt, K, F, head, wave, lane, row0, a.n_rows, N.out, N.dst); break;
      case 2: fp8_layer<2, ROWS / 32>(N.packed[l], bias, s, cur, nxt, K, F, head, wave, lane, row0, a.n_rows, N.out, N.dst); break;
      case 3: fp8_layer<3, ROWS / 32>(N.packed[l], bias, s, cur, nxt, K, F, head, wave, lane, row0, a.n_rows, N.out, N.dst); break;
      case 4: fp8_layer<4, ROWS / 32>(N.packed[l], bias, s, cur, nxt, K, F, head, wave, lane, row0, a.n_rows, N.out, N.dst); break;
      case 5: fp8_layer<5, ROWS / 32>(N.packed[l], bias, s, cur, nxt, K, F, head, wave, lane, row0, a.n_rows, N.out, N.dst); break;
      case 6: fp8_layer<6, ROWS / 32>(N.packed[l], bias, s, cur, nxt, K, F, head, wave, lane, row0, a.n_rows, N.out, N.dst); break;
      case 7: fp8_layer<7, ROWS / 32>(N.packed[l], bias, s, cur, nxt, K, F, head, wave, lane, row0, a.n_rows, N.out, N.dst); break;
      default: fp8_layer<8, ROWS / 32>(N.packed[l], bias, s, cur, nxt, K, F, head, wave, lane, row0, a.n_rows, N.out, N.dst); break;
    }
    bias += F;
    __syncthreads();
    unsigned char* t = cur; cur = nxt; nxt = t;
  }
}

int table_of(gmi_fp8* w, const float* params, Fp8Table* t) {
  const ModelLayout& L = w->L;
  t->n = 2 * L.n_layers;
  for (int net = 0; net < 2; ++net)
    for (int l = 0; l < L.n_layers; ++l) {
      const LayerInfo& li = L.net[net][l];
      Fp8Layer& o = t->l[net * L.n_layers + l];
      o.w = params + li.w_off;
      o.b = params + li.b_off;
      o.packed = reinterpret_cast<uint32_t*>(w->base + w->w_off[net][l]);
      o.bias = reinterpret_cast<float*>(w->base + w->b_off[net][l]);
      o.in = li.in; o.out = li.out; o.K = pad64(li.in); o.F = li.head ? li.out_pad : pad64(li.out);
    }
  t->maxbits = reinterpret_cast<uint32_t*>(w->base + w->max_off);
  t->scale = reinterpret_cast<float*>(w->base + w->scale_off);
  t->log_std = params + L.logstd_off;
  t->log_std_out = reinterpret_cast<float*>(w->base + w->logstd_off);
  t->act_dim = L.act_dim;
  return GMI_OK;
}

}  // namespace

extern "C" int gmi_fp8_bind(gmi_t g, const gmi_model_desc* d, gmi_fp8_t* out) {
  if (!out) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_fp8_bind: out is NULL");
  *out = nullptr;
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_fp8_bind: bad instance");
  if (!d) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_fp8_bind: desc is NULL");
  if (d->max_rows < 1) GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_fp8_bind: max_rows < 1");
  gmi_fp8* w = new gmi_fp8();
  gmi_model_desc dd = *d;
  dd.dtype = GMI_DTYPE_BF16;      // the layout's padded sizes (multiples of 32) are those of the matrix-core paths
  const int rc = build_layout(&dd, &w->L);
  if (rc != GMI_OK) { delete w; return rc; }
  size_t bias_bytes = 0;      // the kernel also keeps one net's biases in LDS (the policy net's are never fewer)
  for (const LayerInfo& li : w->L.net[0]) bias_bytes += (size_t)(li.head ? li.out_pad : pad64(li.out)) * 4;
  // 128 rows per workgroup where two such workgroups fit a compute unit's LDS, else 64 rows: the second workgroup
  // (its phases interleave with the first one's) is worth more than fetching each weight block half as often
  const int row_bytes = pad64(w->L.max_width_pad) + 16;
  w->rows = (size_t)2 * 128 * row_bytes + bias_bytes <= kFp8LdsTwo ? 128 : 64;
  w->buf_bytes = w->rows * row_bytes;
  w->lds_bytes = (size_t)2 * w->buf_bytes + bias_bytes;
  if (w->lds_bytes > 160 * 1024 || pad64(w->L.max_width_pad) > 512) {
    delete w;
    GMI_FAIL(GMI_ERR_UNSUPPORTED, "gmi_fp8_bind: the activation buffers of layers this wide (%d) do not fit in LDS",
             w->L.max_width_pad);
  }
  w->device = g->device;
  w->max_rows = d->max_rows;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off += (bytes + 255) & ~(size_t)255; return (int64_t)o; };
  for (int net = 0; net < 2; ++net)
    for (int l = 0; l < w->L.n_layers; ++l) {
      const LayerInfo& li = w->L.net[net][l];
      const int K = pad64(li.in), F = li.head ? li.out_pad : pad64(li.out);
      w->w_off[net].push_back(take((size_t)F * K));
      w->b_off[net].push_back(take((size_t)F * 4));
    }
  w->scale_off = take(2 * kMaxLayers * 4);
  w->max_off = take(2 * kMaxLayers * 4);
  w->logstd_off = take((size_t)w->L.act_dim * 4);
  w->mu_off = take((size_t)d->max_rows * w->L.act_dim * 4);
  w->bytes = off;
  hipError_t e = hipMalloc((void**)&w->base, w->bytes);
  if (e != hipSuccess) {
    delete w;
    GMI_FAIL(GMI_ERR_HIP, "gmi_fp8_bind: hipMalloc(%zu) failed: %s", off, hipGetErrorString(e));
  }
  w->magic = kMagicFp8;
  *out = w;
  return GMI_OK;
}

extern "C" int gmi_fp8_destroy(gmi_fp8_t w) {
  if (!valid(w)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_fp8_destroy: bad handle");
  (void)hipFree(w->base);
  w->magic = 0;
  delete w;
  return GMI_OK;
}

extern "C" int gmi_fp8_refresh(gmi_t g, gmi_fp8_t w, const float* params) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_fp8_refresh: bad instance");
  if (!valid(w)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_fp8_refresh: bad weights");
  if (!params) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_fp8_refresh: params is NULL");
  if (g->device != w->device) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_fp8_refresh: instance and weights live on different devices");
  Fp8Table t;
  table_of(w, params, &t);
  fp8_clear_kernel<<<1, 64, 0, g->stream>>>(t.maxbits, t.n);
  fp8_absmax_kernel<<<dim3(32, (unsigned)t.n), 256, 0, g->stream>>>(t);
  fp8_pack_kernel<<<dim3(64, (unsigned)t.n), 256, 0, g->stream>>>(t);
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}

extern "C" int agent_act_fp8(gmi_t g, gmi_fp8_t w, const float* obs, int32_t n_rows, uint64_t seed, uint32_t step,
                             uint32_t env_offset, float* act, float* logp, float* value, float* mu) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "agent_act_fp8: bad instance");
  if (!valid(w)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "agent_act_fp8: bad weights");
  if (n_rows < 0 || n_rows > w->max_rows)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "agent_act_fp8: n_rows=%d outside 0..max_rows=%d", n_rows, w->max_rows);
  if (n_rows == 0) return GMI_OK;
  if (!obs || !act || !logp || !value) GMI_FAIL(GMI_ERR_INVALID_ARG, "agent_act_fp8: NULL pointer");
  if (g->device != w->device) GMI_FAIL(GMI_ERR_INVALID_ARG, "agent_act_fp8: instance and weights live on different devices");
  const ModelLayout& L = w->L;
  Fp8Args a;
  float* mu_ws = reinterpret_cast<float*>(w->base + w->mu_off);
  for (int net = 0; net < 2; ++net) {
    for (int l = 0; l < L.n_layers; ++l) {
      a.net[net].packed[l] = reinterpret_cast<const uint4*>(w->base + w->w_off[net][l]);
      a.net[net].bias[l] = reinterpret_cast<const float*>(w->base + w->b_off[net][l]);
      a.net[net].K[l] = pad64(L.net[net][l].in);
      a.net[net].F[l] = L.net[net][l].head ? L.net[net][l].out_pad : pad64(L.net[net][l].out);
    }
    a.net[net].scale0 = net * L.n_layers;
    a.net[net].out = net == 0 ? L.act_dim : 1;
    a.net[net].dst = net == 0 ? mu_ws : value;
  }
  a.scale = reinterpret_cast<const float*>(w->base + w->scale_off);
  a.obs = obs;
  a.n_rows = n_rows; a.obs_dim = L.obs_dim; a.n_layers = L.n_layers;
  a.buf_bytes = w->buf_bytes;
  const size_t lds = w->lds_bytes;
  static const hipError_t lds_ok[2] = {
      hipFuncSetAttribute(reinterpret_cast<const void*>(agent_fp8_kernel<128>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024),
      hipFuncSetAttribute(reinterpret_cast<const void*>(agent_fp8_kernel<64>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)};
  GMI_HIP(lds_ok[0]);
  GMI_HIP(lds_ok[1]);
  {
    gmi::ProfScope ps(g, gmi::kClsFusedAgent);
    const dim3 grid((unsigned)((n_rows + w->rows - 1) / w->rows), 2);
    if (w->rows == 128) ps.launch(agent_fp8_kernel<128>, grid, dim3(256), lds, a);
    else ps.launch(agent_fp8_kernel<64>, grid, dim3(256), lds, a);
  }
  GMI_LAUNCH_CHECK();
  const float* log_std = reinterpret_cast<const float*>(w->base + w->logstd_off);
  return gmi::launch_sample(g, mu_ws, log_std, n_rows, L.act_dim, seed, step, env_offset, act, logp, mu);
}
