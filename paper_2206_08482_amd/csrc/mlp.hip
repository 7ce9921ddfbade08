// Linear layers of the policy / value MLPs: forward, input-gradient and weight-gradient products.
//
// BF16 path: v_mfma_f32_32x32x16_bf16 (bf16 operands, fp32 accumulate).  A wavefront of 64 lanes
// feeds the matrix core with 8 consecutive contraction elements per lane for both operands, so both
// operands are staged in LDS with the contraction index contiguous; the weight-gradient product
// contracts over samples, whose index is strided in memory, and transposes 8x8 blocks in registers
// while staging.  F32 path: plain FMA loops (used for small fp32 configurations only).
#include "internal.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int kBK = 64;          // contraction elements staged per step
constexpr int kLds = kBK + 8;    // LDS row stride in bf16 elements (144 B: conflict-free 16 B reads)

typedef float float2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));

// ELU through the hardware base-2 exponential (abs. error ~1e-7, far below bf16 resolution)
__device__ __forceinline__ float elu_f(float z) {
  // The [0, 1] clamp (an output modifier of the exponential, no instruction of its own) makes the exponential term
  // 0 for z > 0, so that one maximum replaces the compare and select; for z <= 0, e^z - 1 >= z, and where rounding
  // puts the computed difference below z (|z| < 1e-7) z is the closer value anyway.
  const float e = __builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(z * 1.44269504f), 0.f, 1.f);
  return __builtin_fmaxf(z, e - 1.0f);
}
// ELU'(z) from the stored output h = ELU(z) >= -1: 1 if h > 0 else h + 1, as one add with the [0, 1] clamp
__device__ __forceinline__ float elu_grad_f(float h) { return __builtin_amdgcn_fmed3f(h + 1.0f, 0.f, 1.f); }
__device__ __forceinline__ float bf16_to_f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
// two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  float2v v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2v));
}

// ------------------------------------------------------------------------------------------------
// y[r, f] = epi(sum_k x[r,k] w[f,k]).  Matrix-core rows = features (weights), columns = samples, so a
// lane ends up with 4 consecutive features of one sample per accumulator quad.
// Workgroup = 4 waves arranged WF x WR; a wave computes TFM x TRM tiles of 32 x 32.
template <int WF, int WR, int TFM, int TRM, int EPI>
__global__ __launch_bounds__(256) void linear_bf16_kernel(gmi::LinearBatch batch, int rows) {
  constexpr int TF = WF * TFM * 32, TR = WR * TRM * 32;
  constexpr int CH_W = TF * (kBK / 8), CH_X = TR * (kBK / 8);      // 16-byte chunks per stage
  constexpr int NCH = (CH_W + CH_X + 255) / 256;
  __shared__ __attribute__((aligned(16))) uint16_t s_w[TF * kLds];
  __shared__ __attribute__((aligned(16))) uint16_t s_x[TR * kLds];

  const gmi::LinearProblem& P = batch.p[blockIdx.z];
  const int f0 = blockIdx.y * TF;
  if (f0 >= P.F) return;
  const int r0 = blockIdx.x * TR;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wf = wave / WR, wr = wave % WR;
  const uint16_t* __restrict__ gw = (const uint16_t*)P.w;
  const uint16_t* __restrict__ gx = (const uint16_t*)P.x;

  floatx16 acc[TFM][TRM];
#pragma unroll
  for (int i = 0; i < TFM; ++i)
#pragma unroll
    for (int j = 0; j < TRM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  uint4 stage[NCH];
  auto load_stage = [&](int k0) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int ch = tid + c * 256;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ch < CH_W) {
        const int row = ch >> 3, kc = ch & 7;
        const int f = f0 + row, k = k0 + kc * 8;
        if (f < P.F && k < P.K) v = *reinterpret_cast<const uint4*>(gw + (int64_t)f * P.ldw + k);
      } else if (ch < CH_W + CH_X) {
        const int c2 = ch - CH_W;
        const int row = c2 >> 3, kc = c2 & 7;
        const int r = r0 + row, k = k0 + kc * 8;
        if (r < rows && k < P.K) v = *reinterpret_cast<const uint4*>(gx + (int64_t)r * P.ldx + k);
      }
      stage[c] = v;
    }
  };
  auto store_stage = [&]() {
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int ch = tid + c * 256;
      if (ch < CH_W) {
        const int row = ch >> 3, kc = ch & 7;
        *reinterpret_cast<uint4*>(&s_w[row * kLds + kc * 8]) = stage[c];
      } else if (ch < CH_W + CH_X) {
        const int c2 = ch - CH_W;
        const int row = c2 >> 3, kc = c2 & 7;
        *reinterpret_cast<uint4*>(&s_x[row * kLds + kc * 8]) = stage[c];
      }
    }
  };

  const int nk = (P.K + kBK - 1) / kBK;
  load_stage(0);
  for (int kt = 0; kt < nk; ++kt) {
    store_stage();
    __syncthreads();
    if (kt + 1 < nk) load_stage((kt + 1) * kBK);
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      bf16x8 a[TFM], b[TRM];
      const int ko = kk * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < TFM; ++i)
        a[i] = *reinterpret_cast<const bf16x8*>(&s_w[((wf * TFM + i) * 32 + (lane & 31)) * kLds + ko]);
#pragma unroll
      for (int j = 0; j < TRM; ++j)
        b[j] = *reinterpret_cast<const bf16x8*>(&s_x[((wr * TRM + j) * 32 + (lane & 31)) * kLds + ko]);
#pragma unroll
      for (int i = 0; i < TFM; ++i)
#pragma unroll
        for (int j = 0; j < TRM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // epilogue: accumulator v of lane l holds feature 8*(v/4) + 4*(l/32) + v%4, sample l%32 of the tile
#pragma unroll
  for (int i = 0; i < TFM; ++i) {
    const int fb = f0 + (wf * TFM + i) * 32;
    if (fb >= P.F) continue;
#pragma unroll
    for (int j = 0; j < TRM; ++j) {
      const int r = r0 + (wr * TRM + j) * 32 + (lane & 31);
      if (r >= rows) continue;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int f = fb + q * 8 + (lane >> 5) * 4;
        float o[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = acc[i][j][q * 4 + t];
        if (EPI == gmi::kEpiBiasElu) {
          const float4 bv = *reinterpret_cast<const float4*>(P.bias + f);
          o[0] = elu_f(o[0] + bv.x); o[1] = elu_f(o[1] + bv.y);
          o[2] = elu_f(o[2] + bv.z); o[3] = elu_f(o[3] + bv.w);
          uint2 pk = make_uint2(pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3]));
          *reinterpret_cast<uint2*>((uint16_t*)P.y + (int64_t)r * P.ldy + f) = pk;
        } else if (EPI == gmi::kEpiBiasHead) {
          float* y = (float*)P.y + (int64_t)r * P.ldy;
#pragma unroll
          for (int t = 0; t < 4; ++t)
            if (f + t < P.F_store) y[f + t] = o[t] + P.bias[f + t];
        } else {
          const uint2 hv = *reinterpret_cast<const uint2*>((const uint16_t*)P.h + (int64_t)r * P.ldh + f);
          const float h0 = bf16_to_f((uint16_t)(hv.x & 0xFFFF)), h1 = bf16_to_f((uint16_t)(hv.x >> 16));
          const float h2 = bf16_to_f((uint16_t)(hv.y & 0xFFFF)), h3 = bf16_to_f((uint16_t)(hv.y >> 16));
          o[0] *= elu_grad_f(h0); o[1] *= elu_grad_f(h1);
          o[2] *= elu_grad_f(h2); o[3] *= elu_grad_f(h3);
          uint2 pk = make_uint2(pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3]));
          *reinterpret_cast<uint2*>((uint16_t*)P.y + (int64_t)r * P.ldy + f) = pk;
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Large-tile variant for wide layers: workgroup tile (WRN*TRW*32 rows) x (2*TFW*32 features), 2 x WRN
// waves, each wave TFW x TRW matrix-core tiles, so one 16-byte LDS fragment feeds TRW (or TFW) MFMAs and
// LDS bandwidth stays below the matrix cores' appetite.  The launcher uses 2 x 4 waves of 4 x 2 (or 2 x 2)
// tiles: two waves per SIMD cover each other's LDS and epilogue latencies, which measured 8-17 % faster
// than 2 x 2 waves of 4 x 4 tiles on the same 256 x 256 workgroup tile (the epilogue alone - ELU on 256
// values per lane - took a third of a workgroup's time with one wave per SIMD).
// K is staged 64 at a time (a full 128-byte line per
// row) into double-buffered LDS (144-byte row stride: conflict-free 16-byte reads), one barrier per
// stage.  Two further stages are in flight in registers: the row operand is first-touch data from
// HBM / the memory-side cache, and with one workgroup per CU only a deep prefetch covers that latency
// (measured: with a single stage in flight the kernel ran at the pace of one memory round trip per stage).
// The accumulators leave through LDS so that the epilogue runs and stores with features contiguous across
// lanes (whole 64..256-byte row segments per store).  Workgroup ids are decoded so that the workgroups
// sharing a row tile run back to back on the same accelerator die (ids are dealt round-robin over the 8
// dies), which keeps that tile in the die's L2.
template <int TFW, int TRW, int EPI, int WRN>
__global__ __launch_bounds__(128 * WRN) void linear_bf16_big_kernel(gmi::LinearBatch batch, int rows, int n_rt,
                                                                    int n_rt_pad, int n_ft) {
  constexpr int NT = 128 * WRN;                                  // 2 x WRN waves
  constexpr int TF = 2 * TFW * 32, TR = WRN * TRW * 32;
  constexpr int CH_W = TF * (kBK / 8), CH_X = TR * (kBK / 8);
  constexpr int NCH = (CH_W + CH_X) / NT;
  constexpr int RPP = NT / 8;                                    // rows staged per pass of the workgroup
  static_assert((CH_W + CH_X) % NT == 0 && CH_W % NT == 0, "stage must divide evenly over the threads");
  constexpr int kStageElems = (TF + TR) * kLds;                  // bf16 elements of one LDS stage
  constexpr int kOutStride = TFW * 32 + 4;                       // floats per staged output row
  constexpr int kMainBytes = 2 * kStageElems * 2;
  constexpr int kOutBytes = 2 * WRN * 32 * kOutStride * 4;
  constexpr int kSmemBytes = kMainBytes > kOutBytes ? kMainBytes : kOutBytes;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kSmemBytes];
  uint16_t* s_stage = reinterpret_cast<uint16_t*>(smem);

  // workgroup id -> (net, feature tile, row tile)
  const int per_net = n_rt_pad * n_ft;
  const int z = blockIdx.x / per_net;
  const int w = blockIdx.x % per_net;
  const int die = w & 7, slot = w >> 3;
  const int ft = slot % n_ft;
  const int rt = (slot / n_ft) * 8 + die;
  if (rt >= n_rt) return;
  const gmi::LinearProblem& P = batch.p[z];
  const int f0 = ft * TF, r0 = rt * TR;
  if (f0 >= P.F) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wf = wave / WRN, wr = wave % WRN;
  const uint16_t* __restrict__ gw = (const uint16_t*)P.w;
  const uint16_t* __restrict__ gx = (const uint16_t*)P.x;

  floatx16 acc[TFW][TRW];
#pragma unroll
  for (int i = 0; i < TFW; ++i)
#pragma unroll
    for (int j = 0; j < TRW; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // chunk = 8 consecutive k of one row; thread t handles rows (t >> 3) + 32 c, k-chunk t & 7.
  // Loads are unconditional (no branches, so the compiler can keep two stages in flight and wait only for
  // the older one): row indices are clamped into the operand (rows past the end only feed outputs that
  // are never stored) and the k offset is clamped into the row, with a select to zero past K.
  constexpr int NCW = CH_W / NT, NCX = CH_X / NT;
  const int crow = tid >> 3, kc8 = (tid & 7) * 8;
  const uint16_t* src_w[NCW];
  const uint16_t* src_x[NCX];
#pragma unroll
  for (int c = 0; c < NCW; ++c) src_w[c] = gw + (int64_t)min(f0 + crow + RPP * c, P.F - 1) * P.ldw;
#pragma unroll
  for (int c = 0; c < NCX; ++c) src_x[c] = gx + (int64_t)min(r0 + crow + RPP * c, rows - 1) * P.ldx;
  const int dst0 = crow * kLds + kc8;
  const int k_last = P.K - 8;
  uint4 st0[NCH], st1[NCH];
  auto load_stage = [&](uint4* st, int k0) {
    const int k = k0 + kc8;
    const bool k_ok = k < P.K;
    const int kq = min(k, k_last);
#pragma unroll
    for (int c = 0; c < NCW; ++c) {
      const uint4 v = *reinterpret_cast<const uint4*>(src_w[c] + kq);
      st[c] = k_ok ? v : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int c = 0; c < NCX; ++c) st[NCW + c] = *reinterpret_cast<const uint4*>(src_x[c] + kq);
  };
  auto store_stage = [&](const uint4* st, int buf) {
    uint16_t* base = s_stage + buf * kStageElems + dst0;
#pragma unroll
    for (int c = 0; c < NCW; ++c) *reinterpret_cast<uint4*>(base + c * RPP * kLds) = st[c];
#pragma unroll
    for (int c = 0; c < NCX; ++c) *reinterpret_cast<uint4*>(base + (TF + c * RPP) * kLds) = st[NCW + c];
  };
  auto compute = [&](int buf) {
    const uint16_t* sw = s_stage + buf * kStageElems;
    const uint16_t* sx = sw + TF * kLds;
#pragma unroll 2
    for (int kk = 0; kk < kBK / 16; ++kk) {
      bf16x8 a[TFW], b[TRW];
      const int ko = kk * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < TFW; ++i)
        a[i] = *reinterpret_cast<const bf16x8*>(&sw[((wf * TFW + i) * 32 + (lane & 31)) * kLds + ko]);
#pragma unroll
      for (int j = 0; j < TRW; ++j)
        b[j] = *reinterpret_cast<const bf16x8*>(&sx[((wr * TRW + j) * 32 + (lane & 31)) * kLds + ko]);
#pragma unroll
      for (int i = 0; i < TFW; ++i)
#pragma unroll
        for (int j = 0; j < TRW; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };

  // stage s lives in LDS buffer s & 1; st1 carries odd stages, st0 even stages.  Stages past K load as
  // zeros (weight operand), so the loop body needs no conditions: a trailing odd stage multiplies by zero.
  const int nk = (P.K + kBK - 1) / kBK;
  load_stage(st0, 0);
  load_stage(st1, kBK);
  store_stage(st0, 0);
  load_stage(st0, 2 * kBK);
  for (int kt = 0; kt < nk; kt += 2) {
    __syncthreads();
    store_stage(st1, 1);
    load_stage(st1, (kt + 3) * kBK);
    compute(0);
    __syncthreads();
    store_stage(st0, 0);
    load_stage(st0, (kt + 4) * kBK);
    compute(1);
  }
  __syncthreads();   // every wave is done reading the stages: LDS becomes the output staging area

  // Each wave owns a [32 rows][TFW*32 features] fp32 staging region and drains one row tile at a time.
  // Everything below is branch-free up to the final predicated store, and the problem's fields live in
  // registers: a conditional block per row made the compiler wait for every earlier store to be
  // acknowledged before each LDS read, which serialised the whole epilogue on memory round trips.
  float* s_out = reinterpret_cast<float*>(smem) + wave * 32 * kOutStride;
  constexpr int kLanesPerRow = TFW * 8;             // lanes covering one row with 4 features each
  constexpr int kRowsPerIter = 64 / kLanesPerRow;
  constexpr int NIT = 32 / kRowsPerIter;
  const int fl = (lane % kLanesPerRow) * 4;         // feature offset inside the wave's feature range
  const int f = f0 + wf * TFW * 32 + fl;
  const bool f_ok = f < P.F;
  const int fq = f_ok ? f : 0;
  uint16_t* __restrict__ yp = (uint16_t*)P.y + fq;
  const uint16_t* __restrict__ hp = (const uint16_t*)P.h + fq;
  const int ldy = P.ldy, ldh = P.ldh;
  float4 bias4 = make_float4(0.f, 0.f, 0.f, 0.f);
  if (EPI == gmi::kEpiBiasElu) bias4 = *reinterpret_cast<const float4*>(P.bias + fq);
  const int rl0 = lane / kLanesPerRow;
#pragma unroll
  for (int j = 0; j < TRW; ++j) {
    const int rbase = r0 + (wr * TRW + j) * 32 + rl0;
    uint2 hv[NIT];
    if (EPI == gmi::kEpiEluGrad) {
#pragma unroll
      for (int it = 0; it < NIT; ++it)
        hv[it] = *reinterpret_cast<const uint2*>(hp + (int64_t)min(rbase + it * kRowsPerIter, rows - 1) * ldh);
    }
#pragma unroll
    for (int i = 0; i < TFW; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 v4 = make_float4(acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]);
        *reinterpret_cast<float4*>(&s_out[(lane & 31) * kOutStride + i * 32 + q * 8 + (lane >> 5) * 4]) = v4;
      }
    __builtin_amdgcn_wave_barrier();     // wave-private region: LDS serves one wave's requests in order
    float4 o[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it)
      o[it] = *reinterpret_cast<const float4*>(&s_out[(it * kRowsPerIter + rl0) * kOutStride + fl]);
    __builtin_amdgcn_wave_barrier();
    // Make every pending global load (bias, h rows) land here, once per pass: otherwise each predicated
    // store block below starts with a wait for *all* outstanding memory operations, earlier stores included.
    if (EPI == gmi::kEpiBiasElu) {
      asm volatile("" : "+v"(bias4.x), "+v"(bias4.y), "+v"(bias4.z), "+v"(bias4.w));
    } else {
#pragma unroll
      for (int it = 0; it < NIT; ++it) asm volatile("" : "+v"(hv[it].x), "+v"(hv[it].y));
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      float4 v = o[it];
      if (EPI == gmi::kEpiBiasElu) {
        v.x = elu_f(v.x + bias4.x); v.y = elu_f(v.y + bias4.y); v.z = elu_f(v.z + bias4.z); v.w = elu_f(v.w + bias4.w);
      } else {
        const float h0 = bf16_to_f((uint16_t)(hv[it].x & 0xFFFF)), h1 = bf16_to_f((uint16_t)(hv[it].x >> 16));
        const float h2 = bf16_to_f((uint16_t)(hv[it].y & 0xFFFF)), h3 = bf16_to_f((uint16_t)(hv[it].y >> 16));
        v.x *= elu_grad_f(h0); v.y *= elu_grad_f(h1);
        v.z *= elu_grad_f(h2); v.w *= elu_grad_f(h3);
      }
      const uint2 pk = make_uint2(pack_bf16(v.x, v.y), pack_bf16(v.z, v.w));
      const int r = rbase + it * kRowsPerIter;
      if (r < rows && f_ok) *reinterpret_cast<uint2*>(yp + (int64_t)r * ldy) = pk;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Weight gradient: D[o, i] = sum_r dz[r, o] x[r, i].  Tile 128 (o) x 128 (i), 2 x 2 waves of 2 x 2
// matrix-core tiles; the contraction runs over the rows of one split, 64 rows per stage.  Each thread
// stages one 8 (rows) x 8 (features) block per step and transposes it in registers so that LDS holds
// [feature][row] with rows contiguous.
__device__ __forceinline__ void transpose8x8(const uint4 in[8], uint4 out[8]) {
  // in[j] = 8 bf16 of row j (features 0..7); out[i] = 8 bf16 of feature i (rows 0..7).
  // One byte-permute per output dword: low halves (even feature) or high halves (odd feature) of the
  // same dword of two consecutive rows.
  const uint32_t* s = reinterpret_cast<const uint32_t*>(in);
  uint32_t* d = reinterpret_cast<uint32_t*>(out);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const uint32_t a = s[(2 * p) * 4 + (i >> 1)];       // row 2p,   features (i&~1), (i|1)
      const uint32_t b = s[(2 * p + 1) * 4 + (i >> 1)];   // row 2p+1
      // v_perm_b32(S0 = b, S1 = a): selector bytes index {S1: 0..3, S0: 4..7}
      d[i * 4 + p] = __builtin_amdgcn_perm(b, a, (i & 1) ? 0x07060302u : 0x05040100u);
    }
  }
}

// LAYOUT: 0 both operands row-major, 1 both in the block layout.  A compile-time constant: a run-time branch around
// the staging loads makes the compiler wait for every load in flight where it should wait for the older of two
// stages (measured: 1.8x the kernel's time).
constexpr int kWgradT = 128;
constexpr int kWgradBuf = 2 * kWgradT * kLds;                        // one LDS stage: [o][row] then [i][row]
template <int LAYOUT>
__device__ __forceinline__ void wgrad_tile(const gmi::WgradProblem& P, int local, int rows, int n_split, int chunk,
                                           float* __restrict__ part, int64_t part_stride, uint16_t* s_stage) {
  constexpr int T = kWgradT;
  constexpr int kBuf = kWgradBuf;
  const int sp = local % n_split;
  const int tile = local / n_split;
  const int n_ti = (P.in_pad + T - 1) / T;
  const int o0 = (tile / n_ti) * T, i0 = (tile % n_ti) * T;
  const int row_begin = sp * chunk;
  const int row_end = min(rows, row_begin + chunk);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wo = wave >> 1, wi = wave & 1;
  const bool is_b = tid >= 128;
  const int t2 = tid & 127;
  const int ld = is_b ? P.ldx : P.lddz;
  const int fmax = is_b ? P.in_pad : P.out_pad;
  const int f0 = is_b ? i0 : o0;                      // first feature of the operand's 128-wide slice
  constexpr bool blocks = LAYOUT == 1;
  const bool natural = blocks && (is_b ? P.x_blocks : P.dz_blocks) == 2;      // k order inside a block's 16-wide step
  const uint16_t* __restrict__ opnd = is_b ? (const uint16_t*)P.x : (const uint16_t*)P.dz;
  // A thread stages 8 rows x 8 features per step: the rows rblk + 8 jj + 32 rt (jj = 0..3, rt = 0, 1) of the stage's
  // 64 -- which 8 rows share a 16-byte piece of LDS does not matter to a sum over rows, as long as both operands
  // agree.  Row-major operand: 16 feature blocks x 8 row blocks, the thread's features are feat .. feat + 7 and it
  // reads 16 bytes of each of its rows.  Block layout (internal.h): 8 feature steps x 2 halves x 8 row blocks; the
  // thread's features are 16 ks + 4 h + {0..3} and 16 ks + 8 + 4 h + {0..3}, row j is slot rblk + 8 (j % 4) of row
  // tile j / 4 of the stage.
  int fblk, rblk, feat;
  int ksl = 0, hb = 0;
  if (blocks) {
    rblk = t2 & 7; hb = (t2 >> 3) & 1; ksl = t2 >> 4;  // 8 consecutive lanes read 128 consecutive bytes of a block
    fblk = 2 * ksl;
    feat = f0 + 16 * ksl;
  } else {
    fblk = t2 & 15; rblk = t2 >> 4;
    feat = f0 + fblk * 8;
  }
  const bool feat_ok = feat < fmax;
  // loads are unconditional (clamped addresses, masked to zero afterwards) so that two stages stay in
  // flight and the compiler waits only for the older one
  const uint16_t* __restrict__ src = opnd + (feat_ok ? feat : 0);
  // LDS holds [feature][row]; the 16-byte slot of row block rblk inside a feature's line is XOR-swizzled
  // with the feature block index: the 16 lanes that write the same row block of 16 different feature
  // blocks are 8 LDS lines apart, which without the swizzle is the same bank group for all of them
  // (measured: 16-way conflicts made every stage cost ~4000 cycles whatever the tile's work).
  // Feature i of the thread's 8 sits at local feature fl(i); its slot is swizzled with fl(i) / 8.
  const int obase = is_b ? T * kLds : 0;
  int sdst_i[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int fl = blocks ? 16 * ksl + (natural ? 8 * hb + i : (i < 4 ? 4 * hb + i : 8 + 4 * hb + (i - 4))) : fblk * 8 + i;
    sdst_i[i] = obase + fl * kLds + ((rblk ^ ((fl >> 3) & 7)) * 8);
  }
  const int nks_op = fmax >> 4;                        // feature steps of a block-layout operand

  floatx16 acc[2][2];
  floatx16 accb[2];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    acc[0][0][v] = acc[0][1][v] = acc[1][0][v] = acc[1][1][v] = 0.f;
    accb[0][v] = accb[1][v] = 0.f;
  }
  const bool do_bias = (i0 == 0) && (wi == 0);
  bf16x8 ones;
#pragma unroll
  for (int v = 0; v < 8; ++v) ones[v] = (__bf16)1.0f;

  uint4 st0[8], st1[8];
  // row pointers of the thread's 8 rows for the stage being loaded next; advanced by 64 rows per stage.
  // Stages wholly inside [row_begin, row_end) need neither clamping nor masking.
  const int64_t ld64 = ld;
  const int rows_alloc = (rows + 127) & ~127;          // block-layout arrays hold whole 128-row tiles
  auto load_stage = [&](uint4* st, int rbase) {
    if (blocks) {
      // stage = rows rbase .. rbase + 63 = row tiles 2 (rbase / 64 % 2) + {0, 1} of workgroup tile rbase / 128
      const int rb = rbase < rows_alloc ? rbase : rows_alloc - 64;      // stages past the end re-read the last one (masked)
      const int tr = rb >> 7, rt = ((rb >> 6) & 1) * 2;
      const int ksg = (feat_ok ? feat : 0) >> 4;
      const uint4* p = reinterpret_cast<const uint4*>(opnd) + (((int64_t)tr * nks_op + ksg) * 4 + rt) * 64 + 32 * hb + rblk;
#pragma unroll
      for (int j = 0; j < 8; ++j) st[j] = p[(j >> 2) * 64 + 8 * (j & 3)];
    } else if (rbase + kBK <= row_end) {
      const uint16_t* p = src + (int64_t)(rbase + rblk) * ld64;
#pragma unroll
      for (int j = 0; j < 8; ++j) st[j] = *reinterpret_cast<const uint4*>(p + (32 * (j >> 2) + 8 * (j & 3)) * ld64);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        st[j] = *reinterpret_cast<const uint4*>(src + (int64_t)min(rbase + rblk + 32 * (j >> 2) + 8 * (j & 3), rows - 1) * ld64);
    }
  };
  // rows past the split (and feature blocks past the operand) are zeroed here, when the data is consumed,
  // not at load time: touching a loaded register right after the load would stall on it
  auto store_stage = [&](const uint4* st, int buf, int rbase) {
    uint4 m[8], tr[8];
    if (rbase + kBK <= row_end && feat_ok) {
#pragma unroll
      for (int j = 0; j < 8; ++j) m[j] = st[j];
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint32_t k = (rbase + rblk + 32 * (j >> 2) + 8 * (j & 3) < row_end && feat_ok) ? 0xFFFFFFFFu : 0u;
        m[j] = make_uint4(st[j].x & k, st[j].y & k, st[j].z & k, st[j].w & k);
      }
    }
    transpose8x8(m, tr);
#pragma unroll
    for (int i = 0; i < 8; ++i) *reinterpret_cast<uint4*>(&s_stage[buf * kBuf + sdst_i[i]]) = tr[i];
  };
  auto compute = [&](int buf) {
    const uint16_t* s_a = s_stage + buf * kBuf;
    const uint16_t* s_b = s_a + T * kLds;
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      bf16x8 a[2], b[2];
      const int kc = kk * 2 + (lane >> 5);          // 16-byte slot (8 rows) of this lane's fragment
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int fr = (wo * 2 + i) * 32 + (lane & 31);
        a[i] = *reinterpret_cast<const bf16x8*>(&s_a[fr * kLds + ((kc ^ ((fr >> 3) & 7)) * 8)]);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int fr = (wi * 2 + j) * 32 + (lane & 31);
        b[j] = *reinterpret_cast<const bf16x8*>(&s_b[fr * kLds + ((kc ^ ((fr >> 3) & 7)) * 8)]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
      if (do_bias) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
          accb[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], ones, accb[i], 0, 0, 0);
      }
    }
  };

  // stage s (64 rows) lives in LDS buffer s & 1; rows past the split load as zeros, so a trailing odd
  // stage adds nothing and the loop body needs no conditions
  const int nst = row_begin < row_end ? (row_end - row_begin + kBK - 1) / kBK : 0;
  if (nst > 0) {
    load_stage(st0, row_begin);
    load_stage(st1, row_begin + kBK);
    store_stage(st0, 0, row_begin);
    load_stage(st0, row_begin + 2 * kBK);
    for (int s2 = 0; s2 < nst; s2 += 2) {
      __syncthreads();
      store_stage(st1, 1, row_begin + (s2 + 1) * kBK);
      load_stage(st1, row_begin + (s2 + 3) * kBK);
      compute(0);
      __syncthreads();
      store_stage(st0, 0, row_begin + (s2 + 2) * kBK);
      load_stage(st0, row_begin + (s2 + 4) * kBK);
      compute(1);
    }
  }

  float* dst = part + (int64_t)sp * part_stride;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int o = o0 + (wo * 2 + i) * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
      if (o >= P.out) continue;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int ii = i0 + (wi * 2 + j) * 32 + (lane & 31);
        if (ii < P.in) dst[P.w_off + (int64_t)o * P.in + ii] = acc[i][j][v];
      }
      if (do_bias && (lane & 31) == 0) dst[P.b_off + o] = accb[i][v];
    }
  }
}

__global__ __launch_bounds__(256) void wgrad_bf16_kernel(gmi::WgradBatch batch, int rows, int n_split,
                                                         int chunk, float* __restrict__ part,
                                                         int64_t part_stride) {
  __shared__ __attribute__((aligned(16))) uint16_t s_stage[2 * kWgradBuf];
  int pi = 0;
  while (pi + 1 < batch.n && (int)blockIdx.x >= batch.blk_start[pi + 1]) ++pi;
  const gmi::WgradProblem& P = batch.p[pi];
  const int local = blockIdx.x - batch.blk_start[pi];
  if (P.dz_blocks) wgrad_tile<1>(P, local, rows, n_split, chunk, part, part_stride, s_stage);
  else wgrad_tile<0>(P, local, rows, n_split, chunk, part, part_stride, s_stage);
}

// ------------------------------------------------------------------------------------------------
// F32 path: one thread per output element.
template <int EPI>
__global__ void linear_f32_kernel(gmi::LinearBatch batch, int rows) {
  const gmi::LinearProblem& P = batch.p[blockIdx.z];
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)rows * P.F) return;
  const int r = (int)(idx / P.F), f = (int)(idx % P.F);
  const float* x = (const float*)P.x + (int64_t)r * P.ldx;
  const float* w = (const float*)P.w + (int64_t)f * P.wsf;
  float acc = 0.f;
  for (int k = 0; k < P.K; ++k) acc = fmaf(x[k], w[(int64_t)k * P.wsk], acc);
  if (EPI == gmi::kEpiBiasElu) {
    const float z = acc + P.bias[f];
    ((float*)P.y)[(int64_t)r * P.ldy + f] = z > 0.f ? z : expm1f(z);
  } else if (EPI == gmi::kEpiBiasHead) {
    if (f < P.F_store) ((float*)P.y)[(int64_t)r * P.ldy + f] = acc + P.bias[f];
  } else {
    const float h = ((const float*)P.h)[(int64_t)r * P.ldh + f];
    ((float*)P.y)[(int64_t)r * P.ldy + f] = acc * elu_grad_f(h);
  }
}

// grid.x over (out*in + out) outputs of one problem, grid.y = split, grid.z = problem
__global__ void wgrad_f32_kernel(gmi::WgradBatch batch, int rows, int chunk, float* __restrict__ part,
                                 int64_t part_stride) {
  const gmi::WgradProblem& P = batch.p[blockIdx.z];
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int nw = P.out * P.in;
  if (idx >= nw + P.out) return;
  const int sp = blockIdx.y;
  const int rb = sp * chunk, re = min(rows, rb + chunk);
  const float* dz = (const float*)P.dz;
  const float* x = (const float*)P.x;
  float acc = 0.f;
  float* dst = part + (int64_t)sp * part_stride;
  if (idx < nw) {
    const int o = idx / P.in, i = idx % P.in;
    for (int r = rb; r < re; ++r) acc = fmaf(dz[(int64_t)r * P.lddz + o], x[(int64_t)r * P.ldx + i], acc);
    dst[P.w_off + idx] = acc;
  } else {
    const int o = idx - nw;
    for (int r = rb; r < re; ++r) acc += dz[(int64_t)r * P.lddz + o];
    dst[P.b_off + o] = acc;
  }
}

template <int TFW, int TRW, int WRN>
int launch_bf16_big(gmi::ProfScope& ps, int epi, int rows, const gmi::LinearBatch& b, int maxF) {
  constexpr int TF = 2 * TFW * 32, TR = WRN * TRW * 32;
  const int n_rt = (rows + TR - 1) / TR, n_ft = (maxF + TF - 1) / TF;
  const int n_rt_pad = (n_rt + 7) & ~7;
  const unsigned grid = (unsigned)(n_rt_pad * n_ft * b.n);
  if (epi == gmi::kEpiBiasElu)
    ps.launch(linear_bf16_big_kernel<TFW, TRW, gmi::kEpiBiasElu, WRN>, dim3(grid), dim3(128 * WRN), 0, b, rows, n_rt,
              n_rt_pad, n_ft);
  else
    ps.launch(linear_bf16_big_kernel<TFW, TRW, gmi::kEpiEluGrad, WRN>, dim3(grid), dim3(128 * WRN), 0, b, rows, n_rt,
              n_rt_pad, n_ft);
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}

template <int WF, int WR, int TFM, int TRM>
int launch_bf16_cfg(gmi::ProfScope& ps, int epi, int rows, const gmi::LinearBatch& b, int maxF) {
  constexpr int TF = WF * TFM * 32, TR = WR * TRM * 32;
  dim3 grid((rows + TR - 1) / TR, (maxF + TF - 1) / TF, b.n);
  switch (epi) {
    case gmi::kEpiBiasElu:
      ps.launch(linear_bf16_kernel<WF, WR, TFM, TRM, gmi::kEpiBiasElu>, dim3(grid), dim3(256), 0, b, rows); break;
    case gmi::kEpiBiasHead:
      ps.launch(linear_bf16_kernel<WF, WR, TFM, TRM, gmi::kEpiBiasHead>, dim3(grid), dim3(256), 0, b, rows); break;
    default:
      ps.launch(linear_bf16_kernel<WF, WR, TFM, TRM, gmi::kEpiEluGrad>, dim3(grid), dim3(256), 0, b, rows); break;
  }
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}

}  // namespace

namespace gmi {

int launch_linear(gmi_instance* g, int dtype, int epi, int rows, const LinearBatch& b) {
  if (rows <= 0 || b.n <= 0) return GMI_OK;
  int maxF = 0;
  for (int i = 0; i < b.n; ++i) maxF = b.p[i].F > maxF ? b.p[i].F : maxF;
  if (dtype != GMI_DTYPE_F32) {
    for (int i = 0; i < b.n; ++i) {
      const LinearProblem& p = b.p[i];
      if ((p.K & 31) || (p.F & 31) || (p.ldx & 7) || (p.ldw & 7) || (epi != kEpiBiasHead && (p.ldy & 3)) ||
          (epi == kEpiEluGrad && (p.ldh & 3)))
        GMI_FAIL(GMI_ERR_BAD_SHAPE, "launch_linear: bf16 path needs padded dims (K=%d F=%d)", p.K, p.F);
    }
  }
  // kernel variant (see KernelClass): large tiles for wide layers of big batches, else by feature count
  int variant;
  if (dtype == GMI_DTYPE_F32) {
    variant = 5;
  } else if (epi != kEpiBiasHead && rows >= 8192 && maxF > 64) {
    // choose the large tile whose padding waste over the feature range is smallest
    const int waste256 = (maxF + 255) / 256 * 256 - maxF, waste128 = (maxF + 127) / 128 * 128 - maxF;
    variant = (maxF > 128 && waste256 <= waste128) ? 0 : 1;
  } else if (maxF % 128 == 0 || maxF > 256) {
    variant = 2;
  } else if (maxF % 64 == 0) {
    variant = 3;
  } else if (maxF <= 96) {
    variant = 4;
  } else {
    variant = 2;
  }
  const int role = epi == kEpiEluGrad ? 2 : (epi == kEpiBiasHead ? 1 : 0);
  ProfScope ps(g, variant == 5 ? (int)kClsLinearF32 : kClsLinear + 3 * variant + role);
  {
    // algorithmic work: 2 K F flops per row; each row's input and output once (heads write fp32, the
    // input-gradient product also reads the layer's stored activation), the weights once
    const double es = dtype == GMI_DTYPE_F32 ? 4.0 : 2.0;
    double fl = 0.0, by = 0.0;
    for (int i = 0; i < b.n; ++i) {
      const double K = b.p[i].K_log > 0 ? b.p[i].K_log : b.p[i].K, F = b.p[i].F_log > 0 ? b.p[i].F_log : b.p[i].F;
      fl += 2.0 * rows * K * F;
      by += rows * (K * es + F * (role == 1 ? 4.0 : es) + (role == 2 ? F * es : 0.0)) + K * F * es;
    }
    ps.work(fl, by);
  }
  switch (variant) {
    case 5: {
      dim3 grid((unsigned)(((int64_t)rows * maxF + 255) / 256), 1, b.n);
      switch (epi) {
        case kEpiBiasElu: ps.launch(linear_f32_kernel<kEpiBiasElu>, dim3(grid), dim3(256), 0, b, rows); break;
        case kEpiBiasHead: ps.launch(linear_f32_kernel<kEpiBiasHead>, dim3(grid), dim3(256), 0, b, rows); break;
        default: ps.launch(linear_f32_kernel<kEpiEluGrad>, dim3(grid), dim3(256), 0, b, rows); break;
      }
      GMI_LAUNCH_CHECK();
      return GMI_OK;
    }
    case 0: return launch_bf16_big<4, 2, 4>(ps, epi, rows, b, maxF);
    case 1: return launch_bf16_big<2, 2, 4>(ps, epi, rows, b, maxF);
    case 2: return launch_bf16_cfg<2, 2, 2, 2>(ps, epi, rows, b, maxF);
    case 3: return launch_bf16_cfg<1, 4, 2, 2>(ps, epi, rows, b, maxF);
    default: return launch_bf16_cfg<1, 4, 1, 2>(ps, epi, rows, b, maxF);
  }
}

int launch_wgrad(gmi_instance* g, int dtype, int rows, int n_split, int chunk, WgradBatch& b, float* part,
                 int64_t part_stride) {
  if (b.n <= 0) return GMI_OK;
  ProfScope ps(g, kClsWgrad);
  {
    // algorithmic work: 2 in out flops per row; every layer's input and output gradient read once, one
    // fp32 partial per split written
    const double es = dtype == GMI_DTYPE_F32 ? 4.0 : 2.0;
    double fl = 0.0, by = 0.0;
    for (int i = 0; i < b.n; ++i) {
      fl += 2.0 * rows * (double)b.p[i].in * b.p[i].out;
      by += rows * es * (b.p[i].in + b.p[i].out) + 4.0 * n_split * ((double)b.p[i].in * b.p[i].out + b.p[i].out);
    }
    ps.work(fl, by);
  }
  if (dtype == GMI_DTYPE_F32) {
    int maxn = 0;
    for (int i = 0; i < b.n; ++i) {
      const int n = b.p[i].out * b.p[i].in + b.p[i].out;
      maxn = n > maxn ? n : maxn;
    }
    dim3 grid((maxn + 255) / 256, n_split, b.n);
    ps.launch(wgrad_f32_kernel, dim3(grid), dim3(256), 0, b, rows, chunk, part, part_stride);
    GMI_LAUNCH_CHECK();
    return GMI_OK;
  }
  int total = 0;
  for (int i = 0; i < b.n; ++i) {
    b.blk_start[i] = total;
    total += ((b.p[i].out_pad + 127) / 128) * ((b.p[i].in_pad + 127) / 128) * n_split;
  }
  b.blk_start[b.n] = total;
  ps.launch(wgrad_bf16_kernel, dim3(total), dim3(256), 0, b, rows, n_split, chunk, part, part_stride);
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}

}  // namespace gmi
