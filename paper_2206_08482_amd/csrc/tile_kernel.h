// Row-tile trainer kernel for the wide model shapes (every hidden width a multiple of 128): minibatch gather,
// forward pass, clipped-surrogate / value loss and the whole input-gradient chain of one minibatch (stage (ii)
// of Section 5.1 of the paper, the "DRL Trainer" role of Section 3) in one launch per minibatch.
//
// A workgroup of 4 waves owns 128 samples and keeps their current activations in LDS, as the second operands of
// the 32x32x16 matrix instruction: block (k step ks, row tile rt) = 1 KiB, lane L of it = the 8 contraction
// values of sample 32 rt + L % 32 that operand lane L takes.  Every product is computed transposed,
// H^T = W X^T, and a wave owns a slice of the layer's OUTPUT FEATURES for all 128 samples (F / 128 feature tiles x
// 4 row tiles, at most 16 accumulator tiles = 256 registers): per k step it fetches its own weight blocks straight
// from the second-level cache into registers (no other wave of the workgroup needs them) and the 4 activation
// blocks from LDS, i.e. 8 KiB of operands for 16 matrix instructions.  (With a wave per 32 samples and the weights
// in LDS every wave reads every weight block: 1 KiB of LDS traffic per matrix instruction, which is the LDS
// bandwidth of a compute unit.)  The weights come from the chain stream of the register-chained kernel
// (chain_kernel.h): its blocks are the first operands of exactly these products, its k order inside a 16-wide
// step is the order in which the matrix instruction leaves its results in a lane, so a lane's 8 results of a
// k step are written back to LDS as one 16-byte piece at its own lane's slot.
//
// A layer is: k loop (all accumulators of the layer live at once) - barrier - epilogue (bias + ELU, or x ELU' of
// the stored activation; conversion; the results into LDS in place of the layer's input; from there they go to memory
// for the weight-gradient kernel) - barrier.  The next layer's first weight blocks are fetched before the epilogue.
//
// TileShapeFwd is the same walk cut after the heads (agent_act / agent_value of these models: Section 3, "DRL Agent"):
// nothing is stored for the weight gradients and the heads' results go out as policy means and values.
#pragma once
#include "chain_kernel.h"

namespace gmi_tile {
using namespace gmi_chain;

constexpr int kRows = 128;        // samples per workgroup
constexpr int kWaves = 4;
constexpr int kRing = 16;         // weight blocks in flight per wave: 16 / (feature tiles per wave) k steps
constexpr int kHPre = 3;          // tiles whose stored activations are fetched ahead in an input-gradient epilogue

template <int... DIMS>
struct TileShape {
  static constexpr bool fwd = false;      // TileShapeFwd: the forward pass alone (inference)
  static constexpr int NL = (int)sizeof...(DIMS) - 1;
  static constexpr ChainDims dims() { return ChainDims{NL, 4, {DIMS...}}; }
  static constexpr int nseg() { return cd_nseg(dims()); }
  static constexpr int maxks() { return cd_maxdim(dims()) / 16; }
  static constexpr int bias_total() {
    int n = 0;
    for (int l = 0; l < NL; ++l) n += dims().d[l + 1];
    return n;
  }
  static constexpr int bias_off(int l) {
    int n = 0;
    for (int i = 0; i < l; ++i) n += dims().d[i + 1];
    return n;
  }
  static constexpr int seg_blk0(int s) {
    int n = 0;
    for (int i = 0; i < s; ++i) n += cd_seg_blocks(dims(), i);
    return n;
  }
  static constexpr size_t x_bytes() { return (size_t)maxks() * 4 * 1024; }
  static constexpr size_t lds_bytes() { return x_bytes() + (size_t)bias_total() * 4 + (size_t)(kWaves * 40 + 64) * 4; }
  static constexpr bool valid() {
    const ChainDims D = dims();
    if (D.d[NL] != 32 || D.d[0] % 16 != 0) return false;
    for (int l = 1; l < NL; ++l)
      if (D.d[l] % 128 != 0) return false;
    // the loss epilogue's per-wave transposition buffers live in the activation area behind the head layer's input
    return x_bytes() >= 65536 + (size_t)kWaves * kScrBytes && D.d[NL - 1] / 16 * 4096 <= 65536;
  }
};

// The same shape for inference: the walk ends after the heads, nothing is stored for the weight gradients, and the
// heads' results go out as policy means and values (the products and their order are the trainer's forward pass).
template <int... DIMS>
struct TileShapeFwd : TileShape<DIMS...> {
  static constexpr bool fwd = true;
};
// Segments the kernel runs for shape S.
template <class S>
constexpr int n_run() { return S::fwd ? S::NL : S::nseg(); }

template <class S, int SEG>
struct Seg {
  static constexpr ChainDims D = S::dims();
  static constexpr int K = cd_K(D, SEG), F = cd_F(D, SEG), NKS = K / 16, NFT = F / 32;
  static constexpr bool head = SEG == S::NL - 1;
  static constexpr bool bwd = SEG >= S::NL;
  static constexpr bool last = !S::fwd && SEG == S::nseg() - 1;
  static constexpr int layer = cd_layer(D, SEG);
  static constexpr int FTW = head ? 1 : NFT / kWaves;     // feature tiles per wave
  static constexpr int RT = head ? 1 : 4;                 // row tiles per wave (the head: one row tile per wave)
  static constexpr int GS = NFT >= 4 ? 4 : NFT;           // tiles per group of the stream (chain_kernel.h)
  static constexpr int DEP = kRing / FTW < NKS ? kRing / FTW : NKS;      // k steps of weight blocks in flight
  static constexpr int XD = FTW >= 4 ? 1 : 2;             // k steps the activation blocks are read ahead (a k step of
                                                          // fewer products is shorter than an LDS round trip)
  static constexpr int blk0 = S::seg_blk0(SEG);
  // The segment's input, which the previous segment's epilogue left in LDS, goes to memory block by block (for the
  // weight-gradient kernel and for ELU') DURING this segment's k loop: h[layer] in a forward segment, dz[layer] in an
  // input-gradient segment.  (Stores issued in the epilogue would all be older than the next k loop's weight
  // fetches, and the memory counter is in order: the loop would wait for every one of them.)  Not for the first
  // segment (the gather stores its rows) nor the first input-gradient segment (the loss epilogue stores the head's).
  static constexpr int HK = NKS > 6 ? NKS - 6 : 0;        // k step at which an input-gradient segment starts to fetch ELU' inputs
  static constexpr bool store_x = !S::fwd && ((SEG >= 1 && SEG <= S::NL - 1) || SEG > S::NL);
  static_assert(head || NFT % kWaves == 0, "feature tiles divide over the waves");
  static_assert(!head || NFT == 1, "the head is one 32-wide tile");
};

template <class S>
struct Ctx {
  floatx16 acc[4][4];
  uint4 wq[kRing];                   // weight blocks of k steps g .. g + DEP - 1: block (ks, a) at (ks % DEP) * FTW + a
  uint4 xq[3][4];                    // activation blocks of k steps g .. g + XD (ring indexed by k step % 3)
  uint4 sx[2];                       // blocks of the activation area on their way to memory (store_x)
  uint4 hq[kHPre + 1][2];            // stored activations of the tiles ahead (input-gradient epilogues)
  const uint4* wnet;                 // this net's stream
  uint4* X;                          // activation area
  const float* s_bias;
  float* s_red;
  char* scr;                         // this wave's transposition buffer (loss epilogue only)
  int64_t slot;                      // experience slot of this lane's sample of the head layer
  float l_act[16], l_lo, l_ad, l_rt;
  int tid, lane, wave, s, hh;
  int row0, net;                     // first row of the workgroup's tile
};

// First weight block of wave `wave` in segment SEG: its FTW tiles are consecutive tiles of one group of the stream.
template <class S, int SEG>
__device__ __forceinline__ const uint4* seg_weights(const Ctx<S>& c) {
  using G = Seg<S, SEG>;
  const int ft0 = G::head ? 0 : c.wave * G::FTW;
  const int off = G::blk0 + (ft0 / 4) * 4 * G::NKS + (ft0 % 4);
  return c.wnet + (int64_t)off * 64;
}
template <class S, int SEG, int KS>
__device__ __forceinline__ void issue_weights(Ctx<S>& c, const uint4* wseg) {
  using G = Seg<S, SEG>;
  if constexpr (KS < G::NKS) {
#pragma unroll
    for (int a = 0; a < G::FTW; ++a) c.wq[(KS % G::DEP) * G::FTW + a] = (wseg + (KS * G::GS + a) * 64)[c.lane];
  }
}
// The first DEP k steps of segment SEG (issued before the previous segment's epilogue).
template <class S, int SEG, int KS = 0>
__device__ __forceinline__ void issue_first_weights(Ctx<S>& c) {
  if constexpr (SEG < n_run<S>()) {
    if constexpr (KS < Seg<S, SEG>::DEP) {
      issue_weights<S, SEG, KS>(c, seg_weights<S, SEG>(c));
      issue_first_weights<S, SEG, KS + 1>(c);
    }
  }
}

template <class S, int SEG, int KS>
__device__ __forceinline__ void read_x(Ctx<S>& c) {
  using G = Seg<S, SEG>;
  if constexpr (KS < G::NKS) {
#pragma unroll
    for (int b = 0; b < G::RT; ++b) c.xq[KS % 3][b] = c.X[(KS * 4 + (G::head ? c.wave : b)) * 64 + c.lane];
  }
}

// Block layout of the activation / gradient arrays this kernel leaves for the weight-gradient kernel and for its own
// ELU' factors: exactly the 1 KiB operand blocks of the activation area, workgroup tile after workgroup tile:
// block (k step ks, row tile rt) of the 128 rows of tile tr of an array of NKS k steps starts at 16-byte word
// ((tr * NKS + ks) * 4 + rt) * 64.  (Row-major, a lane's 8 values of a k step are two 8-byte pieces of a row:
// 32 rows x 16 bytes per load or store instruction; as blocks every access is 1 KiB contiguous.)
__device__ __forceinline__ int64_t block_word(int tr, int nks, int ks, int rt) { return (((int64_t)tr * nks + ks) * 4 + rt) * 64; }

// Stored activations h[layer] of tile T = a * RT + b of this wave (input-gradient epilogue of segment SEG): the
// lane's own slots of the blocks (2 ft, b) and (2 ft + 1, b), i.e. the values at the positions of its 16 results.
template <class S, int SEG, int T>
__device__ __forceinline__ void fetch_h(Ctx<S>& c, const ChainArgs& a) {
  using G = Seg<S, SEG>;
  if constexpr (G::bwd && T < G::FTW * G::RT) {
    constexpr int ta = T / G::RT, tb = T % G::RT;
    constexpr int nks = G::D.d[G::layer] / 16;
    const int ft = c.wave * G::FTW + ta;
    const uint4* p = reinterpret_cast<const uint4*>(a.h[c.net][G::layer]) + block_word(blockIdx.x, nks, 2 * ft, tb) + c.lane;
    c.hq[T % (kHPre + 1)][0] = p[0];
    c.hq[T % (kHPre + 1)][1] = p[4 * 64];
  }
}

template <class S, int SEG, int T>
__device__ __forceinline__ void fetch_h_first(Ctx<S>& c, const ChainArgs& a) {
  if constexpr (T < kHPre) {
    fetch_h<S, SEG, T>(c, a);
    fetch_h_first<S, SEG, T + 1>(c, a);
  }
}

// The small operations that ride along with the products of k step KS, by index I: I < RT: the activation block of
// row tile I for k step KS + XD; then, where the segment's input goes to memory (store_x), wave w's share of that
// move: I = RT reads block (KS, w) of the activation area, I = RT + 1 stores the block read a k step earlier.
template <class S, int SEG>
__device__ __forceinline__ uint4* store_x_array(const Ctx<S>& c, const ChainArgs& a) {
  using G = Seg<S, SEG>;
  return reinterpret_cast<uint4*>(G::bwd ? a.dz[c.net][G::layer] : a.h[c.net][G::layer]);
}
template <class S, int SEG, int KS, int I>
__device__ __forceinline__ void aux_op(Ctx<S>& c, const ChainArgs& a) {
  using G = Seg<S, SEG>;
  if constexpr (I < G::RT) {
    if constexpr (KS + G::XD < G::NKS)
      c.xq[(KS + G::XD) % 3][I] = c.X[((KS + G::XD) * 4 + (G::head ? c.wave : I)) * 64 + c.lane];
  } else if constexpr (G::store_x) {
    if constexpr (I == G::RT) {
      c.sx[KS & 1] = c.X[(KS * 4 + c.wave) * 64 + c.lane];
    } else if constexpr (KS >= 1) {
      (store_x_array<S, SEG>(c, a) + block_word(blockIdx.x, G::NKS, KS - 1, c.wave))[c.lane] = c.sx[(KS - 1) & 1];      // arrays hold whole tiles
    }
  }
}
template <class S, int SEG, int KS, int FIDX, int I>
__device__ __forceinline__ void aux_slot(Ctx<S>& c, const ChainArgs& a) {
  using G = Seg<S, SEG>;
  constexpr int NAUX = G::RT + 2, NFREE = G::FTW * (G::RT - 1);
  if constexpr (I < NAUX) {
    if constexpr (I % NFREE == FIDX) aux_op<S, SEG, KS, I>(c, a);
    aux_slot<S, SEG, KS, FIDX, I + 1>(c, a);
  }
}

// Product M = a * RT + b of k step KS and what follows it.  A wave issues in order and a matrix instruction keeps
// its unit busy for 32 cycles: the fetches and address arithmetic of a k step, issued in one block, leave the unit
// idle meanwhile (measured: ~100-170 of a k step's 256 / 512 cycles), one or two of them after every product do not.
// The next weight block of feature tile a follows the last product that reads the present one.
template <class S, int SEG, int KS, int M>
__device__ __forceinline__ void k_products(Ctx<S>& c, const ChainArgs& a, const uint4* wseg) {
  using G = Seg<S, SEG>;
  if constexpr (M < G::FTW * G::RT) {
    constexpr int ta = M / G::RT, tb = M % G::RT;
    c.acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
        __builtin_bit_cast(bf16x8, c.wq[(KS % G::DEP) * G::FTW + ta]), __builtin_bit_cast(bf16x8, c.xq[KS % 3][tb]),
        c.acc[ta][tb], 0, 0, 0);
    if constexpr (tb == G::RT - 1) {
      if constexpr (KS + G::DEP < G::NKS)
        c.wq[(KS % G::DEP) * G::FTW + ta] = (wseg + ((KS + G::DEP) * G::GS + ta) * 64)[c.lane];
      if constexpr (G::RT == 1) {                                 // the head: one product per k step
        aux_op<S, SEG, KS, 0>(c, a);
        aux_op<S, SEG, KS, 1>(c, a);
        aux_op<S, SEG, KS, 2>(c, a);
      }
    } else {
      aux_slot<S, SEG, KS, ta * (G::RT - 1) + tb, 0>(c, a);
    }
    __builtin_amdgcn_sched_barrier(0);
    k_products<S, SEG, KS, M + 1>(c, a, wseg);
  }
}

template <class S, int SEG, int KS>
__device__ __forceinline__ void k_steps(Ctx<S>& c, const ChainArgs& a, const uint4* wseg) {
  using G = Seg<S, SEG>;
  if constexpr (KS < G::NKS) {
    if constexpr (G::bwd && KS == G::HK) {          // the first tiles' stored activations, late enough not to hold up
      fetch_h_first<S, SEG, 0>(c, a);               // the weight fetches behind them, early enough to be there
    }
    k_products<S, SEG, KS, 0>(c, a, wseg);
    k_steps<S, SEG, KS + 1>(c, a, wseg);
  }
}

// Epilogue of tile T of a hidden forward layer or of an input-gradient layer.
template <class S, int SEG, int T>
__device__ __forceinline__ void tile_epilogue(Ctx<S>& c, const ChainArgs& a) {
  using G = Seg<S, SEG>;
  if constexpr (T < G::FTW * G::RT) {
    constexpr int ta = T / G::RT, tb = T % G::RT;
    const int ft = c.wave * G::FTW + ta;
    fetch_h<S, SEG, T + kHPre>(c, a);
    const floatx16& acc = c.acc[ta][tb];
    uint32_t w[8];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float v0 = acc[4 * q + 0], v1 = acc[4 * q + 1], v2 = acc[4 * q + 2], v3 = acc[4 * q + 3];
      if constexpr (G::bwd) {
        const uint4 hb = c.hq[T % (kHPre + 1)][q / 2];
        const uint32_t h01 = q % 2 == 0 ? hb.x : hb.z, h23 = q % 2 == 0 ? hb.y : hb.w;
        v0 *= elu_grad_f(bf16_lo(h01)); v1 *= elu_grad_f(bf16_hi(h01));
        v2 *= elu_grad_f(bf16_lo(h23)); v3 *= elu_grad_f(bf16_hi(h23));
      } else {
        v0 = elu_f(v0); v1 = elu_f(v1); v2 = elu_f(v2); v3 = elu_f(v3);      // the bias is in the sums already
      }
      w[2 * q] = pack_bf16(v0, v1);
      w[2 * q + 1] = pack_bf16(v2, v3);
    }
    c.X[((2 * ft + 0) * 4 + tb) * 64 + c.lane] = make_uint4(w[0], w[1], w[2], w[3]);
    c.X[((2 * ft + 1) * 4 + tb) * 64 + c.lane] = make_uint4(w[4], w[5], w[6], w[7]);
    tile_epilogue<S, SEG, T + 1>(c, a);
  }
}

// This lane's loss inputs (sample row0 + 32 wave + s): unconditional loads, rows and features past the end read a
// valid neighbour, their results are dropped.
template <class S>
__device__ __forceinline__ void fetch_loss_inputs(Ctx<S>& c, const ChainArgs& a) {
  c.l_lo = a.b_logp[c.slot]; c.l_ad = a.b_adv[c.slot]; c.l_rt = a.b_ret[c.slot];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int f = 8 * (i >> 2) + 4 * c.hh + (i & 3);
    const int fc = f < a.act_dim ? f : a.act_dim - 1;
    c.l_act[i] = a.b_act[c.slot * a.act_dim + fc];
  }
}

// Loss on the wave's 32 samples (row tile `wave` of the workgroup) from the head's accumulators: lane = sample s,
// half hh; register i = feature 8 (i / 4) + 4 hh + i % 4.  Leaves the head gradient as the two k steps of the first
// input-gradient product in the activation area and, as the same blocks, in dz[NL - 1], and the workgroup's
// statistics row.
template <class S>
__device__ __forceinline__ void loss_epilogue(Ctx<S>& c, const ChainArgs& a, const floatx16& acc) {
  constexpr int HB = S::bias_off(S::NL - 1);
  const int A = a.act_dim;
  const int wrow0 = c.row0 + 32 * c.wave;
  const int row = wrow0 + c.s;
  const bool ok = row < a.rows;
  const float inv_m = 1.0f / (float)a.rows;
  float d[16];
  float* red = c.s_red + c.wave * 40;
  if (c.net == 0) {
    const float* s_ls = c.s_red + kWaves * 40;      // [f] log_std, [32 + f] exp(-log_std) (0 for f >= A)
    float z[16], isg[16];
    float lp = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int f0 = 8 * q + 4 * c.hh;
      const float4 ls4 = *reinterpret_cast<const float4*>(s_ls + f0);
      const float4 ig4 = *reinterpret_cast<const float4*>(s_ls + 32 + f0);
      const float4 b4 = *reinterpret_cast<const float4*>(c.s_bias + HB + f0);
      const float lsv[4] = {ls4.x, ls4.y, ls4.z, ls4.w}, igv[4] = {ig4.x, ig4.y, ig4.z, ig4.w};
      const float bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = 4 * q + e;
        const float mu = acc[i] + bv[e];
        isg[i] = igv[e];
        z[i] = (c.l_act[i] - mu) * igv[e];                    // 0 for f >= A
        lp += f0 + e < A ? -0.5f * z[i] * z[i] - lsv[e] - 0.918938533204672742f : 0.f;
      }
    }
    lp += __shfl_xor(lp, 32, 64);                   // the other half holds the other 16 features
    float s_pl = 0.f, s_kl = 0.f, s_cf = 0.f, g_lp = 0.f;
    if (ok) {
      const float lo = c.l_lo, ad = c.l_ad;
      const float ratio = __expf(lp - lo);
      const float u1 = ratio * ad;
      const float u2 = fminf(fmaxf(ratio, 1.0f - a.clip), 1.0f + a.clip) * ad;
      g_lp = (u1 <= u2) ? -(ad * ratio) * inv_m : 0.f;
      if (c.hh == 0) {                               // each sample counts once
        s_pl = -fminf(u1, u2);
        s_kl = lo - lp;
        s_cf = fabsf(ratio - 1.0f) > a.clip ? 1.f : 0.f;
      }
    }
    // log_std gradient partials g_lp (z^2 - 1): transposed through the wave's buffer as [feature][sample] fp32,
    // then lane f < 32 sums feature f's 32 samples in a fixed order
    float* tp = reinterpret_cast<float*>(c.scr);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int f = 8 * (i >> 2) + 4 * c.hh + (i & 3);
      d[i] = g_lp * z[i] * isg[i];
      tp[f * 33 + c.s] = g_lp * (z[i] * z[i] - 1.0f);
    }
    if (c.lane < 32) {
      float sum = 0.f;
#pragma unroll
      for (int k = 0; k < 32; ++k) sum += tp[c.lane * 33 + k];
      red[8 + c.lane] = c.lane < A ? sum : 0.f;
    }
    s_pl = wave_sum64(s_pl); s_kl = wave_sum64(s_kl); s_cf = wave_sum64(s_cf);
    if (c.lane == 0) { red[0] = s_pl; red[1] = s_kl; red[2] = s_cf; }
  } else {
    float s_vl = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) d[i] = 0.f;
    if (ok && c.hh == 0) {
      const float dv = acc[0] + c.s_bias[HB] - c.l_rt;
      s_vl = dv * dv;
      d[0] = 2.0f * a.c_v * dv * inv_m;
    }
    s_vl = wave_sum64(s_vl);
    if (c.lane == 0) red[0] = s_vl;
  }
  uint32_t w[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) w[q] = pack_bf16(d[2 * q], d[2 * q + 1]);
  c.X[(0 * 4 + c.wave) * 64 + c.lane] = make_uint4(w[0], w[1], w[2], w[3]);
  c.X[(1 * 4 + c.wave) * 64 + c.lane] = make_uint4(w[4], w[5], w[6], w[7]);
  {
    uint4* arr = reinterpret_cast<uint4*>(a.dz[c.net][S::NL - 1]);
    (arr + block_word(blockIdx.x, 2, 0, c.wave))[c.lane] = make_uint4(w[0], w[1], w[2], w[3]);      // arrays hold whole tiles
    (arr + block_word(blockIdx.x, 2, 1, c.wave))[c.lane] = make_uint4(w[4], w[5], w[6], w[7]);
  }
  // workgroup sums -> this tile's row of the statistics partials
  __syncthreads();
  float* out = a.stat_part + (int64_t)blockIdx.x * (gmi::kStatStride + A);
  if (c.net == 0) {
    if (c.tid < 3) {
      float v = 0.f;
      for (int wv = 0; wv < kWaves; ++wv) v += c.s_red[wv * 40 + c.tid];
      out[c.tid == 0 ? 0 : (c.tid == 1 ? 3 : 4)] = v;
    }
    if (c.tid == 3) {
      float ent = 0.f;
      if (blockIdx.x == 0)
        for (int j = 0; j < A; ++j) ent += a.log_std[j] + 1.418938533204672742f;
      out[2] = ent;
      out[5] = out[6] = out[7] = 0.f;
    }
    if (c.tid >= 64 && c.tid < 64 + A) {
      const int j = c.tid - 64;
      float v = 0.f;
      for (int wv = 0; wv < kWaves; ++wv) v += c.s_red[wv * 40 + 8 + j];
      out[gmi::kStatStride + j] = v;
    }
  } else if (c.tid == 0) {
    float v = 0.f;
    for (int wv = 0; wv < kWaves; ++wv) v += c.s_red[wv * 40];
    out[1] = v;
  }
}

// Inference: the head's results of row tile `wave` (lane = row, register i = feature 8 (i / 4) + 4 hh + i % 4) plus
// the head's bias go out as policy means [rows, act_dim] or as values [rows].
template <class S>
__device__ __forceinline__ void head_outputs(Ctx<S>& c, const ChainArgs& a, const floatx16& acc) {
  constexpr int HB = S::bias_off(S::NL - 1);
  const int row = c.row0 + 32 * c.wave + c.s;
  if (row >= a.rows) return;
  if (c.net == 0) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int f = 8 * (i / 4) + 4 * c.hh + (i % 4);
      if (f < a.act_dim) a.mu_out[(int64_t)row * a.act_dim + f] = acc[i] + c.s_bias[HB + f];
    }
  } else if (c.hh == 0) {
    a.val_out[row] = acc[0] + c.s_bias[HB];
  }
}

template <class S, int SEG>
__device__ __forceinline__ void run_segment(Ctx<S>& c, const ChainArgs& a) {
  if constexpr (SEG < n_run<S>()) {
    using G = Seg<S, SEG>;
    const uint4* wseg = seg_weights<S, SEG>(c);
    if constexpr (!G::bwd && !G::head) {
      // the accumulators start at the bias (register i of a lane = feature 8 (i / 4) + 4 hh + i % 4 of the tile)
      constexpr int boff = S::bias_off(G::layer);
#pragma unroll
      for (int ta = 0; ta < G::FTW; ++ta) {
        const float* bp = c.s_bias + boff + 32 * (c.wave * G::FTW + ta) + 4 * c.hh;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 b4 = *reinterpret_cast<const float4*>(bp + 8 * q);
#pragma unroll
          for (int tb = 0; tb < G::RT; ++tb) {
            c.acc[ta][tb][4 * q + 0] = b4.x; c.acc[ta][tb][4 * q + 1] = b4.y;
            c.acc[ta][tb][4 * q + 2] = b4.z; c.acc[ta][tb][4 * q + 3] = b4.w;
          }
        }
      }
    } else {
#pragma unroll
      for (int ta = 0; ta < G::FTW; ++ta)
#pragma unroll
        for (int tb = 0; tb < G::RT; ++tb)
#pragma unroll
          for (int v = 0; v < 16; ++v) c.acc[ta][tb][v] = 0.f;
    }
    read_x<S, SEG, 0>(c);
    if constexpr (G::XD > 1) read_x<S, SEG, 1>(c);
    k_steps<S, SEG, 0>(c, a, wseg);
    if constexpr (G::store_x)
      (store_x_array<S, SEG>(c, a) + block_word(blockIdx.x, G::NKS, G::NKS - 1, c.wave))[c.lane] = c.sx[(G::NKS - 1) & 1];
    issue_first_weights<S, SEG + 1>(c);
    __syncthreads();                       // every wave is done with the layer's input
    // this lane's loss inputs: cold loads, issued where a long stretch of arithmetic follows and no younger load is
    // waited for (the memory counter is in order)
    if constexpr (!S::fwd && SEG == (S::NL >= 3 ? S::NL - 3 : 0)) fetch_loss_inputs<S>(c, a);
    if constexpr (G::head && S::fwd) {
      head_outputs<S>(c, a, c.acc[0][0]);
    } else if constexpr (G::head) {
      loss_epilogue<S>(c, a, c.acc[0][0]);
    } else {
      tile_epilogue<S, SEG, 0>(c, a);
    }
    __syncthreads();
    if constexpr (G::last) {
      // nothing consumes the last results on chip: row tile `wave` of the activation area goes to dz[layer - 1]
      // block by block, the way a k loop moves its input
      uint4* arr = reinterpret_cast<uint4*>(a.dz[c.net][G::layer - 1]);
#pragma unroll 8
      for (int ks = 0; ks < G::F / 16; ++ks)
        (arr + block_word(blockIdx.x, G::F / 16, ks, c.wave))[c.lane] = c.X[(ks * 4 + c.wave) * 64 + c.lane];      // arrays hold whole tiles
    }
    run_segment<S, SEG + 1>(c, a);
  }
}

template <class S>
__global__ __launch_bounds__(kWaves * 64) void train_tile_kernel(ChainArgs a) {
  static_assert(S::valid(), "shape not supported by the row-tile trainer kernel");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  constexpr ChainDims D = S::dims();
  Ctx<S> c;
  c.tid = threadIdx.x;
  c.lane = c.tid & 63;
  c.wave = __builtin_amdgcn_readfirstlane(c.tid >> 6);
  c.s = c.lane & 31;
  c.hh = c.lane >> 5;
  c.net = S::fwd ? (int)blockIdx.y + a.net0 : (int)blockIdx.y;
  c.row0 = blockIdx.x * kRows;
  c.X = reinterpret_cast<uint4*>(smem_raw);
  float* s_bias = reinterpret_cast<float*>(smem_raw + S::x_bytes());
  c.s_bias = s_bias;
  c.s_red = s_bias + S::bias_total();
  c.scr = reinterpret_cast<char*>(smem_raw) + 65536 + c.wave * kScrBytes;
  c.wnet = reinterpret_cast<const uint4*>(a.wstream[c.net]);

  issue_first_weights<S, 0>(c);
  {
    int off = 0;
#pragma unroll
    for (int l = 0; l < S::NL; ++l) {
      for (int f = c.tid; f < D.d[l + 1]; f += kWaves * 64) s_bias[off + f] = a.bias[c.net][l][f];
      off += D.d[l + 1];
    }
  }
  for (int i = c.tid; i < kWaves * 40; i += kWaves * 64) c.s_red[i] = 0.f;
  if (c.tid < 32) {                      // per-feature constants of the Gaussian log-prob (policy net)
    const int fc = c.tid < a.act_dim ? c.tid : a.act_dim - 1;
    const float ls = a.log_std[fc];
    c.s_red[kWaves * 40 + c.tid] = ls;
    c.s_red[kWaves * 40 + 32 + c.tid] = c.tid < a.act_dim ? expf(-ls) : 0.f;
  }
  if constexpr (!S::fwd) {
    // this lane's sample of the head layer (rows past the batch take the last sample; their results are dropped)
    const int row = c.row0 + 32 * c.wave + c.s;
    const int rc = row < a.rows ? row : a.rows - 1;
    const int sm = a.idx ? a.idx[rc] : rc;
    c.slot = (int64_t)(sm / a.n_envs) * a.ld_envs + (sm % a.n_envs);
  }
  {
    // The gather: the workgroup's 128 observation rows as the first layer's operand blocks in natural k order (lane
    // (s, h) of block (ks, rt) holds features 16 ks + 8 h .. + 7 of sample 32 rt + s), zero padded.  A lane takes
    // 16-byte piece jj + 4 it of row 16 g + rr: 16 lanes write 256 consecutive bytes of LDS, 4 lanes read 64
    // consecutive bytes of a row.  The policy net's workgroups also leave the same blocks in x0b for the
    // weight-gradient kernel.  All loads unconditional (clamped addresses, selected values).
    constexpr int NP = D.d[0] / 8;                       // 16-byte pieces of a row
    const int rr = c.lane & 15, jj = c.lane >> 4;
    const int O = a.obs_dim;
    constexpr int NI = (NP + 3) / 4;
    int sm[2];
#pragma unroll
    for (int gi = 0; gi < 2; ++gi) {
      const int row = c.row0 + 16 * (c.wave + kWaves * gi) + rr;
      const int rc = row < a.rows ? row : a.rows - 1;
      sm[gi] = a.idx ? a.idx[rc] : rc;
    }
    uint4 v[2][NI];
    if (a.x0_ready != 0) {                               // workgroup-uniform; no branch around a single load
#pragma unroll
      for (int gi = 0; gi < 2; ++gi) {
        const int row = c.row0 + 16 * (c.wave + kWaves * gi) + rr;
        const uint16_t* src = a.x0_ready == 1 ? a.x0 + (int64_t)row * D.d[0] : a.x16 + (int64_t)sm[gi] * D.d[0];
#pragma unroll
        for (int it = 0; it < NI; ++it) {
          const int j = 4 * it + jj;
          v[gi][it] = *reinterpret_cast<const uint4*>(src + 8 * (j < NP ? j : NP - 1));
        }
      }
    } else {
#pragma unroll
      for (int gi = 0; gi < 2; ++gi) {
        const int64_t slot = (int64_t)(sm[gi] / a.n_envs) * a.ld_envs + (sm[gi] % a.n_envs);
        const float* orow = a.b_obs + slot * O;
#pragma unroll
        for (int it = 0; it < NI; ++it) {
          const int j = 4 * it + jj;
          const int jc = j < NP ? j : NP - 1;
          float f[8];
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const int f0 = 8 * jc + 4 * q;                  // O % 4 == 0: a piece is inside the row or past it
            const float4 t = *reinterpret_cast<const float4*>(orow + (f0 < O ? f0 : O - 4));
            f[4 * q + 0] = f0 < O ? t.x : 0.f; f[4 * q + 1] = f0 < O ? t.y : 0.f;
            f[4 * q + 2] = f0 < O ? t.z : 0.f; f[4 * q + 3] = f0 < O ? t.w : 0.f;
          }
          v[gi][it] = make_uint4(pack_bf16(f[0], f[1]), pack_bf16(f[2], f[3]), pack_bf16(f[4], f[5]), pack_bf16(f[6], f[7]));
        }
      }
    }
    uint4* xb = reinterpret_cast<uint4*>(a.x0b) + block_word(blockIdx.x, D.d[0] / 16, 0, 0);
#pragma unroll
    for (int gi = 0; gi < 2; ++gi) {
      const int r = 16 * (c.wave + kWaves * gi) + rr;
#pragma unroll
      for (int it = 0; it < NI; ++it) {
        const int j = 4 * it + jj;
        if (j < NP) {
          const int w = ((j >> 1) * 4 + (r >> 5)) * 64 + (r & 31) + 32 * (j & 1);
          c.X[w] = v[gi][it];
          if (!S::fwd && c.net == 0) xb[w] = v[gi][it];      // arrays hold whole tiles
        }
      }
    }
  }
  __syncthreads();
  run_segment<S, 0>(c, a);
}

template <class S>
bool shape_matches(const ModelLayout& L) {
  constexpr ChainDims D = S::dims();
  if (L.n_layers != D.nl) return false;
  for (int net = 0; net < 2; ++net)
    for (int l = 0; l < D.nl; ++l)
      if (L.net[net][l].in_pad != D.d[l] || L.net[net][l].out_pad != D.d[l + 1]) return false;
  return true;
}

template <class S>
int launch_shape(gmi_instance* g, const ChainArgs& a, int rows, int* tiles_out, double flops, double bytes) {
  static bool attr = false;
  const size_t lds = S::lds_bytes();
  const int tiles = (rows + kRows - 1) / kRows;
  *tiles_out = tiles;
  if (!S::fwd && tiles > gmi::kLossBlocksMax) return GMI_ERR_UNSUPPORTED;      // one statistics row per tile
  if (a.x0_ready == 0 && (a.obs_dim % 4 != 0 || a.obs_dim < 4)) return GMI_ERR_UNSUPPORTED;
  if (!attr) {
    GMI_HIP(hipFuncSetAttribute((const void*)train_tile_kernel<S>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr = true;
  }
  gmi::ProfScope ps(g, S::fwd ? gmi::kClsFusedAgent : gmi::kClsChainTrain);
  ps.work(flops, bytes);
  ps.launch(train_tile_kernel<S>, dim3(tiles, S::fwd ? 2 - a.net0 : 2), dim3(kWaves * 64), lds, a);
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}

}  // namespace gmi_tile

namespace gmi {
// One function per shape compiled for the row-tile kernel (tile_p<k>.hip), with the contract of the chained kernel's
// parts (chain_kernel.h): GMI_ERR_UNSUPPORTED if the model has another shape; rows == 0 only asks (the answer: the
// stream's group size 4, plus 256 for the gather from the bf16 copy of all observations).
constexpr int kTileParts = 2;
constexpr int kTileFwdParts = 2;
#define GMI_TILE_PART_DECL(k)                                                                              \
  int launch_tile_part##k(gmi_instance* g, const ModelLayout& L, const gmi_chain::ChainArgs& a, int rows, \
                          int* tiles_out, double flops, double bytes)
GMI_TILE_PART_DECL(0); GMI_TILE_PART_DECL(1);
#define GMI_TILE_FWD_PART_DECL(k)                                                                              \
  int launch_tile_fwd_part##k(gmi_instance* g, const ModelLayout& L, const gmi_chain::ChainArgs& a, int rows, \
                              int* tiles_out, double flops, double bytes)
GMI_TILE_FWD_PART_DECL(0); GMI_TILE_FWD_PART_DECL(1);
#define GMI_TILE_FWD_PART_DEFINE(k, ...)                                                          \
  GMI_TILE_FWD_PART_DECL(k) {                                                                     \
    using S = gmi_tile::TileShapeFwd<__VA_ARGS__>;                                                \
    if (!gmi_tile::shape_matches<S>(L)) return GMI_ERR_UNSUPPORTED;                               \
    if (rows == 0) { *tiles_out = 4; return GMI_OK; }                                             \
    return gmi_tile::launch_shape<S>(g, a, rows, tiles_out, flops, bytes);                        \
  }
#define GMI_TILE_PART_DEFINE(k, ...)                                                              \
  GMI_TILE_PART_DECL(k) {                                                                         \
    using S = gmi_tile::TileShape<__VA_ARGS__>;                                                   \
    if (!gmi_tile::shape_matches<S>(L)) return GMI_ERR_UNSUPPORTED;                               \
    if (rows == 0) { *tiles_out = 4 | 256; return GMI_OK; }                                       \
    return gmi_tile::launch_shape<S>(g, a, rows, tiles_out, flops, bytes);                        \
  }
}  // namespace gmi
