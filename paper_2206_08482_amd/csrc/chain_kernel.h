// Register-chained trainer kernel: minibatch gather, forward pass, clipped-surrogate / value loss and the whole
// input-gradient chain of one minibatch (stage (ii) of Section 5.1 of the paper, the "DRL Trainer" role of
// Section 3) in one launch per minibatch.
//
// A wave owns 32 samples and carries their activations from layer to layer IN REGISTERS.  Every product is
// computed transposed, H^T = W X^T: the weights are the first operand of the 32x32x16 matrix instruction
// (row = output feature), the activations the second (lane = sample).  The result then has lane = sample and
// its 16 registers hold 16 of the tile's 32 features, which is -- up to a fixed permutation of the features
// inside each 16-wide k step -- exactly the second-operand layout of the next layer.  A permutation of the
// contraction index is free as long as the weights use the same one, so the weights are kept in a second
// shadow copy (the "chain stream") whose 1 KiB blocks are already permuted and already in the order the kernel
// consumes them.  No activation ever goes through LDS on its way to the next layer.
//
// The 4 or 8 waves of a workgroup walk the stream in lockstep; the stream is staged through three LDS slots
// (16 KiB chunks, global loads issued several chunks ahead into registers), so a workgroup reads every weight
// once for its 128 or 256 samples.  Activations and gradients that the weight-gradient kernel needs are written
// row-major through a small per-wave LDS transposition buffer, so that rows leave the chip as 64..256-byte
// pieces.  The epilogue of a group of feature tiles (bias + ELU or ELU', conversion, that store) is a list of
// small items; shapes with room for a second accumulator set run the items of one group between the matrix
// instructions of the next (DEFER).
//
// Layout of this file: the plan (cd_*: pure functions of the layer widths, shared by kernel and host), the
// kernel's arguments and per-lane context, chunk movement, epilogue items, the k-step loop, the kernel, and the
// launch helpers that chain_p<k>.hip instantiate for one shape each.

#pragma once
#include "internal.h"

namespace gmi_chain {


typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
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
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// ---------------------------------------------------------------------------------------------------------
// The plan: which 1 KiB weight blocks the kernel consumes in which order.  Pure functions of the padded layer
// widths d[0..nl] (d[0] = input, d[nl] = head), used at compile time by the kernel and at run time by the
// host when it describes the stream to the packing kernel.
//
// Segment s < nl is the forward product of layer s (K = d[s] in, F = d[s+1] out); segment s >= nl is the
// input-gradient product of layer l = 2 nl - 1 - s (K = d[l+1], F = d[l]), l = nl-1 .. 1.  A segment's F/32
// feature tiles are cut into groups of 4, then 2, then 1 tiles; a group's blocks are ordered k step major
// (block (ks, t) = tile t of the group, k step ks); a chunk is 16 / (group size) k steps of one group,
// i.e. at most 16 blocks.
struct ChainDims {
  int nl;
  int gmax;              // largest group: 4 or 2 feature tiles
  int d[GMI_MAX_HIDDEN + 2];
};
__host__ __device__ constexpr int cd_nseg(const ChainDims& D) { return 2 * D.nl - 1; }
__host__ __device__ constexpr int cd_layer(const ChainDims& D, int s) { return s < D.nl ? s : 2 * D.nl - 1 - s; }
__host__ __device__ constexpr int cd_K(const ChainDims& D, int s) { return s < D.nl ? D.d[s] : D.d[cd_layer(D, s) + 1]; }
__host__ __device__ constexpr int cd_F(const ChainDims& D, int s) { return s < D.nl ? D.d[s + 1] : D.d[cd_layer(D, s)]; }
// nft tiles = nft / gmax groups of gmax, then (2), then (1)
__host__ __device__ constexpr int cd_ngroups(int nft, int gmax) {
  return nft / gmax + ((nft % gmax) >= 2 ? 1 : 0) + ((nft % gmax) & 1);
}
__host__ __device__ constexpr int cd_gsize(int nft, int gi, int gmax) {
  const int full = nft / gmax;
  if (gi < full) return gmax;
  if (gi == full && (nft % gmax) >= 2) return 2;
  return 1;
}
__host__ __device__ constexpr int cd_gtile0(int nft, int gi, int gmax) {
  const int full = nft / gmax;
  if (gi <= full) return gmax * gi;
  return gmax * full + 2;
}
__host__ __device__ constexpr int cd_kcsteps(int gs) { return 16 / gs; }
__host__ __device__ constexpr int cd_group_chunks(int nks, int gs) { return (nks + cd_kcsteps(gs) - 1) / cd_kcsteps(gs); }
__host__ __device__ constexpr int cd_seg_chunks(const ChainDims& D, int s) {
  const int nft = cd_F(D, s) / 32, nks = cd_K(D, s) / 16;
  int n = 0;
  for (int gi = 0; gi < cd_ngroups(nft, D.gmax); ++gi) n += cd_group_chunks(nks, cd_gsize(nft, gi, D.gmax));
  return n;
}
__host__ __device__ constexpr int cd_seg_blocks(const ChainDims& D, int s) { return (cd_F(D, s) / 32) * (cd_K(D, s) / 16); }
__host__ __device__ constexpr int cd_nchunks(const ChainDims& D) {
  int n = 0;
  for (int s = 0; s < cd_nseg(D); ++s) n += cd_seg_chunks(D, s);
  return n;
}
__host__ __device__ constexpr int cd_nblocks(const ChainDims& D) {
  int n = 0;
  for (int s = 0; s < cd_nseg(D); ++s) n += cd_seg_blocks(D, s);
  return n;
}
__host__ __device__ constexpr int cd_maxdim(const ChainDims& D) {
  int m = 0;
  for (int i = 0; i <= D.nl; ++i) m = D.d[i] > m ? D.d[i] : m;
  return m;
}

struct ChunkInfo {
  int seg, gi, gs, tile0, ks0, nks, blk_off, nblk;
  bool first, last;      // first / last chunk of its group
  int gord;              // ordinal of the group among all groups of the plan
  int prev_last;         // index of the last chunk of the previous group (-1 for the first group)
  int seg_nks;           // k steps of the segment
  int group_chunks;      // chunks of this chunk's group
  int last_in;           // 0 for the group's last chunk, 1 for the one before, ...
};
__host__ __device__ constexpr ChunkInfo cd_chunk(const ChainDims& D, int c) {
  ChunkInfo ci = {0, 0, 0, 0, 0, 0, 0, 0, false, false, 0, -1, 0, 0, 0};
  int blk = 0, cc = 0, gord = 0;
  for (int s = 0; s < cd_nseg(D); ++s) {
    const int nft = cd_F(D, s) / 32, nks = cd_K(D, s) / 16;
    for (int gi = 0; gi < cd_ngroups(nft, D.gmax); ++gi, ++gord) {
      const int gs = cd_gsize(nft, gi, D.gmax), nc = cd_group_chunks(nks, gs), kcs = cd_kcsteps(gs);
      const int group_first = cc;
      for (int kc = 0; kc < nc; ++kc) {
        const int k0 = kc * kcs, n = (nks - k0) < kcs ? (nks - k0) : kcs;
        if (cc == c) {
          ci.seg = s; ci.gi = gi; ci.gs = gs; ci.tile0 = cd_gtile0(nft, gi, D.gmax); ci.ks0 = k0; ci.nks = n;
          ci.blk_off = blk; ci.nblk = n * gs; ci.first = kc == 0; ci.last = kc == nc - 1;
          ci.gord = gord; ci.prev_last = group_first - 1; ci.seg_nks = nks; ci.group_chunks = nc; ci.last_in = nc - 1 - kc;
          return ci;
        }
        blk += n * gs;
        ++cc;
      }
    }
  }
  return ci;
}

// The epilogue of a group (bias + ELU or ELU', conversion, row-major store) is cut into items: 4 per tile
// (a quad of the lane's 16 results each) and then the 2 * gs store steps of the transposition buffer.
__host__ __device__ constexpr int cd_items(int gs) { return 6 * gs; }
// Deferred epilogues: a group whose last chunk is cl may run its items inside the k steps of the next group
// (on a second accumulator set), where the matrix unit hides them.  avail = the k steps of the next group that
// may carry items: all of them inside a segment; across a segment boundary only those before the next
// segment starts to read this group's results (k step 2 * tile0).  0 = the epilogue runs at once: the head
// (its loss needs the whole workgroup), the last group of the plan, and groups with too few k steps after them.
__host__ __device__ constexpr int cd_defer_avail(const ChainDims& D, int cl, bool enabled) {
  if (!enabled || cl < 0 || cl + 1 >= cd_nchunks(D)) return 0;
  const ChunkInfo ci = cd_chunk(D, cl);
  if (!ci.last || ci.seg == D.nl - 1) return 0;
  const ChunkInfo nx = cd_chunk(D, cl + 1);
  int avail = nx.seg_nks;
  if (nx.seg != ci.seg && 2 * ci.tile0 < avail) avail = 2 * ci.tile0;
  return avail >= 4 ? avail : 0;
}

// number of k steps in the chunks before chunk c (the operand ring below is indexed by it)
__host__ __device__ constexpr int cd_ksteps_before(const ChainDims& D, int c) {
  int n = 0;
  for (int i = 0; i < c; ++i) n += cd_chunk(D, i).nks;
  return n;
}

// ---------------------------------------------------------------------------------------------------------
struct ChainArgs {
  const char* wstream[2];                          // chain stream of the policy / value net
  const float* bias[2][GMI_MAX_HIDDEN + 1];        // fp32 [out_pad] per layer
  uint16_t* x0;                                    // [rows, d[0]] bf16: the minibatch's observations, written here for
                                                   // the weight-gradient kernel (by the policy net's workgroups)
  uint16_t* h[2][GMI_MAX_HIDDEN + 1];              // h[net][l], l = 1 .. nl-1: input of layer l, [rows, d[l]]
  uint16_t* dz[2][GMI_MAX_HIDDEN + 1];             // dz[net][l], l = 0 .. nl-1: gradient at layer l's output, [rows, d[l+1]]
  const float* log_std;
  // the experience buffer the minibatch is drawn from: sample idx[r] lives at slot
  // (idx[r] / n_envs) * ld_envs + idx[r] % n_envs of its time-major arrays
  const int32_t* idx;                              // [rows]
  const float *b_obs, *b_act, *b_logp, *b_adv, *b_ret;
  int n_envs, ld_envs, obs_dim;
  int x0_ready;                                    // 1: x0 already holds the gathered rows (observation rows that cannot
                                                   // be read as 16-byte pieces are gathered by gather_kernel beforehand);
                                                   // 2: the rows are gathered from x16
  const uint16_t* x16;                             // bf16 copy of all observations, [sample index][d[0]] (x0_ready == 2)
  int rows, act_dim;
  float clip, c_v;
  float* stat_part;                                // [tiles][kStatStride + act_dim]
  // inference (the forward-only row-tile kernel, tile_kernel.h): workgroup row y works on net net0 + y; results of the heads
  int net0;
  float* mu_out;                                   // [rows, act_dim] policy means
  float* val_out;                                  // [rows] values
  uint16_t* x0b;                                   // row-tile kernel: x0 in its block layout (tile_kernel.h)
};

constexpr int kSlotBytes = 16 * 1024;              // one chunk
constexpr int kSlots = 3;                          // chunk c lives in slot c % 3: while chunk c is multiplied, chunk c+1 is
                                                   // already visible (its first operands are prefetched) and c+2 lands
constexpr int kScrStride = 272;                    // bytes per row of a wave's transposition buffer (256 + 16)
constexpr int kScrBytes = 32 * kScrStride;

// A compile-time description of one model shape: NW waves per workgroup, DEPTH chunks of weights in flight,
// GMAX tiles in the largest group, DEFER = 1 if epilogues run inside the next group's products, HFETCH and MODE (see
// below), then the padded widths d[0..nl].
template <int NW_, int DEPTH_, int GMAX_, int DEFER_, int HFETCH_, int MODE_, int... DIMS>
struct ChainShape {
  static constexpr int NW = NW_, NT = NW_ * 64, DEPTH = DEPTH_, GMAX = GMAX_;
  static constexpr bool DEFER = DEFER_ != 0;
  static constexpr bool X16 = MODE_ == 2;     // trainer that can also gather its rows from the bf16 copy of all observations
                                              // (x0_ready == 2; only the shapes of models with unaligned observation rows
                                              // carry that code: its mere presence cost the 400-wide shapes 8 %)
  static_assert(MODE_ == 0 || MODE_ == 2, "MODE: 0 trainer, 2 trainer with the bf16-copy gather");
  static constexpr int HFETCH = HFETCH_;      // without DEFER: a group fetches its stored activations this many chunks before its end
  static_assert(GMAX_ == 4 || GMAX_ == 2, "groups of at most 4 or 2 tiles");
  static constexpr int NL = (int)sizeof...(DIMS) - 1;
  static constexpr int LPT = (16 * 64 + NT - 1) / NT;      // 16-byte pieces of a chunk per thread
  static constexpr ChainDims dims() { return ChainDims{NL, GMAX_, {DIMS...}}; }
  static constexpr int maxks() { return cd_maxdim(dims()) / 16; }
  static constexpr int nch() { return cd_nchunks(dims()); }
  static constexpr int items(int gs) { return cd_items(gs); }
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
  static constexpr size_t lds_bytes() {
    return kSlots * (size_t)kSlotBytes + (size_t)NW * kScrBytes + (size_t)bias_total() * 4 + (size_t)(NW * 40 + 64) * 4;
  }
};

template <class S>
struct Ctx {
  uint4 xa[S::maxks()], xb[S::maxks()];      // activation operands of the current layer: in / out (ping-pong by segment)
  floatx16 acc[2][4];                    // two accumulator sets: groups alternate (see cd_defer_avail)
  uint4 stage[S::DEPTH][S::LPT];         // weight chunks in flight
  bf16x8 wq[3][4];                       // weight operands of k steps g, g+1, g+2 (ring indexed by g % 3)
  uint4 ht[8];                           // stored activations of the group (input-gradient segments)
  uint4 ipre[2];                         // LDS operand of the epilogue item in work / of the next one
  int64_t slot;                          // this lane's sample in the experience buffer
  float l_act[16], l_lo, l_ad, l_rt;     // this lane's loss inputs (fetched at kernel start): actions of its 16
                                         // features, old log-prob, advantage, return
  const uint4* wsrc;                     // this net's stream
  char* lds;                             // workgroup LDS base
  char* scr;                             // this wave's transposition buffer
  const float* s_bias;
  float* s_red;                          // [NW][40]
  int tid, lane, wave, s, hh;            // s = lane % 32 (sample in the wave's tile), hh = lane / 32
  int row0, net;
};

// Every chunk moves as a full 16 KiB: pieces past a short chunk's end belong to the next chunk (or to the
// stream's tail padding) and land in slot space nobody reads.  No branch surrounds a load or store: the
// memory-counter bookkeeping of the compiler then waits for exactly the chunk that is needed (with a branch it
// waited for almost every load in flight).
template <class S, int C>
__device__ __forceinline__ void issue_chunk(Ctx<S>& c) {
  if constexpr (C < S::nch()) {
    constexpr ChunkInfo ci = cd_chunk(S::dims(), C);
#pragma unroll
    for (int i = 0; i < S::LPT; ++i) c.stage[C % S::DEPTH][i] = c.wsrc[(int64_t)ci.blk_off * 64 + c.tid + i * S::NT];
  }
}
template <class S, int C>
__device__ __forceinline__ void land_chunk(Ctx<S>& c) {
  if constexpr (C < S::nch()) {
    uint4* slot = reinterpret_cast<uint4*>(c.lds + (C % kSlots) * kSlotBytes);
#pragma unroll
    for (int i = 0; i < S::LPT; ++i) slot[c.tid + i * S::NT] = c.stage[C % S::DEPTH][i];
  }
}

// Row-major store of a group's packed results: the wave's transposition buffer holds [32 samples][GS*32
// features] bf16; rows leave as 64 * GS byte pieces.
template <int GS>
__device__ __forceinline__ void scr_to_global(const char* scr, int lane, uint16_t* dst, int ld, int col0, int row0,
                                              int rows) {
  constexpr int LPR = 4 * GS, RPI = 64 / LPR;    // lanes per row, rows per instruction
#pragma unroll
  for (int it = 0; it < 32 / RPI; ++it) {
    const int r = it * RPI + lane / LPR, ch = lane % LPR;
    const uint4 v = *reinterpret_cast<const uint4*>(scr + r * kScrStride + ch * 16);
    *reinterpret_cast<uint4*>(dst + (int64_t)(row0 + r) * ld + col0 + ch * 8) = v;     // arrays hold whole tiles
  }
}
template <int GS>
__device__ __forceinline__ void global_to_regs(uint4* ht, int lane, const uint16_t* src, int ld, int col0, int row0,
                                               int rows) {
  constexpr int LPR = 4 * GS, RPI = 64 / LPR;
#pragma unroll
  for (int it = 0; it < 32 / RPI; ++it) {
    const int r = it * RPI + lane / LPR, ch = lane % LPR;
    ht[it] = *reinterpret_cast<const uint4*>(src + (int64_t)(row0 + r) * ld + col0 + ch * 8);
  }
}
template <int GS>
__device__ __forceinline__ void regs_to_scr(const uint4* ht, int lane, char* scr) {
  constexpr int LPR = 4 * GS, RPI = 64 / LPR;
#pragma unroll
  for (int it = 0; it < 32 / RPI; ++it) {
    const int r = it * RPI + lane / LPR, ch = lane % LPR;
    *reinterpret_cast<uint4*>(scr + r * kScrStride + ch * 16) = ht[it];
  }
}

__device__ __forceinline__ float wave_sum64(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Loss on the wave's 32 samples, from the head's accumulators (lane = sample s, half hh; register i = feature
// 8 (i / 4) + 4 hh + i % 4).  Leaves the head gradient as the first two k steps of `xo` and in the wave's
// transposition buffer, and per-wave partial sums in s_red[wave][0..2] (policy: surrogate, kl, clipped;
// value: squared error in [0]) and s_red[wave][8 + f] (log_std gradient partials).
// This lane's loss inputs, fetched one layer before the head needs them (unconditional loads: rows and features
// past the end read a valid neighbour, their results are dropped).
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

template <class S>
__device__ __forceinline__ void loss_epilogue(Ctx<S>& c, const ChainArgs& a, const floatx16& acc, uint4* xo) {
  constexpr int HB = S::bias_off(S::NL - 1);
  const int A = a.act_dim;
  const int row = c.row0 + c.s;
  const bool ok = row < a.rows;
  const float inv_m = 1.0f / (float)a.rows;
  float d[16];
  float* red = c.s_red + c.wave * 40;
  if (c.net == 0) {
    // s_ls[f] = log_std, s_ls[32 + f] = exp(-log_std) (0 for f >= A), staged at kernel start
    const float* s_ls = c.s_red + S::NW * 40;
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
    // log_std gradient partials g_lp (z^2 - 1): transposed through the wave's LDS buffer as [feature][sample]
    // fp32, then lane f < 32 sums feature f's 32 samples in a fixed order
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
  xo[0] = make_uint4(w[0], w[1], w[2], w[3]);
  xo[1] = make_uint4(w[4], w[5], w[6], w[7]);
#pragma unroll
  for (int q = 0; q < 4; ++q)
    *reinterpret_cast<uint2*>(c.scr + c.s * kScrStride + (8 * q + 4 * c.hh) * 2) = make_uint2(w[2 * q], w[2 * q + 1]);
  scr_to_global<1>(c.scr, c.lane, a.dz[c.net][S::NL - 1], 32, 0, c.row0, a.rows);
  // workgroup sums -> this tile's row of the statistics partials
  __syncthreads();
  float* out = a.stat_part + (int64_t)blockIdx.x * (gmi::kStatStride + A);
  if (c.net == 0) {
    if (c.tid < 3) {
      float v = 0.f;
      for (int wv = 0; wv < S::NW; ++wv) v += c.s_red[wv * 40 + c.tid];
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
      for (int wv = 0; wv < S::NW; ++wv) v += c.s_red[wv * 40 + 8 + j];
      out[gmi::kStatStride + j] = v;
    }
  } else if (c.tid == 0) {
    float v = 0.f;
    for (int wv = 0; wv < S::NW; ++wv) v += c.s_red[wv * 40];
    out[1] = v;
  }
}

template <class S, int C, int K, int RING>
__device__ __forceinline__ void fetch_kstep(Ctx<S>& c) {
  if constexpr (C < S::nch()) {
    constexpr ChunkInfo ci = cd_chunk(S::dims(), C);
    if constexpr (K >= ci.nks) {
      fetch_kstep<S, C + 1, K - ci.nks, RING>(c);
    } else {
      const char* slot = c.lds + (C % kSlots) * kSlotBytes + c.lane * 16;
#pragma unroll
      for (int t = 0; t < ci.gs; ++t)
        c.wq[RING][t] = *reinterpret_cast<const bf16x8*>(slot + (K * ci.gs + t) * 1024);
    }
  }
}

// Item I of the epilogue of the group whose last chunk is PC (cd_items): quads first, then the store steps.
// Each item is cut in two: its LDS read into c.ipre[I % 2] (item_load) and the rest (item_compute), so that the
// read of item I + 1 is in flight while item I is worked on.
template <class S, int PC, int I>
__device__ __forceinline__ void item_load(Ctx<S>& c) {
  constexpr ChainDims D = S::dims();
  constexpr ChunkInfo pi = cd_chunk(D, PC);
  constexpr int NL = S::NL, GS = pi.gs;
  constexpr bool bwd = pi.seg >= NL;
  if constexpr (I < 4 * GS) {
    constexpr int t = I / 4, q = I % 4;
    if constexpr (bwd) {
      const uint2 hv = *reinterpret_cast<const uint2*>(c.scr + c.s * kScrStride + (32 * t + 8 * q + 4 * c.hh) * 2);
      c.ipre[I % 2].x = hv.x; c.ipre[I % 2].y = hv.y;
    } else {
      constexpr int boff = S::bias_off(cd_layer(D, pi.seg));
      c.ipre[I % 2] = *reinterpret_cast<const uint4*>(c.s_bias + boff + 32 * (pi.tile0 + t) + 8 * q + 4 * c.hh);
    }
  } else if constexpr (I < S::items(GS)) {
    constexpr int LPR = 4 * GS, RPI = 64 / LPR, it = I - 4 * GS;
    const int r = it * RPI + c.lane / LPR, ch = c.lane % LPR;
    c.ipre[I % 2] = *reinterpret_cast<const uint4*>(c.scr + r * kScrStride + ch * 16);
  }
}
template <class S, int PC, int I>
__device__ __forceinline__ void item_compute(Ctx<S>& c, const ChainArgs& a) {
  constexpr ChainDims D = S::dims();
  constexpr ChunkInfo pi = cd_chunk(D, PC);
  constexpr int NL = S::NL, GS = pi.gs;
  constexpr bool bwd = pi.seg >= NL;
  constexpr int layer = cd_layer(D, pi.seg);
  uint4* xo = (pi.seg & 1) ? c.xa : c.xb;
  const uint4 pre = c.ipre[I % 2];
  if constexpr (I < 4 * GS) {
    constexpr int t = I / 4, q = I % 4;
    const floatx16& acc = c.acc[pi.gord & 1][t];
    float v0 = acc[4 * q + 0], v1 = acc[4 * q + 1], v2 = acc[4 * q + 2], v3 = acc[4 * q + 3];
    if constexpr (bwd) {
      // times ELU'(z) through the stored output h = ELU(z): 1 if h > 0 else h + 1
      const float h0 = bf16_lo(pre.x), h1 = bf16_hi(pre.x), h2 = bf16_lo(pre.y), h3 = bf16_hi(pre.y);
      v0 *= elu_grad_f(h0); v1 *= elu_grad_f(h1);
      v2 *= elu_grad_f(h2); v3 *= elu_grad_f(h3);
    } else {
      v0 = elu_f(v0 + __uint_as_float(pre.x)); v1 = elu_f(v1 + __uint_as_float(pre.y));
      v2 = elu_f(v2 + __uint_as_float(pre.z)); v3 = elu_f(v3 + __uint_as_float(pre.w));
    }
    const uint32_t w0 = pack_bf16(v0, v1), w1 = pack_bf16(v2, v3);
    *reinterpret_cast<uint2*>(c.scr + c.s * kScrStride + (32 * t + 8 * q + 4 * c.hh) * 2) = make_uint2(w0, w1);
    uint4& x = xo[2 * (pi.tile0 + t) + q / 2];
    if constexpr (q % 2 == 0) { x.x = w0; x.y = w1; } else { x.z = w0; x.w = w1; }
  } else {
    constexpr int LPR = 4 * GS, RPI = 64 / LPR, it = I - 4 * GS;
    const int r = it * RPI + c.lane / LPR, ch = c.lane % LPR;
    uint16_t* dst = bwd ? a.dz[c.net][layer - 1] : a.h[c.net][layer + 1];
    constexpr int ld = bwd ? D.d[layer] : D.d[layer + 1];
    *reinterpret_cast<uint4*>(dst + (int64_t)(c.row0 + r) * ld + 32 * pi.tile0 + ch * 8) = pre;    // arrays hold whole tiles
  }
}
// Item I with the read of item I + 1 issued ahead of it -- except the first store step's, which reads what the
// last quad writes.
template <class S, int PC, int I>
__device__ __forceinline__ void item_step(Ctx<S>& c, const ChainArgs& a) {
  constexpr int NQ = 4 * cd_chunk(S::dims(), PC).gs;
  if constexpr (I + 1 != NQ) item_load<S, PC, I + 1>(c);
  item_compute<S, PC, I>(c, a);
  if constexpr (I + 1 == NQ) item_load<S, PC, I + 1>(c);
}
// Items [I, END) one after the other, each in a scheduling region of its own (so that the read of the next
// item stays ahead of the work on this one).  The read of item I must have been issued.
template <class S, int PC, int I, int END>
__device__ __forceinline__ void epilogue_items(Ctx<S>& c, const ChainArgs& a) {
  if constexpr (I < END) {
    item_step<S, PC, I>(c, a);
    __builtin_amdgcn_sched_barrier(0);
    epilogue_items<S, PC, I + 1, END>(c, a);
  }
}

// One k step: its GS products, with the previous group's deferred items between them -- a wave issues in order,
// so an item placed behind a block of products would start only when the last of them has entered the matrix
// unit.  Item i of the slice [I0, I1) follows product i.
template <class S, int C, int K, int T, int I0, int I1>
__device__ __forceinline__ void kstep_products(Ctx<S>& c, const ChainArgs& a, const bf16x8& xk) {
  constexpr ChainDims D = S::dims();
  constexpr ChunkInfo ci = cd_chunk(D, C);
  if constexpr (T < ci.gs || I0 + T < I1) {
    constexpr int g = cd_ksteps_before(D, C) + K;
    if constexpr (T < ci.gs)
      c.acc[ci.gord & 1][T] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c.wq[g % 3][T], xk, c.acc[ci.gord & 1][T], 0, 0, 0);
    if constexpr (I0 + T < I1) {
      item_step<S, ci.prev_last, I0 + T>(c, a);
    }
    // nothing moves across this point: the schedule keeps the LDS reads of k step g+2 ahead of the products of
    // k step g (left to itself the scheduler sinks every read to just before its use, and with one wave per
    // SIMD each product then waits a full LDS round trip)
    if constexpr (I0 + T < I1 || T + 1 >= ci.gs) __builtin_amdgcn_sched_barrier(0);
    kstep_products<S, C, K, T + 1, I0, I1>(c, a, xk);
  }
}

template <class S, int C, int K>
__device__ __forceinline__ void compute_ksteps(Ctx<S>& c, const ChainArgs& a, const uint4* xi) {
  constexpr ChainDims D = S::dims();
  constexpr ChunkInfo ci = cd_chunk(D, C);
  if constexpr (K < ci.nks) {
    constexpr int g = cd_ksteps_before(D, C) + K;
    fetch_kstep<S, C, K + 2, (g + 2) % 3>(c);
    const bf16x8 xk = __builtin_bit_cast(bf16x8, xi[ci.ks0 + K]);
    // the slice of the previous group's deferred epilogue that this k step carries
    constexpr int avail = cd_defer_avail(D, ci.prev_last, S::DEFER);
    if constexpr (avail > 0) {
      constexpr int N = S::items(cd_chunk(D, ci.prev_last).gs), ipk = (N + avail - 1) / avail;
      constexpr int kg = ci.ks0 + K, i0 = kg * ipk < N ? kg * ipk : N, i1 = (i0 + ipk) < N ? (i0 + ipk) : N;
      kstep_products<S, C, K, 0, i0, i1>(c, a, xk);
    } else {
      kstep_products<S, C, K, 0, 0, 0>(c, a, xk);
    }
    compute_ksteps<S, C, K + 1>(c, a, xi);
  }
}

// The stored activations that the input-gradient group after chunk C multiplies its results with (ELU'), fetched
// one group ahead: from the head's chunk for the first such group, then as soon as a group has handed its own
// to the transposition buffer.  (A group's k steps are over long before a fetch issued inside them returns.)
template <class S, int C>
__device__ __forceinline__ void fetch_next_h(Ctx<S>& c, const ChainArgs& a) {
  constexpr ChainDims D = S::dims();
  if constexpr (S::DEFER && C + 1 < S::nch()) {       // without deferred epilogues a group fetches its own, in its last chunk
    constexpr ChunkInfo nx = cd_chunk(D, C + 1);
    static_assert(nx.first, "called at the end of a group");
    if constexpr (nx.seg >= S::NL) {
      constexpr int layer = cd_layer(D, nx.seg);
      global_to_regs<nx.gs>(c.ht, c.lane, a.h[c.net][layer], D.d[layer], 32 * nx.tile0, c.row0, a.rows);
    }
  }
}

template <class S, int C>
__device__ __forceinline__ void chain_step(Ctx<S>& c, const ChainArgs& a) {
  constexpr ChainDims D = S::dims();
  constexpr ChunkInfo ci = cd_chunk(D, C);
  constexpr int seg = ci.seg, NL = S::NL;
  constexpr bool bwd = seg >= NL;
  constexpr int layer = cd_layer(D, seg);
  constexpr int GS = ci.gs;
  // even segments read xa and write xb, odd ones the other way round
  uint4* xi = (seg & 1) ? c.xb : c.xa;
  uint4* xo = (seg & 1) ? c.xa : c.xb;

  issue_chunk<S, C + 1 + S::DEPTH>(c);
  if constexpr (seg == NL - 2 && ci.gi == 0 && ci.first) fetch_loss_inputs<S>(c, a);

  // stored activations of this group's features, for ELU': fetched HFETCH chunks before the group's end
  if constexpr (!S::DEFER && bwd && (ci.last_in == (S::HFETCH < ci.group_chunks ? S::HFETCH : ci.group_chunks) - 1))
    global_to_regs<GS>(c.ht, c.lane, a.h[c.net][layer], D.d[layer], 32 * ci.tile0, c.row0, a.rows);

  if constexpr (ci.first) {
#pragma unroll
    for (int t = 0; t < GS; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) c.acc[ci.gord & 1][t][v] = 0.f;
  }
  compute_ksteps<S, C, 0>(c, a, xi);

  if constexpr (ci.last) {
    if constexpr (!bwd && layer == NL - 1) {
      static_assert(GS == 1, "the head is one 32-wide tile");
      fetch_next_h<S, C>(c, a);
      loss_epilogue<S>(c, a, c.acc[ci.gord & 1][0], xo);
    } else {
      // the stored activations go to the transposition buffer now (the previous group's items are done with it),
      // the rest of the epilogue either now or inside the next group's k steps
      if constexpr (bwd) {
        regs_to_scr<GS>(c.ht, c.lane, c.scr);
        fetch_next_h<S, C>(c, a);
      }
      item_load<S, C, 0>(c);
      if constexpr (cd_defer_avail(D, C, S::DEFER) == 0) epilogue_items<S, C, 0, S::items(GS)>(c, a);
    }
  }

  if constexpr (C + 1 < S::nch()) {
    land_chunk<S, C + 2>(c);
    __syncthreads();
    chain_step<S, C + 1>(c, a);
  }
}

template <class S>
__global__ __launch_bounds__(S::NW * 64) void train_chain_kernel(ChainArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  constexpr ChainDims D = S::dims();
  Ctx<S> c;
  c.tid = threadIdx.x;
  c.lane = c.tid & 63;
  c.wave = __builtin_amdgcn_readfirstlane(c.tid >> 6);
  c.s = c.lane & 31;
  c.hh = c.lane >> 5;
  c.net = blockIdx.y;
  c.row0 = (blockIdx.x * S::NW + c.wave) * 32;
  c.lds = reinterpret_cast<char*>(smem_raw);
  c.scr = c.lds + kSlots * kSlotBytes + c.wave * kScrBytes;
  float* s_bias = reinterpret_cast<float*>(c.lds + kSlots * kSlotBytes + S::NW * kScrBytes);
  c.s_bias = s_bias;
  c.s_red = s_bias + S::bias_total();
  c.wsrc = reinterpret_cast<const uint4*>(a.wstream[c.net]);

  // weights first (the longest latency), then biases and the input rows.  Chunk c travels in register set
  // c % DEPTH: chunk 0 is landed at once, which frees its set for chunk DEPTH.
  static_assert(S::DEPTH >= 1 && S::DEPTH <= 4, "1..4 chunks in flight");
  issue_chunk<S, 0>(c);
  land_chunk<S, 0>(c);
  issue_chunk<S, 1>(c);
  if constexpr (S::DEPTH > 1) issue_chunk<S, 2>(c);
  if constexpr (S::DEPTH > 2) issue_chunk<S, 3>(c);
  if constexpr (S::DEPTH > 3) issue_chunk<S, 4>(c);
  {
    int off = 0;
#pragma unroll
    for (int l = 0; l < S::NL; ++l) {
      for (int f = c.tid; f < D.d[l + 1]; f += S::NT) s_bias[off + f] = a.bias[c.net][l][f];
      off += D.d[l + 1];
    }
  }
  for (int i = c.tid; i < S::NW * 40; i += S::NT) c.s_red[i] = 0.f;
  if (c.tid < 32) {                      // per-feature constants of the Gaussian log-prob (policy net)
    const int fc = c.tid < a.act_dim ? c.tid : a.act_dim - 1;
    const float ls = a.log_std[fc];
    c.s_red[S::NW * 40 + c.tid] = ls;
    c.s_red[S::NW * 40 + 32 + c.tid] = c.tid < a.act_dim ? expf(-ls) : 0.f;
  }
  {
    // The gather: this lane's sample (rows past the batch take the last sample; their results are dropped) and
    // the first layer's operand in natural order, lane (s, hh) holding features 16 ks + 8 hh .. + 7 of its
    // observation, converted to bf16 and zero padded.  The policy net's workgroups also leave the converted rows
    // in x0 for the weight-gradient kernel.  All loads unconditional (clamped addresses, selected values).
    const int row = c.row0 + c.s;
    const int rc = row < a.rows ? row : a.rows - 1;
    const int sm = a.idx ? a.idx[rc] : rc;               // no index: rows in order
    c.slot = (int64_t)(sm / a.n_envs) * a.ld_envs + (sm % a.n_envs);
    const float* orow = a.b_obs + c.slot * a.obs_dim;
    const int O = a.obs_dim;
    uint16_t* xw = a.x0 + (int64_t)row * D.d[0] + 8 * c.hh;
    if (a.x0_ready == 1) {                             // wave-uniform
#pragma unroll
      for (int ks = 0; ks < D.d[0] / 16; ++ks) c.xa[ks] = *reinterpret_cast<const uint4*>(xw + 16 * ks);
    } else if (S::X16 && a.x0_ready == 2) {
      // the gather from the bf16 copy of all observations (rows of d[0] elements by sample index)
      if constexpr (S::X16) {
        const uint16_t* xs = a.x16 + (int64_t)sm * D.d[0] + 8 * c.hh;
#pragma unroll
        for (int ks = 0; ks < D.d[0] / 16; ++ks) {
          c.xa[ks] = *reinterpret_cast<const uint4*>(xs + 16 * ks);
          if (c.net == 0) *reinterpret_cast<uint4*>(xw + 16 * ks) = c.xa[ks];
        }
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < D.d[0] / 16; ++ks) {
        const int f0 = 16 * ks + 8 * c.hh;
        float v[8];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int f = f0 + 4 * q;                    // O % 4 == 0: a piece is inside the row or past it
          const float4 t = *reinterpret_cast<const float4*>(orow + (f < O ? f : O - 4));
          v[4 * q + 0] = f < O ? t.x : 0.f; v[4 * q + 1] = f < O ? t.y : 0.f;
          v[4 * q + 2] = f < O ? t.z : 0.f; v[4 * q + 3] = f < O ? t.w : 0.f;
        }
        c.xa[ks] = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
        if (c.net == 0) *reinterpret_cast<uint4*>(xw + 16 * ks) = c.xa[ks];      // arrays hold whole tiles
      }
    }
  }
  land_chunk<S, 1>(c);
  __syncthreads();
  fetch_kstep<S, 0, 0, 0>(c);
  fetch_kstep<S, 0, 1, 1>(c);
  chain_step<S, 0>(c, a);
}

// True if the model has exactly the padded widths of shape S.
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
  const int tiles = (rows + 32 * S::NW - 1) / (32 * S::NW);
  *tiles_out = tiles;
  if (tiles > gmi::kLossBlocksMax) return GMI_ERR_UNSUPPORTED;      // one statistics row per tile
  if (!attr) {
    GMI_HIP(hipFuncSetAttribute((const void*)train_chain_kernel<S>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr = true;
  }
  gmi::ProfScope ps(g, gmi::kClsChainTrain);
  ps.work(flops, bytes);
  ps.launch(train_chain_kernel<S>, dim3(tiles, 2), dim3(S::NT), lds, a);
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}

}  // namespace gmi_chain

namespace gmi {
// One function per compiled shape (chain_p<k>.hip): launches the kernel if the model has exactly that shape,
// GMI_ERR_UNSUPPORTED otherwise.  rows == 0 only asks whether the shape matches (*tiles_out = the
// shape's largest group, which the layout of the weight stream depends on, plus 256 for a trainer shape
// with the bf16-copy gather).
constexpr int kChainParts = 4;
#define GMI_CHAIN_PART_DECL(k)                                                                              \
  int launch_chain_part##k(gmi_instance* g, const ModelLayout& L, const gmi_chain::ChainArgs& a, int rows, \
                           int* tiles_out, double flops, double bytes)
GMI_CHAIN_PART_DECL(0); GMI_CHAIN_PART_DECL(1); GMI_CHAIN_PART_DECL(2); GMI_CHAIN_PART_DECL(3);
// Defines part k for shape S.
#define GMI_CHAIN_PART_DEFINE(k, ...)                                                             \
  GMI_CHAIN_PART_DECL(k) {                                                                        \
    using S = gmi_chain::ChainShape<__VA_ARGS__>;                                                 \
    if (!gmi_chain::shape_matches<S>(L)) return GMI_ERR_UNSUPPORTED;                              \
    if (rows == 0) { *tiles_out = S::GMAX | (S::X16 ? 256 : 0); return GMI_OK; }                  \
    return gmi_chain::launch_shape<S>(g, a, rows, tiles_out, flops, bytes);                       \
  }
}  // namespace gmi
