// Host side of the register-chained trainer kernel (chain_kernel.h): the weight stream in the shadow, its packing
// kernel and the launch.  The kernel itself is compiled once per model shape in chain_p<k>.hip.
#include <stdlib.h>

#include "tile_kernel.h"

namespace {
using namespace gmi_chain;

// ---------------------------------------------------------------------------------------------------------
// Packing kernel: builds one net's chain stream from the row-major bf16 shadows.  One thread per lane of a
// block (16 bytes).  Lane L of block (tile ft, k step ks) of a segment holds, for output row m = 32 ft + L % 32,
// the 8 contraction indices 16 ks + p(L / 32, j), j = 0..7: p(h, j) = 8 h + j for the first forward layer
// (whose input is loaded from memory in natural order) and p(h, j) = 8 (j / 4) + 4 h + j % 4 for every other
// segment (the order in which the matrix instruction leaves a lane's 8 results of a k step).
struct PackSeg {
  int blk_start;          // first block of the segment in the stream
  int K, F;               // padded contraction / output widths
  int natural;            // 1: first forward layer
  int64_t src;            // byte offset into the shadow of the source matrix, row-major [F, K] bf16
};
struct PackTable {
  int n;
  int total_blocks;
  int gmax;               // tiles in the largest group (4 or 2)
  PackSeg s[2 * (GMI_MAX_HIDDEN + 1)];
};

__global__ __launch_bounds__(256) void chain_pack_kernel(PackTable t0, PackTable t1, const char* __restrict__ shadow,
                                                         char* __restrict__ out0, char* __restrict__ out1) {
  const PackTable& tab = blockIdx.y == 0 ? t0 : t1;
  char* out = blockIdx.y == 0 ? out0 : out1;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int blk = (int)(gid >> 6), lane = (int)(gid & 63);
  if (blk >= tab.total_blocks) return;
  int si = 0;
  while (si + 1 < tab.n && blk >= tab.s[si + 1].blk_start) ++si;
  const PackSeg& S = tab.s[si];
  const int nft = S.F >> 5, nks = S.K >> 4;
  int lb = blk - S.blk_start;
  // locate the group: full groups of gmax tiles first, then (2), then (1)
  const int gm = tab.gmax, full = nft / gm;
  int tile0, gs;
  if (lb < full * gm * nks) {
    const int gi = lb / (gm * nks);
    tile0 = gm * gi; gs = gm; lb -= gi * gm * nks;
  } else {
    lb -= full * gm * nks;
    tile0 = gm * full;
    if ((nft % gm) >= 2) {
      if (lb < 2 * nks) { gs = 2; }
      else { lb -= 2 * nks; tile0 += 2; gs = 1; }
    } else {
      gs = 1;
    }
  }
  const int ks = lb / gs, t = lb - ks * gs;
  const int m = 32 * (tile0 + t) + (lane & 31), h = lane >> 5;
  const uint16_t* row = reinterpret_cast<const uint16_t*>(shadow + S.src) + (int64_t)m * S.K + 16 * ks;
  uint16_t e[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) e[j] = row[S.natural ? 8 * h + j : 8 * (j >> 2) + 4 * h + (j & 3)];
  uint4 v;
  v.x = e[0] | ((uint32_t)e[1] << 16); v.y = e[2] | ((uint32_t)e[3] << 16);
  v.z = e[4] | ((uint32_t)e[5] << 16); v.w = e[6] | ((uint32_t)e[7] << 16);
  reinterpret_cast<uint4*>(out)[(int64_t)blk * 64 + lane] = v;
}

ChainDims dims_of(const ModelLayout& L, int gmax = 4) {
  ChainDims D;
  D.nl = L.n_layers;
  D.gmax = gmax;
  for (int l = 0; l < L.n_layers; ++l) { D.d[l] = L.net[0][l].in_pad; D.d[l + 1] = L.net[0][l].out_pad; }
  return D;
}

typedef int (*part_fn)(gmi_instance*, const ModelLayout&, const ChainArgs&, int, int*, double, double);
const part_fn kParts[gmi::kChainParts] = {gmi::launch_chain_part0, gmi::launch_chain_part1, gmi::launch_chain_part2,
                                          gmi::launch_chain_part3};
// The row-tile kernel's shapes (tile_kernel.h) come first: a model shape compiled for both takes that one.
const part_fn kTileFns[gmi::kTileParts] = {gmi::launch_tile_part0, gmi::launch_tile_part1};
const part_fn kTileFwdFns[gmi::kTileFwdParts] = {gmi::launch_tile_fwd_part0, gmi::launch_tile_fwd_part1};

// What the trainer kernel compiled for this model's shape answers to the probe: its largest group, plus 256 if it
// can gather its rows from the bf16 copy of all observations; 0 if there is none.
int compiled_probe(const ModelLayout& L) {
  ChainArgs none = {};
  int v = 0;
  for (int p = 0; p < gmi::kTileParts; ++p)
    if (kTileFns[p](nullptr, L, none, 0, &v, 0.0, 0.0) == GMI_OK) return v;
  for (int p = 0; p < gmi::kChainParts; ++p)
    if (kParts[p](nullptr, L, none, 0, &v, 0.0, 0.0) == GMI_OK) return v;
  return 0;
}
int compiled_gmax(const ModelLayout& L) { return compiled_probe(L) & 255; }
bool compiled_x16(const ModelLayout& L) { return (compiled_probe(L) & 256) != 0; }

}  // namespace


namespace gmi {
using namespace gmi_chain;

// Bytes of one net's chain stream (0 if the two nets' padded widths differ, which only a policy head wider
// than 32 outputs can cause: such models have no chain stream).
int64_t chain_stream_bytes(const ModelLayout& L) {
  if (L.dtype != GMI_DTYPE_BF16) return 0;
  for (int l = 0; l < L.n_layers; ++l)
    if (L.net[0][l].in_pad != L.net[1][l].in_pad || L.net[0][l].out_pad != L.net[1][l].out_pad) return 0;
  return (int64_t)cd_nblocks(dims_of(L)) * 1024 + kSlotBytes;      // tail padding: chunks are fetched as full 16 KiB
}

// Rebuilds both nets' chain streams from the row-major shadows (W for the forward segments, W^T for the
// input-gradient segments).
int launch_chain_pack(gmi_instance* g, gmi_model* m) {
  const ModelLayout& L = m->L;
  if (L.sh_chain_bytes == 0) return GMI_OK;
  const int gmax = compiled_gmax(L);
  if (gmax == 0) return GMI_OK;                        // no chained kernel for this shape: nobody reads the stream
  const ChainDims D = dims_of(L, gmax);
  PackTable t[2];
  for (int net = 0; net < 2; ++net) {
    t[net].n = cd_nseg(D);
    t[net].gmax = gmax;
    int blk = 0;
    for (int s = 0; s < cd_nseg(D); ++s) {
      PackSeg& ps = t[net].s[s];
      const int l = cd_layer(D, s);
      ps.blk_start = blk;
      ps.K = cd_K(D, s);
      ps.F = cd_F(D, s);
      ps.natural = s == 0 ? 1 : 0;
      ps.src = s < D.nl ? L.net[net][l].sh_w : L.net[net][l].sh_wt;
      blk += cd_seg_blocks(D, s);
    }
    t[net].total_blocks = blk;
  }
  const int64_t threads = (int64_t)t[0].total_blocks * 64;
  ProfScope ps(g, kClsShadowTranspose);
  ps.launch(chain_pack_kernel, dim3((unsigned)((threads + 255) / 256), 2), dim3(256), 0, t[0], t[1], (const char*)m->shadow,
            m->shadow + L.sh_chain[0], m->shadow + L.sh_chain[1]);
  GMI_LAUNCH_CHECK();
  return GMI_OK;
}

void fill_chain_emit(const ModelLayout& L, ChainEmit* ce) {
  ce->gmax = 0;
  ce->n_layers = L.n_layers;
  if (L.sh_chain_bytes == 0) return;
  const int gmax = compiled_gmax(L);
  if (gmax == 0) return;
  const ChainDims D = dims_of(L, gmax);
  ce->gmax = gmax;
  for (int net = 0; net < 2; ++net) {
    ce->out[net] = L.sh_chain[net];
    for (int l = 0; l < L.n_layers; ++l) ce->l[net * L.n_layers + l] = ChainEmitLayer{0, -1, l == 0 ? 1 : 0};
    int blk = 0;
    for (int s = 0; s < cd_nseg(D); ++s) {
      ChainEmitLayer& e = ce->l[net * L.n_layers + cd_layer(D, s)];
      if (s < D.nl) e.fwd_blk = blk; else e.bwd_blk = blk;
      blk += cd_seg_blocks(D, s);
    }
  }
}

// Gather of the minibatch rows idx[0..rows) of buffer b + forward + loss + input gradients.
// Leaves m->h, m->dz ready for the weight-gradient launch and one row of statistics / log_std partials per
// tile in m->stat_part (*n_stat_rows rows, the layout of the loss kernel's per-workgroup rows).  GMI_ERR_UNSUPPORTED (no message) if no kernel is compiled for this shape.
int prepare_obs16(gmi_instance* g, gmi_model* m, gmi_buffer* b, bool* ready) {
  const ModelLayout& L = m->L;
  *ready = false;
  if (!b->obs16 || g->fusion < 1 || L.dtype != GMI_DTYPE_BF16 || L.sh_chain_bytes == 0 || L.act_dim > 32 ||
      !compiled_x16(L))
    return GMI_OK;
  const int64_t B = (int64_t)b->d.horizon * b->d.n_envs;
  const int rc = launch_gather_to(g, m, b->d.obs, b->d.n_envs, b->d.ld_envs, nullptr, (int)B, nullptr, b->obs16);
  if (rc == GMI_OK) *ready = true;
  return rc;
}

int launch_train_chain(gmi_instance* g, gmi_model* m, gmi_buffer* b, const gmi_ppo_hparams* hp, const int32_t* idx, int rows,
                       int* n_stat_rows, bool obs16_ready, bool* blocks) {
  const ModelLayout& L = m->L;
  if (L.dtype != GMI_DTYPE_BF16 || L.sh_chain_bytes == 0 || L.act_dim > 32) return GMI_ERR_UNSUPPORTED;
  ChainArgs a;
  for (int net = 0; net < 2; ++net) {
    a.wstream[net] = m->shadow + L.sh_chain[net];
    for (int l = 0; l < L.n_layers; ++l) {
      a.bias[net][l] = reinterpret_cast<const float*>(m->shadow + L.net[net][l].sh_b);
      a.h[net][l] = (uint16_t*)m->h[net][l];
      a.dz[net][l] = (uint16_t*)m->dz[net][l];
    }
  }
  a.x0 = (uint16_t*)m->x0;
  a.x0b = (uint16_t*)m->x0b;
  a.log_std = reinterpret_cast<const float*>(m->shadow + L.sh_logstd);
  a.idx = idx;
  a.b_obs = b->d.obs; a.b_act = b->d.act; a.b_logp = b->d.logp; a.b_adv = b->d.adv; a.b_ret = b->d.ret;
  a.n_envs = b->d.n_envs; a.ld_envs = b->d.ld_envs; a.obs_dim = L.obs_dim;
  a.x0_ready = (L.obs_dim % 4 == 0 && ((uintptr_t)b->d.obs & 15) == 0) ? 0 : 1;
  a.x16 = b->obs16;
  if (a.x0_ready == 1 && obs16_ready && b->obs16 && idx && compiled_x16(L)) a.x0_ready = 2;
  a.rows = rows; a.act_dim = L.act_dim;
  a.clip = hp->clip; a.c_v = hp->c_v;
  a.stat_part = m->stat_part;
  int tiles = 0, rc;
  if (rows < 1 || rows > m->max_rows) return GMI_ERR_UNSUPPORTED;      // the activation arrays hold max_rows (in whole tiles)
  // algorithmic work at the logical (unpadded) widths: forward products of every layer, input-gradient products
  // of every layer but the first; bytes: the input rows and per-sample scalars read, every hidden activation
  // written once and read once (ELU'), every layer's output gradient written once, the weights read once
  double flops = 0.0, bytes = 0.0;
  for (int net = 0; net < 2; ++net) {
    for (int l = 0; l < L.n_layers; ++l) {
      const LayerInfo& li = L.net[net][l];
      flops += 2.0 * rows * (double)li.in * li.out * (l == 0 ? 1.0 : 2.0);
      bytes += 2.0 * li.in * li.out * (l == 0 ? 1.0 : 2.0);                 // bf16 weights, forward (+ transposed)
      bytes += 2.0 * rows * li.out;                                          // gradient at the layer's output
      // fp32 observation rows read and the bf16 copy written (once), or the gathered bf16 rows read, or those read
      // from the copy of all observations and written in minibatch order
      if (l == 0) bytes += net == 0 ? (a.x0_ready == 1 ? 2.0 : (a.x0_ready == 2 ? 4.0 : 6.0)) * rows * li.in : 0.0;
      else bytes += 2.0 * 2.0 * rows * li.in;                                // hidden activation: written, read back
    }
  }
  bytes += 4.0 * rows * (L.act_dim + 3);
  if (compiled_gmax(L) == 0) return GMI_ERR_UNSUPPORTED;
  if (a.x0_ready == 1) {  // unaligned observation rows: the gather kernel converts them (a lane-wise gather of 4-byte
                          // pieces at the start of the chained kernel measured slower than the separate launch)
    rc = launch_gather(g, m, b->d.obs, b->d.n_envs, b->d.ld_envs, idx, rows, nullptr);
    if (rc != GMI_OK) return rc;
  }
  rc = GMI_ERR_UNSUPPORTED;
  *blocks = false;
  for (int p = 0; p < kTileParts && rc == GMI_ERR_UNSUPPORTED; ++p) rc = kTileFns[p](g, L, a, rows, &tiles, flops, bytes);
  if (rc == GMI_OK) *blocks = true;
  for (int p = 0; p < kChainParts && rc == GMI_ERR_UNSUPPORTED; ++p) rc = kParts[p](g, L, a, rows, &tiles, flops, bytes);
  if (rc != GMI_OK) return rc;
  *n_stat_rows = tiles;
  return GMI_OK;
}

bool forward_chain_reads_x0(const gmi_model* m, const float* obs) {
  return !(m->L.obs_dim % 4 == 0 && ((uintptr_t)obs & 15) == 0);
}

// Inference through the forward-only row-tile kernel (agent_act / agent_value of the models too large for the fused
// agent kernel): the same stream, the same products in the same order as the trainer's forward pass.
int launch_forward_chain(gmi_instance* g, gmi_model* m, const float* obs, int n_rows, float* mu, float* val,
                         bool x0_valid) {
  const ModelLayout& L = m->L;
  if (L.dtype != GMI_DTYPE_BF16 || L.sh_chain_bytes == 0 || L.act_dim > 32) return GMI_ERR_UNSUPPORTED;
  if (n_rows < 1 || n_rows > m->max_rows) return GMI_ERR_UNSUPPORTED;
  ChainArgs a = {};
  int probe = 0, rc = GMI_ERR_UNSUPPORTED;
  for (int p = 0; p < kTileFwdParts && rc == GMI_ERR_UNSUPPORTED; ++p) rc = kTileFwdFns[p](nullptr, L, a, 0, &probe, 0.0, 0.0);
  if (rc != GMI_OK) return rc;      // no forward-only kernel compiled for this shape
  for (int net = 0; net < 2; ++net) {
    a.wstream[net] = m->shadow + L.sh_chain[net];
    for (int l = 0; l < L.n_layers; ++l) a.bias[net][l] = reinterpret_cast<const float*>(m->shadow + L.net[net][l].sh_b);
  }
  a.x0 = (uint16_t*)m->x0;
  a.log_std = reinterpret_cast<const float*>(m->shadow + L.sh_logstd);
  a.idx = nullptr;
  a.b_obs = obs;
  a.n_envs = n_rows; a.ld_envs = n_rows; a.obs_dim = L.obs_dim;
  a.x0_ready = forward_chain_reads_x0(m, obs) ? 1 : 0;
  a.rows = n_rows; a.act_dim = L.act_dim;
  a.net0 = mu ? 0 : 1;
  a.mu_out = mu; a.val_out = val;
  if (a.x0_ready && !x0_valid) {
    rc = launch_gather(g, m, obs, n_rows, n_rows, nullptr, n_rows, nullptr);
    if (rc != GMI_OK) return rc;
  }
  double flops = 0.0, bytes = 0.0;
  for (int net = a.net0; net < 2; ++net)
    for (int l = 0; l < L.n_layers; ++l) {
      const LayerInfo& li = L.net[net][l];
      flops += 2.0 * n_rows * (double)li.in * li.out;
      bytes += 2.0 * li.in * li.out;
    }
  bytes += (a.x0_ready ? 2.0 : 4.0) * n_rows * L.obs_dim * (2 - a.net0) + 4.0 * n_rows * ((mu ? L.act_dim : 0) + 1);
  int tiles = 0;
  rc = GMI_ERR_UNSUPPORTED;
  for (int p = 0; p < kTileFwdParts && rc == GMI_ERR_UNSUPPORTED; ++p) rc = kTileFwdFns[p](g, L, a, n_rows, &tiles, flops, bytes);
  return rc;
}

}  // namespace gmi
