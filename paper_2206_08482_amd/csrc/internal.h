// Internal declarations shared by the translation units of libgmidrl (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stdio.h>
#include <string>
#include <tuple>
#include <type_traits>
#include <utility>
#include <vector>

#include "../../include/gmidrl.h"
#include "../../include/gmidrl_bench.h"

namespace gmi {

void set_error(const char* fmt, ...);

#define GMI_FAIL(code, ...)            \
  do {                                 \
    ::gmi::set_error(__VA_ARGS__);     \
    return (code);                     \
  } while (0)

#define GMI_HIP(expr)                                                              \
  do {                                                                             \
    hipError_t e__ = (expr);                                                       \
    if (e__ != hipSuccess) {                                                       \
      ::gmi::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__),     \
                       __FILE__, __LINE__);                                        \
      return GMI_ERR_HIP;                                                          \
    }                                                                              \
  } while (0)

#define GMI_LAUNCH_CHECK()                                                         \
  do {                                                                             \
    hipError_t e__ = hipGetLastError();                                            \
    if (e__ != hipSuccess) {                                                       \
      ::gmi::set_error("kernel launch failed: %s (%s:%d)", hipGetErrorString(e__), \
                       __FILE__, __LINE__);                                        \
      return GMI_ERR_HIP;                                                          \
    }                                                                              \
  } while (0)

constexpr uint32_t kMagicInstance = 0x474d4931;  // "GMI1"
constexpr uint32_t kMagicModel = 0x474d494d;
constexpr uint32_t kMagicEnv = 0x474d4945;
constexpr uint32_t kMagicBuffer = 0x474d4942;

static inline int pad32(int x) { return (x + 31) & ~31; }
static inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

}  // namespace gmi

namespace gmi {
// Kernel classes of the built-in per-launch timer (gmi_profile_*).
// One class per kernel symbol, so that a class average can be set beside a profiler's per-kernel
// average.  The linear-layer classes are kClsLinear + 3 * variant + role:
//   variant 0 linear_bf16_big_kernel<4,2,*,4> (256x256 tile)  1 linear_bf16_big_kernel<2,2,*,4> (256x128)
//           2 linear_bf16_kernel<2,2,2,2,*> (128x128)         3 linear_bf16_kernel<1,4,2,2,*> (256x64)
//           4 linear_bf16_kernel<1,4,1,2,*> (128x64)
//   role    0 forward hidden layer (bias + ELU)   1 forward head   2 input gradient (ELU')
// (kClsGae covers gae_kernel and normalize_kernel, kClsLinearF32 the three fp32 epilogues, kClsFusedAgent the
// one-launch agent forward of a model: agent_fused_kernel, or the forward-only row-tile kernel for the shapes that
// have one -- a model uses one or the other.)
enum KernelClass {
  kClsGather = 0, kClsWgrad, kClsLoss, kClsAdam, kClsShadowTranspose, kClsEnvStep, kClsSample,
  kClsCollect, kClsGae, kClsPermutation, kClsFusedAgent, kClsFusedRollout,
  kClsLinearF32, kClsChainTrain, kClsLinear, kClsCount = kClsLinear + 15
};
static_assert(kClsCount < 32, "class masks are 32-bit");
struct ProfSlot {
  std::vector<hipEvent_t> start, stop;
  size_t used = 0;
  double flops = 0.0, bytes = 0.0;   // algorithmic work of the timed launches, where the launcher states it
};
}  // namespace gmi

struct gmi_instance {
  uint32_t magic;
  int device;
  hipStream_t stream;
  hipEvent_t event;      // used by gmi_transfer
  hipEvent_t wait_event; // used by gmi_wait_stream
  int cu_count;
  int fusion;            // 1: use the row-tile fused kernels where the model fits them (default)
  uint32_t prof_mask;    // bit c set: launches of kernel class c carry timing events
  gmi::ProfSlot prof[gmi::kClsCount];
};

namespace gmi {
// Launches kernels of one class on the instance's stream.  While the class is being timed every launch
// carries its own pair of HIP events that receive the kernel's begin and end timestamps
// (hipExtLaunchKernel), so a class average is the kernels' execution time without launch gaps.
struct ProfScope {
  gmi_instance* g;
  int cls;
  bool on;
  ProfScope(gmi_instance* g_, int cls_);
  // adds the algorithmic work of the launches in this scope (counted only while the class is timed)
  void work(double flops, double bytes);
  // next unused event pair of the class (created on demand); false if none could be made
  bool next_events(hipEvent_t* a, hipEvent_t* b);

  // Arguments are converted to the kernel's exact parameter types before their addresses are taken.
  template <typename... KArgs, typename... Args>
  void launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, Args&&... args) {
    static_assert(sizeof...(KArgs) == sizeof...(Args), "kernel argument count");
    std::tuple<std::remove_cv_t<KArgs>...> t{static_cast<KArgs>(std::forward<Args>(args))...};
    launch_impl(reinterpret_cast<const void*>(kernel), grid, block, lds, t, std::index_sequence_for<KArgs...>{});
  }

 private:
  template <typename T, size_t... I>
  void launch_impl(const void* kernel, dim3 grid, dim3 block, size_t lds, T& t, std::index_sequence<I...>) {
    void* ptrs[] = {const_cast<void*>(static_cast<const void*>(&std::get<I>(t)))...};
    hipEvent_t a, b;
    if (on && next_events(&a, &b))
      (void)hipExtLaunchKernel(kernel, grid, block, ptrs, lds, g->stream, a, b, 0);
    else
      (void)hipLaunchKernel(kernel, grid, block, ptrs, lds, g->stream);
  }
};
}  // namespace gmi

// One linear layer of one net.
struct LayerInfo {
  int in, out;           // logical sizes
  int in_pad, out_pad;   // padded to multiples of 32
  int64_t w_off, b_off;  // offsets into the flat fp32 parameter vector
  int64_t sh_wf;              // bf16 W in matrix-core fragment order (see wfrag_index)
  int64_t sh_w, sh_wt, sh_b;  // byte offsets into the shadow (bf16 W [out_pad,in_pad], bf16 W^T
                              // [in_pad,out_pad], fp32 bias [out_pad])
  bool head;
};

struct ModelLayout {
  int obs_dim, act_dim, n_hidden, n_layers;   // n_layers = n_hidden + 1
  int dtype;
  std::vector<LayerInfo> net[2];              // 0 policy, 1 value
  int64_t logstd_off;                         // into flat params
  int64_t sh_logstd;                          // byte offset into shadow (fp32 [act_dim])
  int64_t n_params;
  int64_t shadow_bytes;
  int64_t weight_bytes;                       // bf16 bytes of one copy of all weights (padded), both nets
  int64_t sh_chain[2];                        // byte offsets of the two nets' chain streams (chain.hip)
  int64_t sh_chain_bytes;                     // bytes of one stream; 0 = this model has none
  int max_width_pad;                          // widest padded activation
};

int build_layout(const gmi_model_desc* d, ModelLayout* L);

struct gmi_model {
  uint32_t magic;
  int device;
  ModelLayout L;
  int max_rows;
  float* params;
  char* shadow;
  float *adam_m, *adam_v;
  // workspace (device, owned)
  void* ws_base;
  size_t ws_bytes;
  // activations: x0 shared by both nets; h[net][l] for l = 1..n_hidden; element type = dtype
  void* x0;
  void* x0b;         // x0 in the block layout of the row-tile trainer kernel (written by that kernel)
  void* h[2][GMI_MAX_HIDDEN + 1];
  void* dz[2][GMI_MAX_HIDDEN + 2];   // dz[net][l] = dL/d(pre-activation of layer l-1's output), l=1..n_layers
  float* mu;        // [max_rows, act_dim]
  float* val;       // [max_rows]
  // minibatch gathers
  float *mb_act, *mb_logp, *mb_adv, *mb_ret;
  // gradient partials [n_split_max, n_params] and stats partials
  float* grad_part;
  int n_split_max;
  float* stat_part; // [n_split_max, 8]
};

struct gmi_env {
  uint32_t magic;
  gmi_env_desc d;
  float* m_t;       // dev [(O + A), O]: rows 0..O-1 = A^T, rows O..O+A-1 = B^T
  uint32_t* episode_step;
};

struct gmi_buffer {
  uint32_t magic;
  gmi_buffer_desc d;
  double* part;     // dev [n_part, 2] partial sums for normalisation
  int n_part;
  int32_t* perm;    // dev [kPermEpochs][horizon * n_envs] minibatch shuffles of up to kPermEpochs epochs at once
  uint16_t* obs16;  // dev [horizon * n_envs][pad32(obs_dim)] bf16 copy of the observations by sample index, made at
                    // the start of an update; only for observation rows that 16-byte loads cannot read (else NULL)
};

static inline bool valid(gmi_t g) { return g && g->magic == gmi::kMagicInstance; }
static inline bool valid(gmi_model_t m) { return m && m->magic == gmi::kMagicModel; }
static inline bool valid(gmi_env_t e) { return e && e->magic == gmi::kMagicEnv; }
static inline bool valid(gmi_buffer_t b) { return b && b->magic == gmi::kMagicBuffer; }

// ---------------------------------------------------------------------------------------------
// Linear-layer launchers (mlp.hip).  Element type T of activations is float (F32) or bf16 (BF16).
namespace gmi {

enum Epilogue { kEpiBiasElu = 0, kEpiBiasHead = 1, kEpiEluGrad = 2 };

// y[r, f] = epi( sum_k x[r, k] * w(f, k) )      r < rows, f < F, k < K
//   kEpiBiasElu : y = ELU(acc + bias[f])             stored as T       [rows, ldy]
//   kEpiBiasHead: y = acc + bias[f], f < F_store     stored as float   [rows, ldy]
//   kEpiEluGrad : y = acc * ELU'(h[r, f]) through the stored output h: 1 if h > 0 else h + 1; T
// w(f, k): F32 reads w[f * wsf + k * wsk] from the master parameters; BF16 reads the padded shadow
// copy [F, ldw] (k contiguous).
struct LinearProblem {
  const void* x; int ldx;
  const void* w; int ldw; int wsf, wsk;
  const float* bias;
  const void* h; int ldh;
  void* y; int ldy;
  int K, F, F_store;
  int K_log, F_log;         // logical (unpadded) sizes, for the work accounting of the launch timer
};

struct LinearBatch {
  int n;                    // 1 or 2 problems (policy, value) of equal rows / epilogue
  LinearProblem p[2];
};

int launch_linear(gmi_instance* g, int dtype, int epi, int rows, const LinearBatch& batch);

// dW[o, i] = sum_r dz[r, o] * x[r, i],  db[o] = sum_r dz[r, o], reduced over row splits:
// split sp covers rows [sp*chunk, min(rows, (sp+1)*chunk)) and writes
// part[sp * part_stride + w_off + o*in + i] and part[sp * part_stride + b_off + o].
struct WgradProblem {
  const void* dz; int lddz;
  const void* x; int ldx;
  // 0: the operand is row-major [rows, ld]; 1, 2 (bf16 only): it is in the block layout the row-tile trainer kernel
  // leaves (tile_kernel.h): per 128 rows, per 16-wide feature step ks, per 32-row tile rt, a 1 KiB block whose
  // 16-byte slot s + 32 h holds, of row 32 rt + s, the features 16 ks + 4 h + {0..3} and 16 ks + 8 + 4 h + {0..3} (1)
  // or 16 ks + 8 h + {0..7} (2: the gathered observation rows).  Either both operands are row-major or none is.
  int dz_blocks, x_blocks;
  int out, in, out_pad, in_pad;
  int64_t w_off, b_off;
};
constexpr int kMaxWgradProblems = 2 * (GMI_MAX_HIDDEN + 1);
struct WgradBatch {
  int n;
  WgradProblem p[kMaxWgradProblems];
  int blk_start[kMaxWgradProblems + 1];
};
int launch_wgrad(gmi_instance* g, int dtype, int rows, int n_split, int chunk, WgradBatch& batch,
                 float* part, int64_t part_stride);

}  // namespace gmi

// ---------------------------------------------------------------------------------------------
// Model-level helpers (model.hip) used by the agent and trainer entry points.
namespace gmi {

static inline size_t elem_size(int dtype) { return dtype == GMI_DTYPE_BF16 ? 2 : 4; }

// x0[r, :] <- obs of sample idx[r] (identity when idx == NULL), converted to the model's element
// type, zero padded to the padded width; optionally also gathers act / logp / adv / ret rows.
// Sample s of a buffer lives at slot (s / n_envs) * ld_envs + s % n_envs.
int launch_gather(gmi_instance* g, gmi_model* m, const float* obs, int n_envs, int ld_envs,
                  const int32_t* idx, int rows, const gmi_buffer_desc* extras);
// The same with the rows written to x_out (of the model's activation type) instead of m->x0.
int launch_gather_to(gmi_instance* g, gmi_model* m, const float* obs, int n_envs, int ld_envs,
                     const int32_t* idx, int rows, const gmi_buffer_desc* extras, void* x_out);

// Runs both nets (or only the value net) on the rows staged in m->x0; keeps hidden activations in
// m->h[net][l]; writes m->mu [rows, A] and m->val [rows].
int forward_nets(gmi_instance* g, gmi_model* m, int rows, bool policy, bool value, float* mu_dst,
                 float* val_dst);

int launch_agent_fused(gmi_instance* g, gmi_model* m, const float* obs, int n, uint64_t seed, uint32_t step,
                       uint32_t env_offset, float* act, float* logp, float* value, float* mu_out, bool do_policy);


// Shuffles of epochs epoch0 .. epoch0 + n_epochs - 1 into out[e][n], one launch.
constexpr int kPermEpochs = 8;
int launch_permutation(gmi_instance* g, int n, uint64_t seed, uint32_t iteration, uint32_t epoch0, int n_epochs, int32_t* out);

// Register-chained trainer kernel (chain.hip): its weight stream in the shadow and the launch.
int64_t chain_stream_bytes(const ModelLayout& L);
int launch_chain_pack(gmi_instance* g, gmi_model* m);
// Where shadow_transpose_kernel puts the blocks of the chain streams (the layout launch_chain_pack writes): per
// entry of the shadow table (net-major) the first block of the layer's forward and input-gradient segments.
struct ChainEmitLayer {
  int fwd_blk, bwd_blk;      // bwd_blk < 0: the first layer has no input-gradient segment
  int natural;               // 1: k indices of a lane in natural order (first forward layer)
};
struct ChainEmit {
  int gmax;                  // tiles in the largest group; 0: the model has no chain stream
  int n_layers;
  int64_t out[2];            // byte offsets of the two nets' streams in the shadow
  ChainEmitLayer l[kMaxWgradProblems];
};
void fill_chain_emit(const ModelLayout& L, ChainEmit* ce);
// Forward pass of n_rows observation rows through the forward-only row-tile kernel: policy means into mu (NULL: value
// net only) and values into val.  GMI_ERR_UNSUPPORTED (no message) if no such kernel is compiled for the shape.
int launch_forward_chain(gmi_instance* g, gmi_model* m, const float* obs, int n_rows, float* mu, float* val,
                         bool x0_valid = false);
// Whether that kernel would read the bf16 rows m->x0 (made by the gather kernel) instead of obs itself.
bool forward_chain_reads_x0(const gmi_model* m, const float* obs);
// The collection stage for the models too large for the one-launch rollout kernel: per step the forward-only kernel
// and one env-step launch that also decides the actions and stores the experience (model.hip).
int rollout_stepwise(gmi_instance* g, gmi_model* m, gmi_env* env, gmi_buffer* b, float* obs, uint64_t seed,
                     uint32_t step0, uint32_t env_offset, float* last_value);
// What the collection stage of a model too large for the one-launch rollout kernel adds to an env step: the action
// decision from the policy means of the step, the experience store of the step, the bf16 rows of the next state.
struct StepFuse {
  const float* mu;            // [N, A] policy means of this step
  const float* log_std;       // [A]
  uint32_t ak0, ak1, a_env_offset;      // the agent's Philox key and env offset (the simulator has its own)
  float* b_obs;               // slot t of the experience arrays: obs [N, O] (NULL: the slot already holds this state),
  float* b_act;               // act [N, A],
  float* b_logp;              // logp [N]
  uint16_t* x16_next;         // bf16 rows [N, o_pad] of the next state, or NULL
  int o_pad;
};
// env_step's launch; fuse != NULL: act is not read (the actions are decided in the kernel), reward and done point
// into slot t of the experience arrays.
int launch_env_step(gmi_instance* g, gmi_env* env, const float* obs, const float* act, uint32_t step, float* next_obs,
                    float* reward, uint8_t* done, const StepFuse* fuse);
// The action decision from given means: act = mu + exp(log_std) * eps, logp, optional copy of mu (model.hip).
int launch_sample(gmi_instance* g, const float* mu, const float* log_std, int n_rows, int act_dim, uint64_t seed,
                  uint32_t step, uint32_t env_offset, float* act, float* logp, float* mu_out);
// obs16_ready: b->obs16 holds the bf16 copy of the buffer's present observations (prepare_obs16).
// *blocks = whether the hidden activations and gradients were left in the row-tile kernel's block layout.
int launch_train_chain(gmi_instance* g, gmi_model* m, gmi_buffer* b, const gmi_ppo_hparams* hp, const int32_t* idx, int rows,
                       int* n_stat_rows, bool obs16_ready, bool* blocks);
// Before the minibatches of an update: converts all observations of the buffer into b->obs16 if the chained kernel
// will run and cannot read the fp32 rows itself.  *ready = whether it did.
int prepare_obs16(gmi_instance* g, gmi_model* m, gmi_buffer* b, bool* ready);

}  // namespace gmi

namespace gmi {
constexpr int kSplitMin = 16;        // row splits of the weight-gradient reduction: lower and
constexpr int kSplitMax = 32;        // upper bound of the per-model choice below

// Row splits for a weight-gradient launch over n_tiles 128x128 output tiles.  Two workgroups fit a
// compute unit, so up to 512 are resident at once; few-tile models get more splits to approach that.
// The count stays a multiple of 8: workgroups go round-robin over the 8 XCDs, so with split = index % count
// every tile of one split (which reads the same rows) lands on the same XCD and shares its L2.  Counts
// that are not a multiple of 8 measured 1.4-2x slower.
static inline int wgrad_split_limit(int n_tiles) {
  int s = (512 / (n_tiles > 0 ? n_tiles : 1)) / 8 * 8;
  if (s < kSplitMin) s = kSplitMin;
  if (s > kSplitMax) s = kSplitMax;
  return s;
}
constexpr int kLossBlocksMax = 2048; // rows of per-workgroup loss statistics (one more row holds their sum)
constexpr int kStatStride = 8;       // per-workgroup statistics slots before the log_std partials

// Fragment-major weight copy for the row-tile fused kernels: the weights of (32-feature tile ft, 16-wide
// k step ks) form one 1 KiB block in which lane L of a wave owns the 8 consecutive k values of feature
// ft*32 + L%32 starting at ks*16 + (L/32)*8, i.e. exactly its operand of the 32x32x16 bf16 matrix
// instruction.  A wave then fetches an operand with one fully coalesced 16-byte-per-lane load instead of
// touching 32 weight rows (measured: the row-major fetch kept the texture addresser busy ~4x longer).
__host__ __device__ static inline int64_t wfrag_index(int o, int i, int in_pad) {
  const int ft = o >> 5, ks = i >> 4, lane = (o & 31) + 32 * ((i & 15) >> 3);
  return (((int64_t)ft * (in_pad >> 4) + ks) * 64 + lane) * 8 + (i & 7);
}

// Where each parameter lives in the flat vector and in the bf16 shadow (kernel argument).
struct ShadowLayer {
  int64_t w_off, b_off;
  int in, out, in_pad, out_pad;
  int64_t sh_w, sh_wt, sh_b, sh_wf;
};
struct ShadowTable {
  int n;
  ShadowLayer l[kMaxWgradProblems];
  int64_t logstd_off, sh_logstd;
  int act_dim;
  int64_t n_params;
};
static inline ShadowTable make_shadow_table(const ModelLayout& L) {
  ShadowTable t;
  t.n = 0;
  for (int net = 0; net < 2; ++net)
    for (const LayerInfo& li : L.net[net]) {
      ShadowLayer& s = t.l[t.n++];
      s.w_off = li.w_off; s.b_off = li.b_off; s.in = li.in; s.out = li.out;
      s.in_pad = li.in_pad; s.out_pad = li.out_pad; s.sh_w = li.sh_w; s.sh_wt = li.sh_wt; s.sh_b = li.sh_b; s.sh_wf = li.sh_wf;
    }
  t.logstd_off = L.logstd_off;
  t.sh_logstd = L.sh_logstd;
  t.act_dim = L.act_dim;
  t.n_params = L.n_params;
  return t;
}
}  // namespace gmi
