/*
 * gmidrl.h -- C ABI of the MI355X-native PPO agent/trainer hot path of GMI-DRL.
 *
 * The paper's unit of execution is the GMI ("GPU multiplexing instance", Section 2): a
 * resource-adjustable sub-GPU that hosts one or more of the three DRL roles of Section 3
 * (environment simulator, agent, trainer) and talks to other GMIs by send/recv (Listing 1).
 * Here a GMI is a HIP stream restricted to a set of compute units of one gfx950 device; all
 * instances of a process share one address space, so "sending" experience or parameters to
 * another instance is an ordering (event) plus, optionally, a device-to-device copy.
 *
 * Conventions
 *  - Every function returns 0 (GMI_OK) or a negative gmi_status.  gmi_last_error() returns a
 *    thread-local, human-readable message for the last failure on the calling thread.
 *  - "dev" pointers are device memory owned by the caller (e.g. PyTorch tensors); they must stay
 *    valid until the work that uses them has completed.  "host" pointers are ordinary host memory
 *    read during the call.  The library allocates device memory only inside *_bind / gmi_create
 *    and frees it in the matching *_destroy; no compute call allocates.
 *  - Every compute call is asynchronous on its instance's stream.  Ordering between instances is
 *    established only by gmi_transfer(); gmi_sync() blocks the host.  The library never waits for
 *    streams it does not own unless told to: whatever the caller put into a dev buffer on another stream
 *    (an allocator's fill, a copy) must have completed before the call that touches the buffer is made, or
 *    gmi_wait_stream() must have ordered the instance behind that stream.
 *  - All randomness is a pure function of (seed, stream id, step, env index, element) through
 *    Philox4x32-10: counter = (env index, step, stream id, block), key = (seed low, seed high).
 *    Stream ids: 0 action noise, 1 environment noise, 2 done draw, 3 reset state, 4 shuffle.
 *    Element j of a per-env vector uses block j/4; words (0,1) of a block give normals 0,1 and
 *    words (2,3) give normals 2,3 (Box-Muller, see gmi_noise_fill).
 *  - Matrices are row-major.  Experience is time-major: [T, ld_envs] (scalars per step and env)
 *    or [T, ld_envs, dim]; sample index of (t, env) in a batch is t * n_envs + env.
 *  - Flat parameter vector (fp32 master): policy net W_0,b_0,...,W_L,b_L, value net the same,
 *    then log_std[act_dim].  W_l is [out_l, in_l] row-major; L = n_hidden; the policy head has
 *    act_dim outputs and the value head 1.  Both nets use ELU (alpha = 1) on hidden layers and a
 *    linear head (policy shapes of the paper's Table 6 are "in:h1:...:out" in this notation).
 */
#ifndef GMIDRL_H
#define GMIDRL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GMI_OK = 0,
  GMI_ERR_INVALID_ARG = -1,
  GMI_ERR_BAD_SHAPE = -2,
  GMI_ERR_BAD_HANDLE = -3,
  GMI_ERR_HIP = -4,
  GMI_ERR_UNSUPPORTED = -5
} gmi_status;

typedef enum { GMI_DTYPE_F32 = 0, GMI_DTYPE_BF16 = 1 } gmi_dtype;

#define GMI_MAX_HIDDEN 8

typedef struct gmi_instance* gmi_t;
typedef struct gmi_model* gmi_model_t;
typedef struct gmi_env* gmi_env_t;
typedef struct gmi_buffer* gmi_buffer_t;

/* ------------------------------------------------------------------ instances --------------- */

/* Creates an instance: a stream on `device` whose kernels run only on the compute units whose
 * bit is set in cu_mask (bit i of word i/32 = CU i; the paper's GMI_manager.add_GMI + set_GPU of
 * Listing 1, with the SM share of a GMI expressed as a CU set).  cu_mask == NULL or n_words == 0
 * gives an unrestricted stream.  An all-zero mask is GMI_ERR_INVALID_ARG.  host: cu_mask. */
int gmi_create(const uint32_t* cu_mask, uint32_t n_words, int device, gmi_t* out);
int gmi_destroy(gmi_t gmi);
/* The instance's hipStream_t (as void*), e.g. for torch.cuda.ExternalStream. NULL on bad handle. */
void* gmi_stream(gmi_t gmi);
/* Blocks the host until all work queued on the instance has finished. */
int gmi_sync(gmi_t gmi);
/* Makes the instance wait for everything queued so far on a stream of the caller (a hipStream_t as void*; NULL =
 * the device's default stream): work queued on the instance after this call starts only when that work has
 * finished.  For data the caller produces on streams of its own (an allocator's fill, a copy) -- the on-device
 * alternative to synchronising the host before a call that touches such a buffer.  Does not block the host. */
int gmi_wait_stream(gmi_t gmi, void* hip_stream);
/* Number of compute units enabled for the instance (device CU count if unrestricted). */
int gmi_cu_count(gmi_t gmi);
const char* gmi_last_error(void);
/* enable != 0 (default): agent_act / agent_value, rollout_collect and ppo_update use the kernels that carry a tile
 * of rows through all layers of both nets in one launch wherever the model has one; 0: one launch per layer.  Both
 * give results within the same tolerances (tests compare each with the oracle). */
int gmi_set_fusion(gmi_t gmi, int enable);

/* Hands data from instance `src` to instance `dst` (the paper's asynchronous send / synchronous
 * recv of Listing 1, and the experience / parameter movements of Table 5, which on one device need
 * no host bounce): work queued on dst after this call sees everything queued on src before it.
 * If bytes > 0 and src_ptr != dst_ptr, a device-to-device copy of `bytes` is queued on src first.
 * bytes == 0 or src_ptr == dst_ptr: ordering only.  src == dst is allowed (plain copy). dev ptrs.
 * The wait is queued on dst's stream.  Measured on MI355X: while the stream of a CU-masked instance holds
 * work that waits for such an event, kernels of all other instances run about 1.6 times slower; a
 * caller that hands work to masked instances does better to gmi_sync(src) on the host first and to
 * queue the dependent work afterwards (no call of this function needed then). */
int gmi_transfer(gmi_t src, gmi_t dst, const void* src_ptr, void* dst_ptr, size_t bytes);

/* ------------------------------------------------------------------ model ------------------- */

typedef struct {
  int32_t obs_dim;
  int32_t act_dim;
  int32_t n_hidden;                 /* 1..GMI_MAX_HIDDEN */
  int32_t hidden[GMI_MAX_HIDDEN];
  int32_t dtype;                    /* gmi_dtype: arithmetic of the MLP products.
                                       F32: fp32 FMA.  BF16: bf16 operands on MFMA, fp32 accumulate,
                                       fp32 master parameters and optimizer state. */
  int32_t max_rows;                 /* largest number of rows (envs of agent_act, samples of one
                                       minibatch) any call through this binding will process */
} gmi_model_desc;

/* Number of fp32 elements of the flat parameter vector / bytes of the bf16 shadow for a desc
 * (the shadow is needed for dtype BF16 only; returns 0 bytes for F32). */
int64_t gmi_model_param_count(const gmi_model_desc* desc);
int64_t gmi_model_shadow_bytes(const gmi_model_desc* desc);

/* Binds a model to an instance and allocates that binding's activation workspace.
 *  params  dev fp32 [P]   master parameters (read by F32 forward; read/written by ppo_update)
 *  shadow  dev bytes      bf16 copies of the weights in MFMA-friendly padded layouts, plus fp32
 *                         biases and log_std; opaque to the caller, gmi_model_shadow_bytes() long,
 *                         256-byte aligned; written by gmi_model_refresh_shadow and ppo_update,
 *                         read by agent_act / value.  Several bindings (agent instances and the
 *                         trainer instance) may share one params/shadow pair.  NULL for F32.
 *  adam_m, adam_v  dev fp32 [P]  Adam moments; NULL for an inference-only binding (ppo_update then
 *                         fails with GMI_ERR_INVALID_ARG). */
int gmi_model_bind(gmi_t gmi, const gmi_model_desc* desc, float* params, void* shadow,
                   float* adam_m, float* adam_v, gmi_model_t* out);
int gmi_model_destroy(gmi_model_t model);
/* Rebuilds the shadow from the master parameters (after the caller initialised or replaced them). */
int gmi_model_refresh_shadow(gmi_t gmi, gmi_model_t model);

/* ------------------------------------------------------------------ environment ------------- */

typedef struct {
  int32_t n_envs;
  int32_t obs_dim;
  int32_t act_dim;
  float noise_std;
  float reward_scale;
  uint32_t done_period;      /* > 0: done when (episode_step + 1) % done_period == 0 */
  uint32_t done_threshold;   /* done_period == 0: done when the done-stream word < threshold */
  uint64_t seed;
  uint32_t env_offset;       /* index of this binding's env 0 in the Philox counter */
} gmi_env_desc;

/* The synthetic linear-Gaussian simulator that stands in for the paper's physics simulator role
 * (Section 3, "DRL Environment Simulator"; co-located with the agent in one instance, Section 5.1).
 *  a_mat dev fp32 [O,O], b_mat dev fp32 [O,A]: read at bind time (transposed copies are kept).
 *  episode_step dev u32 [N]: per-env step counter, read and updated by env_step. */
int gmi_env_bind(gmi_t gmi, const gmi_env_desc* desc, const float* a_mat, const float* b_mat,
                 uint32_t* episode_step, gmi_env_t* out);
int gmi_env_destroy(gmi_env_t env);

/* One transition of all N envs:
 *   next_obs = obs A^T + act B^T + noise_std * xi,  xi ~ N(0,1) (stream 1)
 *   reward   = reward_scale * (-|obs|^2 - 0.01 |act|^2)
 *   done     = periodic or Bernoulli (integer compare of the stream-2 word with done_threshold)
 *   where done: next_obs = fresh N(0,1) state (stream 3), episode_step = 0; else episode_step += 1
 * obs dev [N,O], act dev [N,A] in; next_obs dev [N,O] (must not alias obs), reward dev [N],
 * done dev u8 [N] out.  step = global interaction index (iteration * horizon + t). */
int env_step(gmi_t gmi, gmi_env_t env, const float* obs, const float* act, uint32_t step,
             float* next_obs, float* reward, uint8_t* done);

/* ------------------------------------------------------------------ agent ------------------- */

/* Action decision of the agent role (Section 3, "DRL Agent") for n_rows envs:
 *   mu = pi(obs), value = V(obs), eps ~ N(0,1) (stream 0, env index = env_offset + row)
 *   act = mu + exp(log_std) * eps,  logp = sum_j [-eps_j^2/2 - log_std_j - ln(2 pi)/2]
 * obs dev [n,O] in; act dev [n,A], logp dev [n], value dev [n] out; mu dev [n,A] out or NULL. */
int agent_act(gmi_t gmi, gmi_model_t model, const float* obs, int32_t n_rows, uint64_t seed,
              uint32_t step, uint32_t env_offset, float* act, float* logp, float* value, float* mu);

/* value = V(obs) only: the bootstrap value of the state after the last collected step. */
int agent_value(gmi_t gmi, gmi_model_t model, const float* obs, int32_t n_rows, float* value);

/* Agents that only serve, in 8-bit floating point (the agent role of Section 3 needs the forward pass alone).
 * A gmi_fp8_t holds, in device memory it owns, the model's weights as E4M3 (the OCP 8-bit format: 4 exponent bits,
 * bias 7, 3 mantissa bits, largest value 448) in matrix-instruction operand order, one power-of-two scale per
 * layer (the smallest s with max|W_l| / s <= 448), fp32 biases and log_std, and a [max_rows, act_dim] fp32 array
 * for the means.  desc: shapes and max_rows as for gmi_model_bind (dtype is ignored); layers up to 512 wide (GMI_ERR_UNSUPPORTED beyond what fits in LDS).
 * gmi_fp8_refresh quantises from params dev fp32 [P] (the flat parameter vector of gmi_model_bind) on the
 * instance's stream: call it after every parameter publication the agent should see. */
typedef struct gmi_fp8* gmi_fp8_t;
int gmi_fp8_bind(gmi_t gmi, const gmi_model_desc* desc, gmi_fp8_t* out);
int gmi_fp8_refresh(gmi_t gmi, gmi_fp8_t weights, const float* params);
int gmi_fp8_destroy(gmi_fp8_t weights);

/* agent_act through the fp8 weights: the observation and every hidden activation are rounded to E4M3 (nearest
 * even, saturating at +-448, no scale), products accumulate in fp32, then scale, fp32 bias and ELU; the heads'
 * outputs are fp32.  Noise, action and log-density exactly as agent_act.  Same arguments and layouts as agent_act;
 * n_rows <= the binding's max_rows. */
int agent_act_fp8(gmi_t gmi, gmi_fp8_t weights, const float* obs, int32_t n_rows, uint64_t seed, uint32_t step,
                  uint32_t env_offset, float* act, float* logp, float* value, float* mu);

/* ------------------------------------------------------------------ experience -------------- */

typedef struct {
  int32_t horizon;     /* T */
  int32_t n_envs;      /* N: envs (columns) covered by this binding */
  int32_t ld_envs;     /* column stride of the arrays (>= N); > N when the binding is a column
                          slice of a wider buffer shared by several agent instances */
  int32_t obs_dim;
  int32_t act_dim;
  float* obs;          /* dev [T, ld, O] */
  float* act;          /* dev [T, ld, A] */
  float* logp;         /* dev [T, ld]   */
  float* val;          /* dev [T, ld]   */
  float* rew;          /* dev [T, ld]   */
  uint8_t* done;       /* dev [T, ld]   */
  float* adv;          /* dev [T, ld]   written by gae_compute */
  float* ret;          /* dev [T, ld]   written by gae_compute */
} gmi_buffer_desc;

/* Experience buffer: one array per type of data (the per-type "channels" of Section 4.2), time
 * major so that one step's write is one contiguous slab per array.  The binding owns a small
 * workspace on the device (partial sums of the advantage normalisation; 8 index arrays of T * N
 * int32 for the minibatch shuffles of ppo_update; if obs_dim is not a multiple of 4 or obs is not
 * 16-byte aligned, T * N rows of obs_dim rounded up to a multiple of 32 two-byte elements, into which
 * ppo_update copies the observations it is called on), freed by gmi_buffer_destroy. */
int gmi_buffer_bind(gmi_t gmi, const gmi_buffer_desc* desc, gmi_buffer_t* out);
int gmi_buffer_destroy(gmi_buffer_t buf);

/* Stores step t's experience (state, action, log-prob, value, reward, done) of N envs into slot t
 * (Section 3: the agent records experience vectors for the trainer).  All inputs dev, [N,...]. */
int collect_experience(gmi_t gmi, gmi_buffer_t buf, int32_t t, const float* obs, const float* act,
                       const float* logp, const float* value, const float* reward,
                       const uint8_t* done);

/* The whole experience-collection stage (Section 5.1, stage (i)) of one instance that hosts simulator and
 * agent together (Section 3): for t = 0 .. T-1 (T = the buffer's horizon), with step = step0 + t,
 *   agent_act(obs_t) -> env_step(obs_t, act_t) -> collect_experience(slot t), obs_{t+1} = next_obs,
 * then last_value = V(obs_T).  Same arithmetic and Philox counters as those calls made one by one, but one
 * launch: each workgroup keeps its envs' state on chip for all T steps.
 *  obs dev [N,O]: in = obs_0, out = obs_T (updated in place); last_value dev [N] out;
 *  seed / env_offset: the agent's (as in agent_act); the simulator uses its binding's own.
 *  The env's episode_step array advances by T steps.  BF16 models only.  One launch for models whose (padded) bf16
 *  weights total at most 1 MiB and whose 32-env tile fits the on-chip memory; larger models that have a forward-only
 *  kernel of their own (the 512-wide shapes) and T >= 2 take two launches per step (that kernel, then one env-step
 *  launch that also decides the actions and stores the experience; obs_t passes through slot t of the buffer);
 *  otherwise GMI_ERR_UNSUPPORTED and nothing has run (use the per-step calls). */
int rollout_collect(gmi_t gmi, gmi_model_t model, gmi_env_t env, gmi_buffer_t buf, float* obs,
                    uint64_t seed, uint32_t step0, uint32_t env_offset, float* last_value);

/* Generalized advantage estimation over the horizon, then returns, then optional normalisation:
 *   delta_t = r_t + gamma v_{t+1} (1-d_t) - v_t (v_T = last_value),  A_t = delta_t + gamma lambda (1-d_t) A_{t+1}
 *   ret = A + v;  normalize != 0: A <- (A - mean) / (std + 1e-8) over all T*N entries.
 * last_value dev [N]. */
int gae_compute(gmi_t gmi, gmi_buffer_t buf, const float* last_value, float gamma, float lambda,
                int normalize);

/* gae_compute for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it): no buffer binding is needed -- a binding owns allocations -- and the call itself
 * allocates nothing.  Same kernels and results as gae_compute on a binding of the same arrays.
 *  rew, val dev [T, ld] fp32, done dev [T, ld] u8, last_value dev [N]: inputs;  adv, ret dev [T, ld]: outputs
 *  (all caller-owned; columns N..ld-1 are not touched).
 *  The per-workgroup partial sums of the normalisation live in a fixed array of 256 KiB that the library holds on
 *  every device it runs on until the process ends; it covers n_envs <= 4 194 304 (more: GMI_ERR_BAD_SHAPE, nothing
 *  runs).  All calls on one device share that array: calls with normalize != 0 that overlap on one device (two
 *  instances, or two host threads) race on it -- order them.  Asynchronous on the instance's stream like every
 *  compute call. */
int gae_compute_static(gmi_t gmi, int32_t horizon, int32_t n_envs, int32_t ld_envs, const float* rew,
                       const float* val, const uint8_t* done, const float* last_value, float gamma, float lambda,
                       int normalize, float* adv, float* ret);

/* ------------------------------------------------------------------ trainer ----------------- */

typedef struct {
  float clip;          /* surrogate clip range */
  float c_v;           /* value-loss coefficient */
  float c_e;           /* entropy coefficient */
  float lr, beta1, beta2, adam_eps;
  int32_t epochs;
  int32_t minibatch;   /* must divide T*N */
  uint64_t seed;       /* shuffle seed */
  uint32_t iteration;  /* shuffle counter: permutation is a function of (seed, iteration, epoch) */
  uint32_t adam_step0; /* number of Adam steps taken before this call */
} gmi_ppo_hparams;

/* Model training stage of the trainer role (Section 3 "DRL Trainer"; stage (ii) of Section 5.1):
 * for each epoch a seeded permutation of the T*N samples, consecutive `minibatch`-sized slices are
 * the minibatches; each does forward of both nets, the clipped-surrogate + value + entropy loss,
 * exact backward, and one Adam step on the fp32 master parameters (and refreshes the shadow).
 * stats_out dev fp32 [epochs * (T*N/minibatch), 5] = per minibatch
 *   {policy loss, value loss, entropy, mean(logp_old - logp), clip fraction}; may be NULL. */
int ppo_update(gmi_t gmi, gmi_model_t model, gmi_buffer_t buf, const gmi_ppo_hparams* hp,
               float* stats_out);

/* Synchronized training of n trainer instances that hold replicas of one model on one GPU (Section 4.1:
 * the replicas' gradients are reduced so that all apply the same update; instances that share an address
 * space need no ring or tree, only an in-memory mean).  models[i] are bindings on instance i of the SAME
 * params / shadow / adam_m / adam_v arrays (each with its own workspace), bufs[i] instance i's experience
 * (all of one size).  Per epoch instance i shuffles its buffer with the key seed + i; minibatch j is the
 * union of the instances' j-th slices of hp->minibatch samples; every instance runs forward / loss /
 * backward of its slice on its own stream, instance 0 then sums all partials (fixed order), divides by n,
 * takes the Adam step and refreshes the shared shadow, and the others wait for it before their next slice.
 * stats_out dev fp32 [epochs * (T*N/minibatch), 5]: means over the instances; may be NULL.
 * host: the three handle arrays.  n = 1 is ppo_update.  At most 16 instances. */
int ppo_update_group(const gmi_t* gmis, const gmi_model_t* models, const gmi_buffer_t* bufs, int32_t n,
                     const gmi_ppo_hparams* hp, float* stats_out);

/* Loss statistics of one minibatch given by explicit sample indices, without updating anything
 * (forward + loss only).  idx dev i32 [n]; stats_out dev fp32 [5]. */
int ppo_evaluate(gmi_t gmi, gmi_model_t model, gmi_buffer_t buf, const gmi_ppo_hparams* hp,
                 const int32_t* idx, int32_t n, float* stats_out);

/* Forward, loss and backward of one minibatch given by explicit sample indices: writes the flat
 * gradient dL/dtheta (dev fp32 [P]) and the stats (dev fp32 [5]); updates nothing. */
int ppo_gradient(gmi_t gmi, gmi_model_t model, gmi_buffer_t buf, const gmi_ppo_hparams* hp,
                 const int32_t* idx, int32_t n, float* grad_out, float* stats_out);

/* One Adam step on caller-supplied arrays (dev fp32 [n]): step = 1-based step index. */
int adam_update(gmi_t gmi, float* params, float* adam_m, float* adam_v, const float* grad,
                int64_t n, const gmi_ppo_hparams* hp, uint32_t step);

/* ------------------------------------------------------------------ utilities --------------- */

/* out[e, j] = standard normal of (seed, stream, step, env_offset + e, element j), dev fp32 [n,dim].
 * Box-Muller on Philox words with integer-defined uniforms: u1 = (2 (w_a >> 9) + 1) / 2^24,
 * quadrant = w_b >> 30, position in quadrant = (2 ((w_b >> 7) & 0x7FFFFF) + 1) / 2^24. */
int gmi_noise_fill(gmi_t gmi, uint64_t seed, uint32_t stream, uint32_t step, uint32_t env_offset,
                   int32_t n_envs, int32_t dim, float* out);
/* out[i] = shuffle permutation of [0,n) for (seed, iteration, epoch), dev i32 [n]. */
int gmi_permutation(gmi_t gmi, int32_t n, uint64_t seed, uint32_t iteration, uint32_t epoch,
                    int32_t* out);

/* ------------------------------------------------------------------ per-launch timing ------- */

/* ------------------------------------------------------------------ instance selection ------ */

/* Trial run of one point of the search: instances per GPU and environments per instance in; runnable
 * (0/1), throughput of ONE instance and its memory footprint out (any consistent units).  Non-zero return
 * aborts the search with an error.  user: the pointer given to gmi_explore. */
typedef int (*gmi_profile_fn)(int32_t gmi_per_gpu, int32_t num_env, int32_t* runnable, double* throughput,
                              double* memory, void* user);
/* Projection of one instance's throughput to the whole system. */
typedef double (*gmi_estimate_fn)(int32_t gmi_per_gpu, int32_t num_gpu, double throughput, void* user);

/* Profiling-based instance exploration (Algorithm 2, Section 5.3 "Workload-aware GMI Selection").
 * For each instances-per-GPU value (in the order given; the paper walks 10 .. 1) the environments-per-
 * instance values are profiled in the order given (the paper: 128, 256, .. 16384).  Non-runnable points are
 * skipped; the first runnable point of an instance size only initialises the trackers; for every later one
 *   R_top = (top - pre_top) / pre_top,  R_mem = (mem - pre_mem) / pre_mem,  Sat = R_top / R_mem
 * (IEEE divisions), the trackers move to this point, Sat < alpha ends this instance size, otherwise the
 * point is projected with estimate() and kept if it beats every earlier projection (strictly).
 * estimate == NULL: throughput * gmi_per_gpu * num_gpu.  All pointers host.  Outputs: the chosen pair
 * (0, 0 if no point was ever recorded) and, if projected != NULL, its projection.  Host-only: no GPU work
 * happens inside this call except what the callbacks do. */
int gmi_explore(gmi_profile_fn profile, void* profile_user, gmi_estimate_fn estimate, void* estimate_user,
                int32_t num_gpu, double alpha, const int32_t* gmi_per_gpu_values, int32_t n_gmi,
                const int32_t* num_env_values, int32_t n_env, int32_t* num_env_out, int32_t* gmi_per_gpu_out,
                double* projected);

/* ------------------------------------------------------------------ experience channels ---- */

/* Channel-based experience sharing between agent and trainer instances (Section 4.2, "Channel-based Experience
 * Sharing") on one GPU.  A channel set is a ring of `capacity` slabs in device memory (allocated by
 * gmi_channels_create, freed by gmi_channels_destroy); a slab is one agent instance's experience of one
 * collection round: [horizon, n_envs] samples.  mode GMI_CHANNELS_MULTI keeps one array per type of data
 * (state, action, log-prob, value, reward, done: the paper's per-type channels); GMI_CHANNELS_UNI keeps one
 * array of interleaved records [obs | act | logp | val | rew | done as float] per sample, the single-channel
 * form the paper compares against.  Every value arrives bit for bit. */
typedef struct gmi_channels* gmi_channels_t;
#define GMI_CHANNELS_MULTI 0
#define GMI_CHANNELS_UNI 1
typedef struct {
  int32_t horizon, n_envs, obs_dim, act_dim;   /* shape of a slab */
  int32_t capacity;                            /* slabs in the ring, 1 .. 4096 */
  int32_t mode;
} gmi_channels_desc;
int gmi_channels_create(const gmi_channels_desc* desc, int device, gmi_channels_t* out);
int gmi_channels_destroy(gmi_channels_t ch);     /* synchronises the device first */

/* Agent side (the paper's dispenser and compressor): copies the filled experience buffer `src` (its n_envs
 * columns, all arrays, in one launch on the agent's stream) and last_value dev [n_envs] into the next free
 * slab.  The agent may refill `src` as soon as its own stream has passed this call.  GMI_ERR_UNSUPPORTED (and
 * nothing done) when all slabs are waiting for the trainer; GMI_ERR_BAD_SHAPE when src is not slab-shaped. */
int gmi_channels_push(gmi_t agent, gmi_channels_t ch, gmi_buffer_t src, const float* last_value);

/* Trainer side (the paper's migrator and batcher): takes the n_slabs (1..8) oldest slabs, of each the env
 * columns [env0, env0 + take) (slicing), and places them side by side in arrival order (stacking) into the
 * columns [dst_col0, dst_col0 + n_slabs * take) of `dst` (obs, act, logp, val, rew, done) and into
 * last_value_out dev [n_slabs * take], in one launch on the trainer's stream, which first waits for the agents'
 * pushes of these slabs.  The slabs are free again once the trainer's stream has passed this call.
 * GMI_ERR_UNSUPPORTED (nothing done) when fewer than n_slabs slabs are waiting. */
int gmi_channels_pop(gmi_t trainer, gmi_channels_t ch, int32_t n_slabs, int32_t env0, int32_t take,
                     gmi_buffer_t dst, int32_t dst_col0, float* last_value_out);

/* Discards the n_slabs oldest waiting slabs unread (host only, nothing is copied): what an agent that must not
 * wait does when the ring is full, so that the trainer always finds the freshest experience (the asynchronous
 * setting of Section 5.2, where serving and training run at their own rates).  The next push into such a slab
 * first waits, on its stream, for the discarded push to finish.  GMI_ERR_UNSUPPORTED (nothing done) when fewer
 * than n_slabs are waiting. */
int gmi_channels_drop(gmi_channels_t ch, int32_t n_slabs);

/* Ring state: slabs waiting, and the totals pushed / popped so far (any pointer may be NULL; slabs discarded =
 * pushed - popped - waiting).  Host only.  push, pop, drop and count may be called from different host threads:
 * the ring state is guarded by a lock (the order of slabs is the order in which pushes took that lock). */
int gmi_channels_count(gmi_channels_t ch, int32_t* waiting, int64_t* pushed, int64_t* popped);

/* The migrator's choice among several trainer instances (Section 4.2: the trainer "with the least workload"):
 * index of the smallest entry of samples_so_far host i64 [n_trainers], the lowest index on ties. */
int gmi_route_least_loaded(const int64_t* samples_so_far, int32_t n_trainers, int32_t* trainer_out);

/* ------------------------------------------------------------------ reduction strategy ------ */

/* The three gradient-reduction strategies for trainer instances (Section 4.1, "Layout-aware Gradient
 * Reduction"). */
#define GMI_REDUCE_MULTI_PROCESS 0   /* reduce across the processes through host memory */
#define GMI_REDUCE_MULTI_RING    1   /* one ring per instance index across GPUs, then a ring over the partial results */
#define GMI_REDUCE_HIERARCHICAL  2   /* per GPU among its instances, then one leader per GPU across GPUs */

/* Communication strategy selection (Algorithm 1).  gmis_per_gpu host i32 [n_gpus]: how many trainer instances
 * each GPU hosts (the lengths of the paper's GMI-to-GPU mapping list).  n_gpus <= 1: multi-process; counts that
 * differ between GPUs, or more instances per GPU than GPUs: hierarchical; otherwise multi-ring.  Host-only.  On
 * the one GPU this build runs on the answer is always the first, and ppo_update_group performs that reduction
 * in device memory. */
int gmi_select_reduction(const int32_t* gmis_per_gpu, int32_t n_gpus, int32_t* strategy_out);

/* Leaders of the hierarchical reduction's cross-GPU step (Section 4.1): on every GPU the instance whose id
 * satisfies id % M == t, M = instances on that GPU.  gmi_ids host i32: the ids GPU by GPU; gpu_start host i32
 * [n_gpus + 1]: GPU p owns gmi_ids[gpu_start[p] .. gpu_start[p+1]); leaders_out host i32 [n_gpus], -1 where no
 * id has that residue. */
int gmi_har_leaders(const int32_t* gmi_ids, const int32_t* gpu_start, int32_t n_gpus, int32_t t,
                    int32_t* leaders_out);

/* Time models of the three strategies (Table 2): g GPUs, t instances per GPU, m_p parameter bytes, b1 the
 * inter-instance bandwidth through host memory, b2 the inter-GPU collective bandwidth (bytes/s). */
int gmi_reduction_time(int32_t strategy, int32_t g, int32_t t, double m_p, double b1, double b2,
                       double* seconds_out);

#ifdef __cplusplus
}
#endif
#endif /* GMIDRL_H */
