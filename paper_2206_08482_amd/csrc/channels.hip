// Channel-based experience sharing between agent and trainer instances (Section 4.2 of the paper) on one GPU.
// A channel set is a ring of slabs in device memory; a slab holds one agent instance's experience of one
// collection round, one array per type of data (state, action, log-prob, value, reward, done, bootstrap value)
// -- or, in the uni-channel form the paper compares against, one array of interleaved records.
//   push  = the agent's dispenser (sorts by type) + the compressor (a slab's arrays move in ONE launch);
//   pop   = the migrator (same GPU: hands the slabs over by an event) + the trainer's batcher (takes a column
//           slice of each of the k oldest slabs and stacks them side by side in the trainer's batch), also one
//           launch for all k slabs.
// The instances share an address space, so a slab moves device-to-device; ordering is by events per slab
// (filled: recorded on the agent's stream, awaited by the trainer's; freed: the other way round).
#include "internal.h"

#include <mutex>

struct gmi_channels {
  uint32_t magic;
  int device;
  gmi_channels_desc d;
  char* base;                 // all slabs
  size_t slab_bytes;
  // byte offsets of a slab's arrays (multi) / of the record array (uni)
  size_t off_obs, off_act, off_logp, off_val, off_rew, off_done, off_rec, off_last;
  int head, count;            // ring state (host)
  int64_t pushed, popped;
  std::vector<hipEvent_t> filled, freed;
  std::vector<char> was_popped, was_dropped;
  std::mutex mu;              // the ring state above: agents and the trainer may call from threads of their own
};

namespace {
constexpr uint32_t kMagicChannels = 0x474d4943;   // "GMIC"
bool valid(gmi_channels_t c) { return c && c->magic == kMagicChannels; }

struct SlabPtrs {
  float *obs, *act, *logp, *val, *rew, *rec, *last;
  uint8_t* done;
};
SlabPtrs slab_ptrs(const gmi_channels* c, int slab) {
  char* p = c->base + (size_t)slab * c->slab_bytes;
  SlabPtrs s;
  s.obs = (float*)(p + c->off_obs); s.act = (float*)(p + c->off_act); s.logp = (float*)(p + c->off_logp);
  s.val = (float*)(p + c->off_val); s.rew = (float*)(p + c->off_rew); s.done = (uint8_t*)(p + c->off_done);
  s.rec = (float*)(p + c->off_rec); s.last = (float*)(p + c->off_last);
  return s;
}

// One launch moves every array of a slab.  The element space [T][n][W] of the widest view (W = O + A + 4
// values per sample) is walked once; value w of a sample is its obs (w < O), act, logp, val, rew or done.
// to_slab != 0: experience buffer (column slice starting at the buffer's own base, row stride ld_envs) -> slab;
// to_slab == 0: slab columns [env0, env0 + take) -> buffer columns [col0, col0 + take).
// blockIdx.y selects one of the launch's slabs (pop stacks several).
struct MoveArgs {
  gmi_buffer_desc b;          // the experience buffer side
  SlabPtrs s[8];              // the slabs of this launch
  int n_slab_envs;            // envs per slab
  int env0, take, col0;       // pop: slice of every slab and first destination column; push: 0, n, 0
  int uni, to_slab;
  const float* last_src;      // push: bootstrap values of the agent [n]
  float* last_dst;            // pop: bootstrap values of the stacked batch
};

__global__ __launch_bounds__(256) void channel_move_kernel(MoveArgs a) {
  const int O = a.b.obs_dim, A = a.b.act_dim, W = O + A + 4, T = a.b.horizon;
  const SlabPtrs& S = a.s[blockIdx.y];
  const int n = a.n_slab_envs, take = a.take;
  const int64_t total = (int64_t)T * take * W;
  const int dcol = a.col0 + (int)blockIdx.y * take;      // pop: this slab's first column in the batch
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int w = (int)(i % W);
    const int64_t te = i / W;
    const int e = (int)(te % take), t = (int)(te / take);
    const int se = a.env0 + e;                                         // env inside the slab
    const int64_t sb = (int64_t)t * n + se;                            // sample index inside the slab
    const int64_t bb = (int64_t)t * a.b.ld_envs + (a.to_slab ? e : dcol + e);   // sample index inside the buffer
    if (a.to_slab) {
      float v;
      if (w < O) v = a.b.obs[bb * O + w];
      else if (w < O + A) v = a.b.act[bb * A + (w - O)];
      else if (w == O + A) v = a.b.logp[bb];
      else if (w == O + A + 1) v = a.b.val[bb];
      else if (w == O + A + 2) v = a.b.rew[bb];
      else v = (float)a.b.done[bb];
      if (a.uni) S.rec[sb * W + w] = v;
      else if (w < O) S.obs[sb * O + w] = v;
      else if (w < O + A) S.act[sb * A + (w - O)] = v;
      else if (w == O + A) S.logp[sb] = v;
      else if (w == O + A + 1) S.val[sb] = v;
      else if (w == O + A + 2) S.rew[sb] = v;
      else S.done[sb] = (uint8_t)v;
    } else {
      float v;
      if (a.uni) v = S.rec[sb * W + w];
      else if (w < O) v = S.obs[sb * O + w];
      else if (w < O + A) v = S.act[sb * A + (w - O)];
      else if (w == O + A) v = S.logp[sb];
      else if (w == O + A + 1) v = S.val[sb];
      else if (w == O + A + 2) v = S.rew[sb];
      else v = (float)S.done[sb];
      if (w < O) a.b.obs[bb * O + w] = v;
      else if (w < O + A) a.b.act[bb * A + (w - O)] = v;
      else if (w == O + A) a.b.logp[bb] = v;
      else if (w == O + A + 1) a.b.val[bb] = v;
      else if (w == O + A + 2) a.b.rew[bb] = v;
      else a.b.done[bb] = (uint8_t)v;
    }
  }
  // bootstrap values ride along
  for (int e = blockIdx.x * 256 + threadIdx.x; e < take; e += gridDim.x * 256) {
    if (a.to_slab) S.last[a.env0 + e] = a.last_src[e];
    else a.last_dst[(int)blockIdx.y * take + e] = S.last[a.env0 + e];
  }
}

size_t up256(size_t x) { return (x + 255) / 256 * 256; }
}  // namespace

extern "C" int gmi_channels_create(const gmi_channels_desc* d, int device, gmi_channels_t* out) {
  if (!d || !out) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_channels_create: NULL argument");
  *out = nullptr;
  if (d->horizon < 1 || d->n_envs < 1 || d->obs_dim < 1 || d->act_dim < 1 || d->capacity < 1 || d->capacity > 4096)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_channels_create: need horizon, n_envs, obs_dim, act_dim >= 1 and 1 <= capacity <= 4096");
  if (d->mode != GMI_CHANNELS_MULTI && d->mode != GMI_CHANNELS_UNI)
    GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_channels_create: unknown mode %d", d->mode);
  int n_dev = 0;
  GMI_HIP(hipGetDeviceCount(&n_dev));
  if (device < 0 || device >= n_dev) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_channels_create: device %d out of range", device);
  GMI_HIP(hipSetDevice(device));
  gmi_channels* c = new gmi_channels();
  c->magic = kMagicChannels;
  c->device = device;
  c->d = *d;
  const size_t TN = (size_t)d->horizon * d->n_envs;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off += up256(bytes); return o; };
  c->off_obs = c->off_act = c->off_logp = c->off_val = c->off_rew = c->off_done = c->off_rec = 0;
  if (d->mode == GMI_CHANNELS_MULTI) {
    c->off_obs = take(TN * d->obs_dim * 4);
    c->off_act = take(TN * d->act_dim * 4);
    c->off_logp = take(TN * 4);
    c->off_val = take(TN * 4);
    c->off_rew = take(TN * 4);
    c->off_done = take(TN);
  } else {
    c->off_rec = take(TN * (size_t)(d->obs_dim + d->act_dim + 4) * 4);
  }
  c->off_last = take((size_t)d->n_envs * 4);
  c->slab_bytes = off;
  c->head = c->count = 0;
  c->pushed = c->popped = 0;
  hipError_t e = hipMalloc((void**)&c->base, c->slab_bytes * d->capacity);
  if (e != hipSuccess) {
    delete c;
    GMI_FAIL(GMI_ERR_HIP, "gmi_channels_create: hipMalloc(%zu) failed: %s", off * d->capacity, hipGetErrorString(e));
  }
  c->filled.resize(d->capacity);
  c->freed.resize(d->capacity);
  c->was_popped.assign(d->capacity, 0);
  c->was_dropped.assign(d->capacity, 0);
  for (int i = 0; i < d->capacity; ++i) {
    if (hipEventCreateWithFlags(&c->filled[i], hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->freed[i], hipEventDisableTiming) != hipSuccess) {
      (void)hipFree(c->base);
      delete c;
      GMI_FAIL(GMI_ERR_HIP, "gmi_channels_create: event creation failed");
    }
  }
  *out = c;
  return GMI_OK;
}

extern "C" int gmi_channels_destroy(gmi_channels_t c) {
  if (!valid(c)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_channels_destroy: bad handle");
  (void)hipDeviceSynchronize();
  for (size_t i = 0; i < c->filled.size(); ++i) { (void)hipEventDestroy(c->filled[i]); (void)hipEventDestroy(c->freed[i]); }
  (void)hipFree(c->base);
  c->magic = 0;
  delete c;
  return GMI_OK;
}

extern "C" int gmi_channels_push(gmi_t g, gmi_channels_t c, gmi_buffer_t src, const float* last_value) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_channels_push: bad instance");
  if (!valid(c)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_channels_push: bad channels");
  if (!::valid(src)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_channels_push: bad buffer");
  if (!last_value) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_channels_push: last_value is NULL");
  const gmi_buffer_desc& b = src->d;
  if (b.horizon != c->d.horizon || b.n_envs != c->d.n_envs || b.obs_dim != c->d.obs_dim || b.act_dim != c->d.act_dim)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_channels_push: buffer [T %d, N %d, O %d, A %d] does not match the channels' slab [%d, %d, %d, %d]",
             b.horizon, b.n_envs, b.obs_dim, b.act_dim, c->d.horizon, c->d.n_envs, c->d.obs_dim, c->d.act_dim);
  std::lock_guard<std::mutex> hold(c->mu);
  if (c->count >= c->d.capacity) GMI_FAIL(GMI_ERR_UNSUPPORTED, "gmi_channels_push: all %d slabs are waiting for the trainer", c->d.capacity);
  if (g->device != c->device) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_channels_push: instance and channels live on different devices");
  const int slab = (c->head + c->count) % c->d.capacity;
  if (c->was_popped[slab]) GMI_HIP(hipStreamWaitEvent(g->stream, c->freed[slab], 0));   // the trainer has read it out
  if (c->was_dropped[slab]) {      // discarded unread: its writer (perhaps another agent's stream) must have finished
    GMI_HIP(hipStreamWaitEvent(g->stream, c->filled[slab], 0));
    c->was_dropped[slab] = 0;
  }
  MoveArgs a;
  a.b = b;
  for (int i = 0; i < 8; ++i) a.s[i] = slab_ptrs(c, slab);
  a.n_slab_envs = c->d.n_envs; a.env0 = 0; a.take = c->d.n_envs; a.col0 = 0;
  a.uni = c->d.mode == GMI_CHANNELS_UNI; a.to_slab = 1;
  a.last_src = last_value; a.last_dst = nullptr;
  const int64_t total = (int64_t)b.horizon * b.n_envs * (b.obs_dim + b.act_dim + 4);
  int64_t blocks = (total + 256 * 8 - 1) / (256 * 8);
  if (blocks > 4 * (int64_t)g->cu_count) blocks = 4 * (int64_t)g->cu_count;   // resident on the instance's CUs
  if (blocks < 1) blocks = 1;
  {
    gmi::ProfScope ps(g, gmi::kClsCollect);
    ps.launch(channel_move_kernel, dim3((unsigned)blocks, 1), dim3(256), 0, a);
  }
  GMI_LAUNCH_CHECK();
  GMI_HIP(hipEventRecord(c->filled[slab], g->stream));
  ++c->count;
  ++c->pushed;
  return GMI_OK;
}

extern "C" int gmi_channels_pop(gmi_t g, gmi_channels_t c, int32_t n_slabs, int32_t env0, int32_t take, gmi_buffer_t dst,
                                int32_t dst_col0, float* last_value_out) {
  if (!valid(g)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_channels_pop: bad instance");
  if (!valid(c)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_channels_pop: bad channels");
  if (!::valid(dst)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_channels_pop: bad buffer");
  if (!last_value_out) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_channels_pop: last_value_out is NULL");
  if (n_slabs < 1 || n_slabs > 8) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_channels_pop: 1 <= n_slabs <= 8 per call");
  std::lock_guard<std::mutex> hold(c->mu);
  if (n_slabs > c->count) GMI_FAIL(GMI_ERR_UNSUPPORTED, "gmi_channels_pop: %d slabs asked for, %d waiting", n_slabs, c->count);
  if (env0 < 0 || take < 1 || env0 + take > c->d.n_envs)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_channels_pop: slice [%d, %d) outside a slab's %d envs", env0, env0 + take, c->d.n_envs);
  const gmi_buffer_desc& b = dst->d;
  if (b.horizon != c->d.horizon || b.obs_dim != c->d.obs_dim || b.act_dim != c->d.act_dim)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_channels_pop: buffer and channels disagree on horizon / obs_dim / act_dim");
  if (dst_col0 < 0 || (int64_t)dst_col0 + (int64_t)n_slabs * take > b.n_envs)
    GMI_FAIL(GMI_ERR_BAD_SHAPE, "gmi_channels_pop: columns [%d, %lld) outside the buffer's %d envs", dst_col0,
             (long long)dst_col0 + (long long)n_slabs * take, b.n_envs);
  if (g->device != c->device) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_channels_pop: instance and channels live on different devices");
  MoveArgs a;
  a.b = b;
  for (int i = 0; i < 8; ++i) {
    const int slab = (c->head + (i < n_slabs ? i : 0)) % c->d.capacity;
    a.s[i] = slab_ptrs(c, slab);
    if (i < n_slabs) GMI_HIP(hipStreamWaitEvent(g->stream, c->filled[slab], 0));
  }
  a.n_slab_envs = c->d.n_envs; a.env0 = env0; a.take = take; a.col0 = dst_col0;
  a.uni = c->d.mode == GMI_CHANNELS_UNI; a.to_slab = 0;
  a.last_src = nullptr; a.last_dst = last_value_out;
  const int64_t total = (int64_t)b.horizon * take * (b.obs_dim + b.act_dim + 4);
  int64_t blocks = (total + 256 * 8 - 1) / (256 * 8);
  const int64_t cap = (4 * (int64_t)g->cu_count + n_slabs - 1) / n_slabs;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  {
    gmi::ProfScope ps(g, gmi::kClsCollect);
    ps.launch(channel_move_kernel, dim3((unsigned)blocks, (unsigned)n_slabs), dim3(256), 0, a);
  }
  GMI_LAUNCH_CHECK();
  for (int i = 0; i < n_slabs; ++i) {
    const int slab = (c->head + i) % c->d.capacity;
    GMI_HIP(hipEventRecord(c->freed[slab], g->stream));
    c->was_popped[slab] = 1;
  }
  c->head = (c->head + n_slabs) % c->d.capacity;
  c->count -= n_slabs;
  c->popped += n_slabs;
  return GMI_OK;
}

extern "C" int gmi_channels_drop(gmi_channels_t c, int32_t n_slabs) {
  if (!valid(c)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_channels_drop: bad handle");
  if (n_slabs < 0) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_channels_drop: n_slabs < 0");
  std::lock_guard<std::mutex> hold(c->mu);
  if (n_slabs > c->count) GMI_FAIL(GMI_ERR_UNSUPPORTED, "gmi_channels_drop: %d slabs to discard, %d waiting", n_slabs, c->count);
  for (int i = 0; i < n_slabs; ++i) c->was_dropped[(c->head + i) % c->d.capacity] = 1;
  c->head = (c->head + n_slabs) % c->d.capacity;
  c->count -= n_slabs;
  return GMI_OK;
}

extern "C" int gmi_channels_count(gmi_channels_t c, int32_t* waiting, int64_t* pushed, int64_t* popped) {
  if (!valid(c)) GMI_FAIL(GMI_ERR_BAD_HANDLE, "gmi_channels_count: bad handle");
  std::lock_guard<std::mutex> hold(c->mu);
  if (waiting) *waiting = c->count;
  if (pushed) *pushed = c->pushed;
  if (popped) *popped = c->popped;
  return GMI_OK;
}

extern "C" int gmi_route_least_loaded(const int64_t* samples_so_far, int32_t n_trainers, int32_t* trainer_out) {
  if (!samples_so_far || !trainer_out || n_trainers < 1) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_route_least_loaded: bad arguments");
  int best = 0;
  for (int i = 1; i < n_trainers; ++i)
    if (samples_so_far[i] < samples_so_far[best]) best = i;
  *trainer_out = best;
  return GMI_OK;
}
