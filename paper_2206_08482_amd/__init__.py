"""Python binding of libgmidrl (the MI355X-native PPO agent/trainer hot path of GMI-DRL).

Argument marshalling only: every function forwards to the C-ABI entry point of the same name
declared in ``include/gmidrl.h``; tensors are PyTorch CUDA(ROCm) tensors used purely as device
memory.  There is no fallback: if the HIP library is missing, importing this package fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgmidrl.so")

GMI_MAX_HIDDEN = 8
DTYPE_F32, DTYPE_BF16 = 0, 1
OK, ERR_INVALID_ARG, ERR_BAD_SHAPE, ERR_BAD_HANDLE, ERR_HIP, ERR_UNSUPPORTED = 0, -1, -2, -3, -4, -5
STREAM_ACTION, STREAM_ENV, STREAM_DONE, STREAM_RESET, STREAM_SHUFFLE = 0, 1, 2, 3, 4

EXPORTS = [
    "gmi_create", "gmi_destroy", "gmi_stream", "gmi_sync", "gmi_cu_count", "gmi_last_error",
    "gmi_wait_stream", "gmi_transfer", "gmi_model_param_count", "gmi_model_shadow_bytes", "gmi_model_bind",
    "gmi_model_destroy", "gmi_model_refresh_shadow", "gmi_env_bind", "gmi_env_destroy", "env_step",
    "agent_act", "agent_value", "gmi_fp8_bind", "gmi_fp8_refresh", "gmi_fp8_destroy", "agent_act_fp8", "gmi_buffer_bind", "gmi_buffer_destroy", "collect_experience",
    "gae_compute", "gae_compute_static", "ppo_update", "ppo_evaluate", "ppo_gradient", "adam_update", "gmi_noise_fill",
    "gmi_permutation", "gmi_profile_enable", "gmi_profile_classes", "gmi_profile_class_name", "gmi_profile_read",
    "gmi_measure_peak", "gmi_bench_linear", "gmi_bench_gae_variant", "gmi_set_fusion", "rollout_collect", "gmi_profile_work", "gmi_explore", "ppo_update_group", "gmi_select_reduction",
    "gmi_har_leaders", "gmi_reduction_time", "gmi_channels_create", "gmi_channels_destroy", "gmi_channels_push",
    "gmi_channels_pop", "gmi_channels_drop", "gmi_channels_count", "gmi_route_least_loaded",
]


PROFILE_FN = C.CFUNCTYPE(C.c_int, C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_double),
                        C.POINTER(C.c_double), C.c_void_p)
ESTIMATE_FN = C.CFUNCTYPE(C.c_double, C.c_int32, C.c_int32, C.c_double, C.c_void_p)


class GmiError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"gmidrl error {code}: {msg}")
        self.code = code


class ModelDesc(C.Structure):
    _fields_ = [("obs_dim", C.c_int32), ("act_dim", C.c_int32), ("n_hidden", C.c_int32),
                ("hidden", C.c_int32 * GMI_MAX_HIDDEN), ("dtype", C.c_int32), ("max_rows", C.c_int32)]


class EnvDesc(C.Structure):
    _fields_ = [("n_envs", C.c_int32), ("obs_dim", C.c_int32), ("act_dim", C.c_int32),
                ("noise_std", C.c_float), ("reward_scale", C.c_float), ("done_period", C.c_uint32),
                ("done_threshold", C.c_uint32), ("seed", C.c_uint64), ("env_offset", C.c_uint32)]


class BufferDesc(C.Structure):
    _fields_ = [("horizon", C.c_int32), ("n_envs", C.c_int32), ("ld_envs", C.c_int32),
                ("obs_dim", C.c_int32), ("act_dim", C.c_int32),
                ("obs", C.c_void_p), ("act", C.c_void_p), ("logp", C.c_void_p), ("val", C.c_void_p),
                ("rew", C.c_void_p), ("done", C.c_void_p), ("adv", C.c_void_p), ("ret", C.c_void_p)]


class ChannelsDesc(C.Structure):
    _fields_ = [("horizon", C.c_int32), ("n_envs", C.c_int32), ("obs_dim", C.c_int32), ("act_dim", C.c_int32),
                ("capacity", C.c_int32), ("mode", C.c_int32)]


class PPOHparams(C.Structure):
    _fields_ = [("clip", C.c_float), ("c_v", C.c_float), ("c_e", C.c_float), ("lr", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("adam_eps", C.c_float),
                ("epochs", C.c_int32), ("minibatch", C.c_int32), ("seed", C.c_uint64),
                ("iteration", C.c_uint32), ("adam_step0", C.c_uint32)]


def load_library(path: str = LIB_PATH) -> C.CDLL:
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2206_08482_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(path)
    vp, i32, u32, u64, f32, i64 = C.c_void_p, C.c_int32, C.c_uint32, C.c_uint64, C.c_float, C.c_int64
    sig = {
        "gmi_create": (C.c_int, [C.POINTER(C.c_uint32), u32, C.c_int, C.POINTER(vp)]),
        "gmi_destroy": (C.c_int, [vp]),
        "gmi_stream": (vp, [vp]),
        "gmi_sync": (C.c_int, [vp]),
        "gmi_cu_count": (C.c_int, [vp]),
        "gmi_last_error": (C.c_char_p, []),
        "gmi_transfer": (C.c_int, [vp, vp, vp, vp, C.c_size_t]),
        "gmi_model_param_count": (i64, [C.POINTER(ModelDesc)]),
        "gmi_model_shadow_bytes": (i64, [C.POINTER(ModelDesc)]),
        "gmi_model_bind": (C.c_int, [vp, C.POINTER(ModelDesc), vp, vp, vp, vp, C.POINTER(vp)]),
        "gmi_model_destroy": (C.c_int, [vp]),
        "gmi_model_refresh_shadow": (C.c_int, [vp, vp]),
        "gmi_env_bind": (C.c_int, [vp, C.POINTER(EnvDesc), vp, vp, vp, C.POINTER(vp)]),
        "gmi_env_destroy": (C.c_int, [vp]),
        "env_step": (C.c_int, [vp, vp, vp, vp, u32, vp, vp, vp]),
        "agent_act": (C.c_int, [vp, vp, vp, i32, u64, u32, u32, vp, vp, vp, vp]),
        "agent_value": (C.c_int, [vp, vp, vp, i32, vp]),
        "gmi_fp8_bind": (C.c_int, [vp, C.POINTER(ModelDesc), C.POINTER(vp)]),
        "gmi_fp8_refresh": (C.c_int, [vp, vp, vp]),
        "gmi_fp8_destroy": (C.c_int, [vp]),
        "agent_act_fp8": (C.c_int, [vp, vp, vp, i32, u64, u32, u32, vp, vp, vp, vp]),
        "gmi_buffer_bind": (C.c_int, [vp, C.POINTER(BufferDesc), C.POINTER(vp)]),
        "gmi_buffer_destroy": (C.c_int, [vp]),
        "collect_experience": (C.c_int, [vp, vp, i32, vp, vp, vp, vp, vp, vp]),
        "rollout_collect": (C.c_int, [vp, vp, vp, vp, vp, u64, u32, u32, vp]),
        "gae_compute": (C.c_int, [vp, vp, vp, f32, f32, C.c_int]),
        "gae_compute_static": (C.c_int, [vp, i32, i32, i32, vp, vp, vp, vp, f32, f32, C.c_int, vp, vp]),
        "ppo_update": (C.c_int, [vp, vp, vp, C.POINTER(PPOHparams), vp]),
        "ppo_update_group": (C.c_int, [C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), i32, C.POINTER(PPOHparams), vp]),
        "ppo_evaluate": (C.c_int, [vp, vp, vp, C.POINTER(PPOHparams), vp, i32, vp]),
        "gmi_channels_create": (C.c_int, [C.POINTER(ChannelsDesc), C.c_int, C.POINTER(vp)]),
        "gmi_channels_destroy": (C.c_int, [vp]),
        "gmi_channels_push": (C.c_int, [vp, vp, vp, vp]),
        "gmi_channels_pop": (C.c_int, [vp, vp, i32, i32, i32, vp, i32, vp]),
        "gmi_channels_drop": (C.c_int, [vp, i32]),
        "gmi_channels_count": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i64), C.POINTER(i64)]),
        "gmi_route_least_loaded": (C.c_int, [C.POINTER(i64), i32, C.POINTER(i32)]),
        "gmi_select_reduction": (C.c_int, [C.POINTER(i32), i32, C.POINTER(i32)]),
        "gmi_har_leaders": (C.c_int, [C.POINTER(i32), C.POINTER(i32), i32, i32, C.POINTER(i32)]),
        "gmi_reduction_time": (C.c_int, [i32, i32, i32, C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double)]),
        "ppo_gradient": (C.c_int, [vp, vp, vp, C.POINTER(PPOHparams), vp, i32, vp, vp]),
        "adam_update": (C.c_int, [vp, vp, vp, vp, vp, i64, C.POINTER(PPOHparams), u32]),
        "gmi_noise_fill": (C.c_int, [vp, u64, u32, u32, u32, i32, i32, vp]),
        "gmi_permutation": (C.c_int, [vp, i32, u64, u32, u32, vp]),
        "gmi_profile_enable": (C.c_int, [vp, u32]),
        "gmi_profile_classes": (C.c_int, []),
        "gmi_profile_class_name": (C.c_char_p, [C.c_int]),
        "gmi_profile_read": (C.c_int, [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(i64)]),
        "gmi_set_fusion": (C.c_int, [vp, C.c_int]),
        "gmi_bench_gae_variant": (C.c_int, [C.c_int]),
        "gmi_wait_stream": (C.c_int, [vp, vp]),
        "gmi_explore": (C.c_int, [PROFILE_FN, vp, ESTIMATE_FN, vp, i32, C.c_double, C.POINTER(i32), i32,
                                  C.POINTER(i32), i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_double)]),
        "gmi_profile_work": (C.c_int, [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
        "gmi_measure_peak": (C.c_int, [vp, C.c_int, vp, C.c_size_t, C.POINTER(C.c_double)]),
        "gmi_bench_linear": (C.c_int, [vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, vp, C.c_size_t,
                                       C.POINTER(C.c_double)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


class _Lazy:
    """Loads libgmidrl.so on first use (so that `python -m paper_2206_08482_amd.build` can import the
    package before the library exists); a missing library raises ImportError at that point."""
    _lib = None

    def __getattr__(self, name):
        if _Lazy._lib is None:
            _Lazy._lib = load_library()
        return getattr(_Lazy._lib, name)


_lib = _Lazy()


def last_error() -> str:
    return _lib.gmi_last_error().decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise GmiError(rc, last_error())


def _ptr(t) -> Optional[int]:
    """Device pointer of a tensor (None passes NULL); tensors must be contiguous CUDA tensors."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise TypeError("expected a device tensor")
    if not t.is_contiguous():
        raise TypeError("expected a contiguous tensor")
    return t.data_ptr()


# ---------------------------------------------------------------- instances
def gmi_create(cu_mask: Optional[Sequence[int]] = None, device: int = 0) -> int:
    out = C.c_void_p()
    if cu_mask is None:
        _check(_lib.gmi_create(None, 0, device, C.byref(out)))
    else:
        arr = (C.c_uint32 * len(cu_mask))(*cu_mask)
        _check(_lib.gmi_create(arr, len(cu_mask), device, C.byref(out)))
    return out.value


def gmi_destroy(gmi: int) -> None:
    _check(_lib.gmi_destroy(gmi))


def gmi_stream(gmi: int) -> int:
    return _lib.gmi_stream(gmi)


def gmi_sync(gmi: int) -> None:
    _check(_lib.gmi_sync(gmi))


def gmi_cu_count(gmi: int) -> int:
    rc = _lib.gmi_cu_count(gmi)
    if rc < 0:
        _check(rc)
    return rc


def gmi_transfer(src: int, dst: int, src_t=None, dst_t=None, nbytes: int = 0) -> None:
    _check(_lib.gmi_transfer(src, dst, _ptr(src_t), _ptr(dst_t), nbytes))


# ---------------------------------------------------------------- model
def model_desc(obs_dim: int, act_dim: int, hidden: Sequence[int], dtype: int, max_rows: int) -> ModelDesc:
    d = ModelDesc()
    d.obs_dim, d.act_dim, d.n_hidden, d.dtype, d.max_rows = obs_dim, act_dim, len(hidden), dtype, max_rows
    for i, h in enumerate(hidden[:GMI_MAX_HIDDEN]):
        d.hidden[i] = h
    return d


def gmi_model_param_count(desc: ModelDesc) -> int:
    n = _lib.gmi_model_param_count(C.byref(desc))
    if n < 0:
        _check(int(n))
    return n


def gmi_model_shadow_bytes(desc: ModelDesc) -> int:
    n = _lib.gmi_model_shadow_bytes(C.byref(desc))
    if n < 0:
        _check(int(n))
    return n


def gmi_model_bind(gmi: int, desc: ModelDesc, params, shadow=None, adam_m=None, adam_v=None) -> int:
    out = C.c_void_p()
    _check(_lib.gmi_model_bind(gmi, C.byref(desc), _ptr(params), _ptr(shadow), _ptr(adam_m),
                               _ptr(adam_v), C.byref(out)))
    return out.value


def gmi_model_destroy(model: int) -> None:
    _check(_lib.gmi_model_destroy(model))


def gmi_model_refresh_shadow(gmi: int, model: int) -> None:
    _check(_lib.gmi_model_refresh_shadow(gmi, model))


# ---------------------------------------------------------------- environment
def env_desc(n_envs, obs_dim, act_dim, noise_std, reward_scale, done_period, done_threshold, seed,
             env_offset=0) -> EnvDesc:
    d = EnvDesc()
    d.n_envs, d.obs_dim, d.act_dim = n_envs, obs_dim, act_dim
    d.noise_std, d.reward_scale = noise_std, reward_scale
    d.done_period, d.done_threshold, d.seed, d.env_offset = done_period, done_threshold, seed, env_offset
    return d


def gmi_env_bind(gmi: int, desc: EnvDesc, a_mat, b_mat, episode_step) -> int:
    out = C.c_void_p()
    _check(_lib.gmi_env_bind(gmi, C.byref(desc), _ptr(a_mat), _ptr(b_mat), _ptr(episode_step), C.byref(out)))
    return out.value


def gmi_env_destroy(env: int) -> None:
    _check(_lib.gmi_env_destroy(env))


def env_step(gmi: int, env: int, obs, act, step: int, next_obs, reward, done) -> None:
    _check(_lib.env_step(gmi, env, _ptr(obs), _ptr(act), step, _ptr(next_obs), _ptr(reward), _ptr(done)))


# ---------------------------------------------------------------- agent
def agent_act(gmi: int, model: int, obs, n_rows: int, seed: int, step: int, env_offset: int, act, logp,
              value, mu=None) -> None:
    _check(_lib.agent_act(gmi, model, _ptr(obs), n_rows, seed, step, env_offset, _ptr(act), _ptr(logp),
                          _ptr(value), _ptr(mu)))


def agent_value(gmi: int, model: int, obs, n_rows: int, value) -> None:
    _check(_lib.agent_value(gmi, model, _ptr(obs), n_rows, _ptr(value)))


def gmi_fp8_bind(gmi: int, desc: ModelDesc) -> int:
    out = C.c_void_p()
    _check(_lib.gmi_fp8_bind(gmi, C.byref(desc), C.byref(out)))
    return out.value


def gmi_fp8_refresh(gmi: int, weights: int, params) -> None:
    _check(_lib.gmi_fp8_refresh(gmi, weights, _ptr(params)))


def gmi_fp8_destroy(weights: int) -> None:
    _check(_lib.gmi_fp8_destroy(weights))


def agent_act_fp8(gmi: int, weights: int, obs, n_rows: int, seed: int, step: int, env_offset: int, act, logp,
                  value, mu=None) -> None:
    _check(_lib.agent_act_fp8(gmi, weights, _ptr(obs), n_rows, seed, step, env_offset, _ptr(act), _ptr(logp),
                              _ptr(value), _ptr(mu)))


# ---------------------------------------------------------------- experience
def buffer_desc(horizon, n_envs, ld_envs, obs_dim, act_dim, obs, act, logp, val, rew, done, adv, ret) -> BufferDesc:
    d = BufferDesc()
    d.horizon, d.n_envs, d.ld_envs, d.obs_dim, d.act_dim = horizon, n_envs, ld_envs, obs_dim, act_dim
    d.obs, d.act, d.logp, d.val = _ptr(obs), _ptr(act), _ptr(logp), _ptr(val)
    d.rew, d.done, d.adv, d.ret = _ptr(rew), _ptr(done), _ptr(adv), _ptr(ret)
    return d


def gmi_buffer_bind(gmi: int, desc: BufferDesc) -> int:
    out = C.c_void_p()
    _check(_lib.gmi_buffer_bind(gmi, C.byref(desc), C.byref(out)))
    return out.value


def gmi_buffer_destroy(buf: int) -> None:
    _check(_lib.gmi_buffer_destroy(buf))


def collect_experience(gmi: int, buf: int, t: int, obs, act, logp, value, reward, done) -> None:
    _check(_lib.collect_experience(gmi, buf, t, _ptr(obs), _ptr(act), _ptr(logp), _ptr(value),
                                   _ptr(reward), _ptr(done)))


def rollout_collect(gmi: int, model: int, env: int, buf: int, obs, seed: int, step0: int, env_offset: int,
                    last_value) -> None:
    _check(_lib.rollout_collect(gmi, model, env, buf, _ptr(obs), seed, step0, env_offset, _ptr(last_value)))


def gae_compute(gmi: int, buf: int, last_value, gamma: float, lam: float, normalize: bool) -> None:
    _check(_lib.gae_compute(gmi, buf, _ptr(last_value), gamma, lam, 1 if normalize else 0))


def gae_compute_static(gmi: int, horizon: int, n_envs: int, ld_envs: int, rew, val, done, last_value, gamma: float,
                       lam: float, normalize: bool, adv, ret) -> None:
    _check(_lib.gae_compute_static(gmi, horizon, n_envs, ld_envs, _ptr(rew), _ptr(val), _ptr(done), _ptr(last_value),
                                   gamma, lam, 1 if normalize else 0, _ptr(adv), _ptr(ret)))


# ---------------------------------------------------------------- trainer
def ppo_hparams(clip=0.2, c_v=0.5, c_e=0.0, lr=3e-4, beta1=0.9, beta2=0.999, adam_eps=1e-8, epochs=1,
                minibatch=256, seed=0, iteration=0, adam_step0=0) -> PPOHparams:
    h = PPOHparams()
    h.clip, h.c_v, h.c_e, h.lr, h.beta1, h.beta2, h.adam_eps = clip, c_v, c_e, lr, beta1, beta2, adam_eps
    h.epochs, h.minibatch, h.seed, h.iteration, h.adam_step0 = epochs, minibatch, seed, iteration, adam_step0
    return h


def ppo_update(gmi: int, model: int, buf: int, hp: PPOHparams, stats_out=None) -> None:
    _check(_lib.ppo_update(gmi, model, buf, C.byref(hp), _ptr(stats_out)))


def ppo_update_group(gmis, models, bufs, hp: PPOHparams, stats_out=None) -> None:
    n = len(gmis)
    if len(models) != n or len(bufs) != n:
        raise ValueError("ppo_update_group: one model and one buffer per instance")
    arr = lambda xs: (C.c_void_p * n)(*xs)
    _check(_lib.ppo_update_group(arr(gmis), arr(models), arr(bufs), n, C.byref(hp), _ptr(stats_out)))


CHANNELS_MULTI, CHANNELS_UNI = 0, 1


def gmi_channels_create(horizon: int, n_envs: int, obs_dim: int, act_dim: int, capacity: int, mode: int = CHANNELS_MULTI,
                        device: int = 0) -> int:
    d = ChannelsDesc(horizon, n_envs, obs_dim, act_dim, capacity, mode)
    out = C.c_void_p()
    _check(_lib.gmi_channels_create(C.byref(d), device, C.byref(out)))
    return out.value


def gmi_channels_destroy(ch: int) -> None:
    _check(_lib.gmi_channels_destroy(ch))


def gmi_channels_push(agent: int, ch: int, src_buffer: int, last_value) -> None:
    _check(_lib.gmi_channels_push(agent, ch, src_buffer, _ptr(last_value)))


def gmi_channels_pop(trainer: int, ch: int, n_slabs: int, env0: int, take: int, dst_buffer: int, dst_col0: int,
                     last_value_out) -> None:
    _check(_lib.gmi_channels_pop(trainer, ch, n_slabs, env0, take, dst_buffer, dst_col0, _ptr(last_value_out)))


def gmi_channels_drop(ch: int, n_slabs: int) -> None:
    _check(_lib.gmi_channels_drop(ch, n_slabs))


def gmi_channels_count(ch: int):
    w, a, b = C.c_int32(0), C.c_int64(0), C.c_int64(0)
    _check(_lib.gmi_channels_count(ch, C.byref(w), C.byref(a), C.byref(b)))
    return w.value, a.value, b.value


def gmi_route_least_loaded(samples_so_far) -> int:
    n = len(samples_so_far)
    arr = (C.c_int64 * n)(*[int(x) for x in samples_so_far])
    out = C.c_int32(-1)
    _check(_lib.gmi_route_least_loaded(arr, n, C.byref(out)))
    return out.value


REDUCE_MULTI_PROCESS, REDUCE_MULTI_RING, REDUCE_HIERARCHICAL = 0, 1, 2


def gmi_select_reduction(mpl) -> int:
    """mpl: the GMI-to-GPU mapping list (ids of the trainer instances GPU by GPU)."""
    counts = (C.c_int32 * max(len(mpl), 1))(*[len(x) for x in mpl])
    out = C.c_int32(-1)
    _check(_lib.gmi_select_reduction(counts, len(mpl), C.byref(out)))
    return out.value


def gmi_har_leaders(mpl, t: int):
    ids = [i for li in mpl for i in li]
    start = [0]
    for li in mpl:
        start.append(start[-1] + len(li))
    a = (C.c_int32 * max(len(ids), 1))(*ids)
    b = (C.c_int32 * len(start))(*start)
    out = (C.c_int32 * max(len(mpl), 1))()
    _check(_lib.gmi_har_leaders(a, b, len(mpl), t, out))
    return [None if out[p] < 0 else out[p] for p in range(len(mpl))]


def gmi_reduction_time(strategy: int, g: int, t: int, m_p: float, b1: float, b2: float) -> float:
    out = C.c_double(0.0)
    _check(_lib.gmi_reduction_time(strategy, g, t, m_p, b1, b2, C.byref(out)))
    return out.value


def ppo_evaluate(gmi: int, model: int, buf: int, hp: PPOHparams, idx, n: int, stats_out) -> None:
    _check(_lib.ppo_evaluate(gmi, model, buf, C.byref(hp), _ptr(idx), n, _ptr(stats_out)))


def ppo_gradient(gmi: int, model: int, buf: int, hp: PPOHparams, idx, n: int, grad_out, stats_out=None) -> None:
    _check(_lib.ppo_gradient(gmi, model, buf, C.byref(hp), _ptr(idx), n, _ptr(grad_out), _ptr(stats_out)))


def adam_update(gmi: int, params, adam_m, adam_v, grad, n: int, hp: PPOHparams, step: int) -> None:
    _check(_lib.adam_update(gmi, _ptr(params), _ptr(adam_m), _ptr(adam_v), _ptr(grad), n, C.byref(hp), step))


# ---------------------------------------------------------------- utilities
def gmi_noise_fill(gmi: int, seed: int, stream: int, step: int, env_offset: int, n_envs: int, dim: int, out) -> None:
    _check(_lib.gmi_noise_fill(gmi, seed, stream, step, env_offset, n_envs, dim, _ptr(out)))


def gmi_permutation(gmi: int, n: int, seed: int, iteration: int, epoch: int, out) -> None:
    _check(_lib.gmi_permutation(gmi, n, seed, iteration, epoch, _ptr(out)))


# ---------------------------------------------------------------- per-launch timing
def gmi_profile_classes() -> int:
    return _lib.gmi_profile_classes()


def gmi_profile_class_name(cls: int) -> Optional[str]:
    n = _lib.gmi_profile_class_name(cls)
    return n.decode() if n else None


def gmi_profile_enable(gmi: int, class_mask: int) -> None:
    _check(_lib.gmi_profile_enable(gmi, class_mask))


def gmi_profile_read(gmi: int, cls: int):
    """(total milliseconds, launches) of kernel class `cls` since profiling was enabled."""
    ms, n = C.c_double(), C.c_int64()
    _check(_lib.gmi_profile_read(gmi, cls, C.byref(ms), C.byref(n)))
    return ms.value, n.value


def gmi_profile_work(gmi: int, cls: int):
    """(flops, bytes) of algorithmic work stated by the launchers of class `cls` while it was timed."""
    fl, by = C.c_double(), C.c_double()
    _check(_lib.gmi_profile_work(gmi, cls, C.byref(fl), C.byref(by)))
    return fl.value, by.value


def gmi_explore(profile, num_gpu: int, alpha: float, gmi_per_gpu_values, num_env_values, estimate=None):
    """Algorithm 2 through the C ABI.  profile(gmi_per_gpu, num_env) -> (runnable, throughput, memory);
    estimate(gmi_per_gpu, num_gpu, throughput) -> projected throughput (None: the library's default).
    Returns (num_env, gmi_per_gpu, projected) or None if no point was recorded."""
    failure = []

    def _profile(k, n, runnable, top, mem, _user):
        try:
            r, t, m = profile(int(k), int(n))
            runnable[0], top[0], mem[0] = (1 if r else 0), float(t), float(m)
            return 0
        except Exception as e:           # an exception cannot cross the C frame: report it afterwards
            failure.append(e)
            return 1

    def _estimate(k, g, top, _user):
        return float(estimate(int(k), int(g), float(top)))

    cb_p = PROFILE_FN(_profile)
    cb_e = ESTIMATE_FN(_estimate) if estimate is not None else C.cast(None, ESTIMATE_FN)
    ks = (C.c_int32 * len(gmi_per_gpu_values))(*gmi_per_gpu_values)
    ns = (C.c_int32 * len(num_env_values))(*num_env_values)
    out_n, out_k, out_p = C.c_int32(), C.c_int32(), C.c_double()
    rc = _lib.gmi_explore(cb_p, None, cb_e, None, num_gpu, alpha, ks, len(gmi_per_gpu_values), ns,
                          len(num_env_values), C.byref(out_n), C.byref(out_k), C.byref(out_p))
    if failure:
        raise failure[0]
    _check(rc)
    if out_n.value == 0 and out_k.value == 0:
        return None
    return out_n.value, out_k.value, out_p.value


def dtype_code(name: str) -> int:
    return {"f32": DTYPE_F32, "bf16": DTYPE_BF16}[name]


def gmi_measure_peak(gmi: int, what: int, scratch) -> float:
    """what = 0: sustained bf16 MFMA TFLOP/s; what = 1: streaming-copy GB/s over `scratch` (a device tensor)."""
    out = C.c_double()
    _check(_lib.gmi_measure_peak(gmi, what, _ptr(scratch), scratch.numel() * scratch.element_size(), C.byref(out)))
    return out.value


def gmi_bench_linear(gmi: int, kind: int, rows: int, K: int, F: int, n_nets: int, reps: int, scratch) -> float:
    """Average microseconds per launch of one bf16 layer product (kind 0 forward, 2 input grad, 3 weight grad)."""
    out = C.c_double()
    _check(_lib.gmi_bench_linear(gmi, kind, rows, K, F, n_nets, reps, _ptr(scratch),
                                 scratch.numel() * scratch.element_size(), C.byref(out)))
    return out.value


def gmi_bench_gae_variant(variant: int) -> None:
    """0: serial walk (default); 1: wavefront scan."""
    _check(_lib.gmi_bench_gae_variant(int(variant)))


def gmi_set_fusion(gmi: int, level: int) -> None:
    """0: one launch per layer; otherwise (default) the one-launch agent, rollout and trainer kernels where the
    model has them."""
    _check(_lib.gmi_set_fusion(gmi, int(level)))


def gmi_wait_stream(gmi: int, stream=None) -> None:
    """Orders the instance behind everything queued so far on `stream` (a torch.cuda.Stream or a raw stream
    handle; None: torch's current stream)."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    handle = getattr(stream, "cuda_stream", stream)
    _check(_lib.gmi_wait_stream(gmi, C.c_void_p(int(handle) if handle else None)))
