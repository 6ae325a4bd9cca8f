"""Thin ctypes binding of libmi355env.so: same names as include/mi355env.h, argument marshalling
only.  Tensors are PyTorch device tensors (PyTorch provides device memory and streams, nothing
else); every step of the path runs inside the library's HIP kernels.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

ENV_PONG, ENV_PONG_PIXELS, ENV_BODY, ENV_CARTPOLE = 0, 1, 2, 3
ENV_PIXELS_SLOT_MAJOR, ENV_PIXELS_ENV_MAJOR, ENV_PIXELS_ORDERED = 1, 2, 3
ENV_STEP_COUNTER_HOST, ENV_STEP_COUNTER_DEVICE = 1, 2
ENV_OBS_RAW, ENV_OBS_NORMALIZED = 1, 2
ENV_CONTACT_PENALTY, ENV_CONTACT_NEWTON = 1, 2
ENV_PIXELS_FULL, ENV_PIXELS_DELTA = 1, 2
ENV_BODY_F64, ENV_BODY_F32 = 1, 2
ENV_OK, ENV_E_ARG, ENV_E_ALLOC, ENV_E_HIP, ENV_E_STATE, ENV_E_UNSUPPORTED, ENV_E_TOO_LARGE = 0, -1, -2, -3, -4, -5, -6
ENV_NOALLOC_MAX_ENVS = 65536

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmi355env.so")
_lib = None


class env_config_t(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("max_score", C.c_int32),
                ("max_episode_steps", C.c_int32), ("armature", C.c_float),
                ("joint_damping", C.c_float), ("friction_mu", C.c_float),
                ("pixel_layout", C.c_int32), ("step_counter", C.c_int32),
                ("obs_scaling", C.c_int32), ("contact_solver", C.c_int32),
                ("pixel_update", C.c_int32), ("body_arithmetic", C.c_int32)]


class env_stats_t(C.Structure):
    _fields_ = [("episodes", C.c_int64), ("length_sum", C.c_int64), ("return_sum", C.c_double),
                ("return_min", C.c_double), ("return_max", C.c_double), ("nonfinite", C.c_int64)]


class EnvError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__("%s failed: %d (%s)" % (what, code, env_strerror(code)))


def lib():
    """Load the shared library (never builds it: run paper_2603_12145_amd/build.py first)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libmi355env.so is not built; run `python paper_2603_12145_amd/build.py`")
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.env_create.argtypes = [C.POINTER(vp), C.c_int, C.c_int64, C.c_uint64,
                                 C.POINTER(env_config_t), vp]
        L.env_destroy.argtypes = [vp]; L.env_destroy.restype = None
        L.env_reset.argtypes = [vp, vp]
        L.env_step.argtypes = [vp, vp, vp, vp, vp]
        L.env_rollout.argtypes = [vp, C.c_int32, vp, vp, vp, vp]
        L.env_stats.argtypes = [vp, C.POINTER(env_stats_t), C.c_int]
        L.env_state_bytes.argtypes = [vp]; L.env_state_bytes.restype = C.c_size_t
        L.env_get_state.argtypes = [vp, vp, C.c_size_t]
        L.env_set_state.argtypes = [vp, vp, C.c_size_t]
        L.env_obs_dim.argtypes = [C.c_int]
        L.env_action_dim.argtypes = [C.c_int]
        L.env_num_envs.argtypes = [vp]; L.env_num_envs.restype = C.c_int64
        L.env_step_count.argtypes = [vp]; L.env_step_count.restype = C.c_uint64
        L.env_set_stream.argtypes = [vp, vp]
        L.env_strerror.argtypes = [C.c_int]; L.env_strerror.restype = C.c_char_p
        L.env_step_pixels_noalloc.argtypes = [C.c_int64, C.c_uint64, C.c_uint64, C.c_int32, vp, vp, vp, vp, vp,
                                              vp, vp]
        L.env_step_pixels_noalloc.restype = C.c_int
        for f in (L.env_create, L.env_reset, L.env_step, L.env_rollout, L.env_stats,
                  L.env_get_state, L.env_set_state, L.env_obs_dim, L.env_action_dim,
                  L.env_set_stream):
            f.restype = C.c_int
        _lib = L
    return _lib


def _dev_ptr(t):
    """Device address of a tensor (or None / a raw integer address)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise TypeError("expected a device tensor")
    if not t.is_contiguous():
        raise TypeError("expected a contiguous tensor")
    return t.data_ptr()


def _check(code, what):
    if code != ENV_OK:
        raise EnvError(code, what)


def env_strerror(code):
    return lib().env_strerror(int(code)).decode()


def env_create(kind, n_envs, seed, cfg=None, stream=None):
    """cfg: dict of env_config_t fields (missing = default); stream: torch.cuda.Stream or None
    (None = torch's current stream).  Returns the opaque handle."""
    import torch
    c = None
    if cfg is not None:
        c = env_config_t(struct_size=C.sizeof(env_config_t), max_score=0, max_episode_steps=0,
                         armature=-1.0, joint_damping=-1.0, friction_mu=-1.0, pixel_layout=0,
                         step_counter=0, obs_scaling=0, contact_solver=0, pixel_update=0, body_arithmetic=0)
        for k, v in cfg.items():
            setattr(c, k, v)
    s = torch.cuda.current_stream() if stream is None else stream
    h = C.c_void_p()
    _check(lib().env_create(C.byref(h), int(kind), int(n_envs), int(seed),
                            None if c is None else C.byref(c), C.c_void_p(s.cuda_stream)),
           "env_create")
    return h


def env_destroy(h):
    lib().env_destroy(h)


def env_reset(h, obs=None):
    _check(lib().env_reset(h, _dev_ptr(obs)), "env_reset")


def env_step(h, actions, obs, reward, done):
    _check(lib().env_step(h, _dev_ptr(actions), _dev_ptr(obs), _dev_ptr(reward), _dev_ptr(done)),
           "env_step")


class PreparedStep:
    """env_step with its arguments marshalled once, for loops that call it with the same buffers
    every step: `step = PreparedStep(h, actions, obs, reward, done); step()`.  Taking the four device
    addresses out of tensors costs about 0.6 us of host time per call, which matters wherever the
    host's share of a call is what bounds the loop (small batches launched with kernel arguments).
    The tensors are kept alive by the object."""

    def __init__(self, h, actions, obs, reward, done):
        self._keep = (actions, obs, reward, done)
        self._call = lib().env_step
        self._args = (h, _dev_ptr(actions), _dev_ptr(obs), _dev_ptr(reward), _dev_ptr(done))

    def __call__(self):
        code = self._call(*self._args)
        if code != ENV_OK:
            raise EnvError(code, "env_step")


def env_rollout(h, T, actions, obs, reward, done):
    _check(lib().env_rollout(h, int(T), _dev_ptr(actions), _dev_ptr(obs), _dev_ptr(reward),
                             _dev_ptr(done)), "env_rollout")


def env_stats(h, reset_counters=False):
    s = env_stats_t()
    _check(lib().env_stats(h, C.byref(s), int(bool(reset_counters))), "env_stats")
    return {k: getattr(s, k) for k, _ in env_stats_t._fields_}


def env_state_bytes(h):
    return int(lib().env_state_bytes(h))


def env_get_state(h):
    """Returns the state blob as a numpy uint8 array (host)."""
    import numpy as np
    buf = np.empty(env_state_bytes(h), np.uint8)
    _check(lib().env_get_state(h, buf.ctypes.data_as(C.c_void_p), buf.nbytes), "env_get_state")
    return buf


def env_set_state(h, blob):
    import numpy as np
    blob = np.ascontiguousarray(blob, np.uint8)
    _check(lib().env_set_state(h, blob.ctypes.data_as(C.c_void_p), blob.nbytes), "env_set_state")


def env_obs_dim(kind):
    return int(lib().env_obs_dim(int(kind)))


def env_action_dim(kind):
    return int(lib().env_action_dim(int(kind)))


def env_num_envs(h):
    return int(lib().env_num_envs(h))


def env_step_count(h):
    return int(lib().env_step_count(h))


def env_set_stream(h, stream):
    """stream: torch.cuda.Stream (or a raw hipStream_t address)."""
    addr = stream if isinstance(stream, int) else stream.cuda_stream
    _check(lib().env_set_stream(h, C.c_void_p(addr)), "env_set_stream")


def env_step_pixels_noalloc(n_envs, seed, step, max_score, state, actions, ring, reward, done, stats=None,
                            stream=None):
    """state: uint32/int32 device tensor [10, n] (in/out); stats: optional device tensor of 48 bytes
    (an env_stats_t); stream: torch.cuda.Stream or None (torch's current stream)."""
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    _check(lib().env_step_pixels_noalloc(int(n_envs), int(seed), int(step), int(max_score), _dev_ptr(state),
                                         _dev_ptr(actions), _dev_ptr(ring), _dev_ptr(reward), _dev_ptr(done),
                                         _dev_ptr(stats), C.c_void_p(s.cuda_stream)), "env_step_pixels_noalloc")

