"""ctypes wrapper of the CartPole oracle (TEST INFRASTRUCTURE)."""
import ctypes as C

import numpy as np

ENV_DTYPE = np.dtype([("x", "f4"), ("xd", "f4"), ("th", "f4"), ("thd", "f4"), ("ep_len", "i4")])


class Stats(C.Structure):
    _fields_ = [("episodes", C.c_int64), ("length_sum", C.c_int64), ("length_min", C.c_int32),
                ("length_max", C.c_int32)]


def _lib():
    from oracle import oracle as orc
    L = orc.lib()
    if not getattr(L, "_cartpole_bound", False):
        vp = C.c_void_p
        L.oracle_cartpole_sin.argtypes = [C.c_float]; L.oracle_cartpole_sin.restype = C.c_float
        L.oracle_cartpole_cos.argtypes = [C.c_float]; L.oracle_cartpole_cos.restype = C.c_float
        L.oracle_cartpole_accel.argtypes = [C.c_float, C.c_float, C.c_float, C.POINTER(C.c_float), C.POINTER(C.c_float)]
        L.oracle_cartpole_create.argtypes = [C.c_int64, C.c_uint64, C.c_int32]; L.oracle_cartpole_create.restype = vp
        L.oracle_cartpole_destroy.argtypes = [vp]
        L.oracle_cartpole_envs.argtypes = [vp]; L.oracle_cartpole_envs.restype = vp
        L.oracle_cartpole_step_count.argtypes = [vp]; L.oracle_cartpole_step_count.restype = C.c_uint64
        L.oracle_cartpole_set_step_count.argtypes = [vp, C.c_uint64]
        L.oracle_cartpole_get_stats.argtypes = [vp, C.POINTER(Stats), C.c_int32]
        L.oracle_cartpole_reset.argtypes = [vp, vp]
        L.oracle_cartpole_rollout.argtypes = [vp, C.c_int32, vp, vp, vp, vp, C.c_int32]
        L._cartpole_bound = True
    return L


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def accel(th, thd, force):
    xa, ta = C.c_float(), C.c_float()
    _lib().oracle_cartpole_accel(th, thd, force, C.byref(xa), C.byref(ta))
    return xa.value, ta.value


def sin_poly(x):
    return _lib().oracle_cartpole_sin(x)


def cos_poly(x):
    return _lib().oracle_cartpole_cos(x)


class CartPole:
    def __init__(self, n, seed, max_steps=500):
        self.L = _lib()
        self.n, self.seed = int(n), int(seed)
        self.h = self.L.oracle_cartpole_create(self.n, self.seed, int(max_steps))

    def __del__(self):
        if getattr(self, "h", None):
            self.L.oracle_cartpole_destroy(self.h)
            self.h = None

    def envs(self):
        addr = self.L.oracle_cartpole_envs(self.h)
        buf = (C.c_char * (ENV_DTYPE.itemsize * self.n)).from_address(addr)
        return np.frombuffer(buf, dtype=ENV_DTYPE)

    @property
    def step_count(self):
        return int(self.L.oracle_cartpole_step_count(self.h))

    @step_count.setter
    def step_count(self, v):
        self.L.oracle_cartpole_set_step_count(self.h, int(v))

    def reset(self):
        obs = np.empty((self.n, 4), np.float32)
        self.L.oracle_cartpole_reset(self.h, _p(obs))
        return obs

    def rollout(self, T, actions=None, nthreads=1):
        obs = np.empty((T, self.n, 4), np.float32)
        rew = np.empty((T, self.n), np.float32)
        done = np.empty((T, self.n), np.uint8)
        if actions is not None:
            actions = np.ascontiguousarray(actions, np.uint8)
            assert actions.shape == (T, self.n)
        self.L.oracle_cartpole_rollout(self.h, T, _p(actions), _p(obs), _p(rew), _p(done), nthreads)
        return obs, rew, done

    def stats(self, clear=False):
        s = Stats()
        self.L.oracle_cartpole_get_stats(self.h, C.byref(s), int(clear))
        return {k: getattr(s, k) for k, _ in Stats._fields_}
