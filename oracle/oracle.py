"""ctypes loader for the CPU oracle (TEST INFRASTRUCTURE — never imported by the product path).

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py use this module.
All arrays are numpy host arrays; nothing here touches a GPU.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

FRAME = 84


class PongEnv(C.Structure):
    _fields_ = [("bx", C.c_float), ("by", C.c_float), ("vx", C.c_float), ("vy", C.c_float),
                ("pa", C.c_float), ("po", C.c_float), ("sa", C.c_int32), ("so", C.c_int32),
                ("ep_ret", C.c_int32), ("ep_len", C.c_int32)]


PONG_ENV_DTYPE = np.dtype([("bx", "f4"), ("by", "f4"), ("vx", "f4"), ("vy", "f4"), ("pa", "f4"),
                           ("po", "f4"), ("sa", "i4"), ("so", "i4"), ("ep_ret", "i4"),
                           ("ep_len", "i4")])


class PongStats(C.Structure):
    _fields_ = [("episodes", C.c_int64), ("return_sum", C.c_int64), ("length_sum", C.c_int64),
                ("return_min", C.c_int32), ("return_max", C.c_int32)]


def lib():
    global _LIB
    if _LIB is None:
        import importlib.util
        spec = importlib.util.spec_from_file_location("build_oracle",
                                                      os.path.join(_HERE, "build_oracle.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        # MI355ENV_ORACLE_LIB: load another build of the oracle (used by the mutation test only)
        path = os.environ.get("MI355ENV_ORACLE_LIB") or mod.build(force=False)
        L = C.CDLL(path)
        u32p = C.POINTER(C.c_uint32)
        L.oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.oracle_draw_block.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32, u32p]
        L.oracle_u01.argtypes = [C.c_uint32]; L.oracle_u01.restype = C.c_float
        L.oracle_u01_open0.argtypes = [C.c_uint32]; L.oracle_u01_open0.restype = C.c_float
        L.oracle_pong_action.argtypes = [C.c_uint32]; L.oracle_pong_action.restype = C.c_int32
        L.oracle_pong_serve_vx.argtypes = [C.c_uint32]; L.oracle_pong_serve_vx.restype = C.c_float
        L.oracle_pong_serve_vy.argtypes = [C.c_uint32]; L.oracle_pong_serve_vy.restype = C.c_float
        L.oracle_uniform.argtypes = [C.c_uint32, C.c_float, C.c_float]
        L.oracle_uniform.restype = C.c_float
        L.oracle_normal_pair.argtypes = [C.c_uint32, C.c_uint32, C.POINTER(C.c_float)]
        L.oracle_pong_step_one.argtypes = [C.POINTER(PongEnv), C.c_int32, C.c_float, C.c_float,
                                           C.c_int32, C.POINTER(C.c_uint8), C.POINTER(C.c_int32),
                                           C.POINTER(C.c_int32)]
        L.oracle_pong_step_one.restype = C.c_float
        L.oracle_pong_render_one.argtypes = [C.POINTER(PongEnv), C.c_void_p]
        L.oracle_pong_reset_one.argtypes = [C.POINTER(PongEnv), C.c_uint64, C.c_uint32, C.c_uint64]
        L.oracle_pong_create.argtypes = [C.c_int64, C.c_uint64, C.c_int32]
        L.oracle_pong_create.restype = C.c_void_p
        L.oracle_pong_destroy.argtypes = [C.c_void_p]
        L.oracle_pong_envs.argtypes = [C.c_void_p]; L.oracle_pong_envs.restype = C.c_void_p
        L.oracle_pong_step_count.argtypes = [C.c_void_p]; L.oracle_pong_step_count.restype = C.c_uint64
        L.oracle_pong_set_step_count.argtypes = [C.c_void_p, C.c_uint64]
        L.oracle_pong_set_normalize.argtypes = [C.c_void_p, C.c_int32]
        L.oracle_pong_get_stats.argtypes = [C.c_void_p, C.POINTER(PongStats), C.c_int32]
        L.oracle_pong_reset.argtypes = [C.c_void_p, C.c_void_p]
        L.oracle_pong_rollout.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_int32]
        L.oracle_pong_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p]
        L.oracle_pong_fill_stack.argtypes = [C.c_void_p, C.c_void_p]
        _bind_body(L)
        _LIB = L
    return _LIB


def _bind_body(L):
    """Rigid-body entry points (present once body.cpp is part of the build)."""
    if not hasattr(L, "oracle_body_create_f32"):
        return
    from oracle import body_binding
    body_binding.bind(L)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def philox(ctr, key):
    c = (C.c_uint32 * 4)(*[int(x) & 0xffffffff for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) & 0xffffffff for x in key])
    o = (C.c_uint32 * 4)()
    lib().oracle_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def draw_block(seed, env, step, stream):
    o = (C.c_uint32 * 4)()
    lib().oracle_draw_block(seed, env, step, stream, o)
    return [int(x) for x in o]


def pong_step_one(state, action, serve_vx, serve_vy, max_score=21):
    """state: dict of the ten PongEnv fields. Returns (new_state, reward, done, fin_ret, fin_len)."""
    e = PongEnv(**state)
    d = C.c_uint8(0); fr = C.c_int32(0); fl = C.c_int32(0)
    r = lib().oracle_pong_step_one(C.byref(e), action, serve_vx, serve_vy, max_score, C.byref(d),
                                   C.byref(fr), C.byref(fl))
    out = {name: getattr(e, name) for name, _ in PongEnv._fields_}
    return out, float(r), int(d.value), int(fr.value), int(fl.value)


def pong_render_one(state):
    e = PongEnv(**state)
    frame = np.zeros((FRAME, FRAME), np.uint8)
    lib().oracle_pong_render_one(C.byref(e), _ptr(frame))
    return frame


class Pong:
    """Batch of N oracle Pong environments (host memory)."""

    def __init__(self, n, seed, max_score=21, normalize=False):
        self.n, self.seed, self.max_score = int(n), int(seed), int(max_score)
        self.h = lib().oracle_pong_create(self.n, self.seed, self.max_score)
        lib().oracle_pong_set_normalize(self.h, int(bool(normalize)))

    def __del__(self):
        if getattr(self, "h", None):
            lib().oracle_pong_destroy(self.h)
            self.h = None

    def envs(self):
        """Structured numpy view (not a copy) of the N environment records."""
        addr = lib().oracle_pong_envs(self.h)
        buf = (C.c_char * (PONG_ENV_DTYPE.itemsize * self.n)).from_address(addr)
        return np.frombuffer(buf, dtype=PONG_ENV_DTYPE)

    @property
    def step_count(self):
        return int(lib().oracle_pong_step_count(self.h))

    @step_count.setter
    def step_count(self, v):
        lib().oracle_pong_set_step_count(self.h, int(v))

    def reset(self):
        obs = np.empty((self.n, 8), np.float32)
        lib().oracle_pong_reset(self.h, _ptr(obs))
        return obs

    def obs(self):
        e = self.envs()
        return np.stack([e["bx"], e["by"], e["vx"], e["vy"], e["pa"], e["po"],
                         e["sa"].astype(np.float32), e["so"].astype(np.float32)], axis=1)

    def rollout(self, T, actions=None, stack=None, nthreads=1, want_obs=True, out=None):
        """out: optional pre-allocated (obs, reward, done) arrays to write into."""
        if out is not None:
            obs, rew, done = out
            assert obs.shape == (T, self.n, 8) and obs.dtype == np.float32
            assert rew.shape == (T, self.n) and done.shape == (T, self.n)
        else:
            obs = np.empty((T, self.n, 8), np.float32) if want_obs else None
            rew = np.empty((T, self.n), np.float32)
            done = np.empty((T, self.n), np.uint8)
        if actions is not None:
            actions = np.ascontiguousarray(actions, np.uint8)
            assert actions.shape == (T, self.n)
        lib().oracle_pong_rollout(self.h, T, _ptr(actions), _ptr(obs), _ptr(rew), _ptr(done),
                                  _ptr(stack), nthreads)
        return obs, rew, done

    def step(self, actions=None, stack=None):
        a = None if actions is None else np.ascontiguousarray(actions, np.uint8).reshape(1, self.n)
        obs, rew, done = self.rollout(1, a, stack)
        return obs[0], rew[0], done[0]

    def fill_stack(self, stack):
        assert stack.shape == (self.n, 4, FRAME, FRAME) and stack.dtype == np.uint8
        lib().oracle_pong_fill_stack(self.h, _ptr(stack))

    def stats(self, clear=False):
        s = PongStats()
        lib().oracle_pong_get_stats(self.h, C.byref(s), int(clear))
        return {"episodes": s.episodes, "return_sum": s.return_sum, "length_sum": s.length_sum,
                "return_min": s.return_min, "return_max": s.return_max}
