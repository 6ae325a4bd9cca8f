"""ctypes declarations and a small wrapper for the rigid-body oracle (TEST INFRASTRUCTURE)."""
import ctypes as C

import numpy as np

NQ, NACT, NOBS = 9, 6, 17


class BodyStats(C.Structure):
    _fields_ = [("episodes", C.c_int64), ("length_sum", C.c_int64), ("return_sum", C.c_double),
                ("return_min", C.c_double), ("return_max", C.c_double), ("nonfinite", C.c_int64)]


def bind(L):
    vp = C.c_void_p
    for sfx in ("_f32", "_f64"):
        g = lambda name: getattr(L, "oracle_body_" + name + sfx)
        g("create").argtypes = [C.c_int64, C.c_uint64, vp]; g("create").restype = vp
        g("destroy").argtypes = [vp]
        g("set_params").argtypes = [vp, vp]
        g("reset").argtypes = [vp, vp]
        g("rollout").argtypes = [vp, C.c_int32, vp, vp, vp, vp, C.c_int32]
        g("get_state").argtypes = [vp, vp]
        g("set_state").argtypes = [vp, vp]
        g("step_count").argtypes = [vp]; g("step_count").restype = C.c_uint64
        g("set_step_count").argtypes = [vp, C.c_uint64]
        g("get_stats").argtypes = [vp, C.POINTER(BodyStats), C.c_int32]
        g("mass_matrix").argtypes = [vp, vp, vp]
        g("bias_gravity").argtypes = [vp, vp, vp, vp, vp]
        g("contact").argtypes = [vp, vp, vp, vp, vp]
        g("point").argtypes = [C.c_int32, C.c_int32, vp, vp, vp, vp, vp, vp]
        g("energy").argtypes = [vp, vp, vp]; g("energy").restype = C.c_double
        g("substep").argtypes = [vp, vp, vp, vp]; g("substep").restype = C.c_int32
        g("solve").argtypes = [vp, vp, vp]; g("solve").restype = C.c_int32
        g("newton_rows").argtypes = [vp, vp, vp, vp, vp, vp]; g("newton_rows").restype = C.c_int32
        g("newton_accel").argtypes = [vp, vp, vp, vp, vp, vp, vp]; g("newton_accel").restype = C.c_int32
        g("draw_actions").argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, vp]
        g("step_margin").argtypes = [vp, vp, vp, vp]; g("step_margin").restype = C.c_double
    L.oracle_body_link.argtypes = [C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_double)]


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Body:
    """Batch of N oracle bodies in float32 (dtype=np.float32) or float64."""

    DEFAULTS = dict(armature=0.1, joint_damping=3.0, friction_mu=0.4, gravity=9.81, contact_k=1e4,
                    contact_c=100.0, h=0.01, gear=120.0, substeps=5, round_state_f32=0,
                    solver=0, newton_iters=8, time_const=0.02, reg_contact=0.02, reg_limit=0.5)

    def __init__(self, n, seed, dtype=np.float32, max_episode_steps=1000, **params):
        from oracle import oracle as orc
        self.L = orc.lib()
        self.dtype = np.dtype(dtype)
        self.sfx = "_f32" if self.dtype == np.float32 else "_f64"
        self.n, self.seed = int(n), int(seed)
        self.params = dict(self.DEFAULTS)
        self.params.update(params)
        cfg = np.array([self.params["armature"], self.params["joint_damping"],
                        self.params["friction_mu"], max_episode_steps], np.float64)
        self.h = self._f("create")(self.n, self.seed, _p(cfg))
        self._push_params()

    def _f(self, name):
        return getattr(self.L, "oracle_body_" + name + self.sfx)

    def _push_params(self):
        p = self.params
        arr = np.array([p["armature"], p["joint_damping"], p["friction_mu"], p["gravity"],
                        p["contact_k"], p["contact_c"], p["h"], p["gear"], p["substeps"],
                        p["round_state_f32"], p["solver"], p["newton_iters"], p["time_const"],
                        p["reg_contact"], p["reg_limit"]], np.float64)
        self._f("set_params")(self.h, _p(arr))

    def set_params(self, **kw):
        self.params.update(kw)
        self._push_params()

    def __del__(self):
        if getattr(self, "h", None):
            self._f("destroy")(self.h)
            self.h = None

    def arr(self, x):
        return np.ascontiguousarray(x, self.dtype)

    @property
    def step_count(self):
        return int(self._f("step_count")(self.h))

    @step_count.setter
    def step_count(self, v):
        self._f("set_step_count")(self.h, int(v))

    def reset(self):
        obs = np.empty((self.n, NOBS), self.dtype)
        self._f("reset")(self.h, _p(obs))
        return obs

    def rollout(self, T, actions=None, nthreads=1, want_obs=True):
        obs = np.empty((T, self.n, NOBS), self.dtype) if want_obs else None
        rew = np.empty((T, self.n), self.dtype)
        done = np.empty((T, self.n), np.uint8)
        if actions is not None:
            actions = self.arr(actions)
            assert actions.shape == (T, self.n, NACT)
        self._f("rollout")(self.h, T, _p(actions), _p(obs), _p(rew), _p(done), nthreads)
        return obs, rew, done

    def get_state(self):
        s = np.empty((self.n, 20), self.dtype)
        self._f("get_state")(self.h, _p(s))
        return s

    def set_state(self, s):
        s = self.arr(s)
        assert s.shape == (self.n, 20)
        self._f("set_state")(self.h, _p(s))

    def stats(self, clear=False):
        s = BodyStats()
        self._f("get_stats")(self.h, C.byref(s), int(clear))
        return {k: getattr(s, k) for k, _ in BodyStats._fields_}

    # ---- components (single configuration) -------------------------------------------------
    def mass_matrix(self, q):
        M = np.empty((NQ, NQ), self.dtype)
        self._f("mass_matrix")(self.h, _p(self.arr(q)), _p(M))
        return M

    def bias_gravity(self, q, v):
        hb, Qg = np.empty(NQ, self.dtype), np.empty(NQ, self.dtype)
        self._f("bias_gravity")(self.h, _p(self.arr(q)), _p(self.arr(v)), _p(hb), _p(Qg))
        return hb, Qg

    def contact(self, q, v):
        Q, F = np.empty(NQ, self.dtype), np.empty((8, 2), self.dtype)
        self._f("contact")(self.h, _p(self.arr(q)), _p(self.arr(v)), _p(Q), _p(F))
        return Q, F

    def point(self, kind, index, q, v=None):
        v = np.zeros(NQ) if v is None else v
        pos, J = np.empty(2, self.dtype), np.empty((2, NQ), self.dtype)
        vel, jd = np.empty(2, self.dtype), np.empty(2, self.dtype)
        self._f("point")(kind, index, _p(self.arr(q)), _p(self.arr(v)), _p(pos), _p(J), _p(vel), _p(jd))
        return pos, J, vel, jd

    def energy(self, q, v):
        return float(self._f("energy")(self.h, _p(self.arr(q)), _p(self.arr(v))))

    def substep(self, q, v, a):
        q, v = self.arr(q).copy(), self.arr(v).copy()
        mask = self._f("substep")(self.h, _p(q), _p(v), _p(self.arr(a)))
        return q, v, mask

    def newton_rows(self, q, v):
        """Constraint rows of the Newton contact model at (q, v): J [m,9], aref [m], D [m]."""
        J, ar, D = np.empty((22, NQ), self.dtype), np.empty(22, self.dtype), np.empty(22, self.dtype)
        m = self._f("newton_rows")(self.h, _p(self.arr(q)), _p(self.arr(v)), _p(J), _p(ar), _p(D))
        return J[:m].copy(), ar[:m].copy(), D[:m].copy()

    def newton_accel(self, q, v, a):
        """Acceleration of one substep, the force without constraints f = M a0, and
        (rows, passes, converged, active-set bits)."""
        acc, f = np.empty(NQ, self.dtype), np.empty(NQ, self.dtype)
        info = np.zeros(4, np.int32)
        ok = self._f("newton_accel")(self.h, _p(self.arr(q)), _p(self.arr(v)), _p(self.arr(a)), _p(acc), _p(f),
                                     _p(info))
        assert ok
        return acc, f, tuple(int(x) for x in info)

    def solve(self, A, b):
        x = np.empty(NQ, self.dtype)
        ok = self._f("solve")(_p(self.arr(A)), _p(self.arr(b)), _p(x))
        return x, bool(ok)

    def step_margin(self, q, v, a):
        """Smallest distance of any decision of one env step from (q, v) under actions a to its
        switching surface (contact heights, joint-limit onsets, signs of v* at limits)."""
        return float(self._f("step_margin")(self.h, _p(self.arr(q)), _p(self.arr(v)), _p(self.arr(a))))

    def draw_actions(self, env, step):
        a = np.empty(NACT, self.dtype)
        self._f("draw_actions")(self.seed, env, step, _p(a))
        return a

    def link(self, i):
        m, l = C.c_double(), C.c_double()
        self.L.oracle_body_link(i, C.byref(m), C.byref(l))
        return m.value, l.value
