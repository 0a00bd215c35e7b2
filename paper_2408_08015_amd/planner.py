"""ctypes binding of the planner's C ABI (include/asteroid_planner.h); argument marshalling
only: Eq. (3)-(11), Alg. 1 and Alg. 2 run in libasteroid_stage.so (host code, no GPU needed)."""
import ctypes as C

import numpy as np

from .binding import _check, load_library

_dp = C.POINTER(C.c_double)
_ip = C.POINTER(C.c_int32)


class ast_plan_problem(C.Structure):
    _fields_ = [("L", C.c_int32), ("N", C.c_int32), ("B", C.c_int32), ("M", C.c_int32),
                ("block", C.c_int32), ("mod_factor", C.c_double), ("opt_factor", C.c_double),
                ("host_tf", _dp), ("host_tb", _dp), ("host_a", _dp), ("host_act", _dp),
                ("host_w", _dp), ("host_u", _dp), ("host_bw", _dp), ("host_fixed", _dp)]


def _lib():
    lib = load_library()
    if not getattr(lib, "_planner_ready", False):
        pp, i32 = C.POINTER(ast_plan_problem), C.c_int32
        lib.asteroid_plan_stage_memory.argtypes = [pp, i32, i32, i32, i32, _dp]
        lib.asteroid_plan_allocate.argtypes = [pp, i32, i32, _ip, i32, i32, _ip, _dp, _dp, _ip]
        lib.asteroid_plan_round_latency.argtypes = [i32, _dp, _dp, _dp, i32, _dp, _ip]
        lib.asteroid_plan_hpp.argtypes = [pp, _ip, _ip, _ip, _ip, _ip, _dp]
        lib._planner_ready = True
    return lib


def _d(a):
    return np.ascontiguousarray(a, dtype=np.float64)


class Problem:
    """Profiler tables and device pool in the layout the C ABI takes.
    tf, tb [N][L][B+1]; a, act, w [L]; u [N]; bw [N][N]; fixed [L] or None (bytes per layer
    outside Eq. (3): workspace, derived weight copies)."""

    def __init__(self, tf, tb, a, act, w, u, bw, B, M, mod_factor=2.0, opt_factor=1.0, block=1, fixed=None):
        self.tf, self.tb, self.a, self.act, self.w, self.u, self.bw = map(_d, (tf, tb, a, act, w, u, bw))
        self.N, self.L = int(self.u.shape[0]), int(self.a.shape[0])
        self.B, self.M = int(B), int(M)
        if self.tf.shape != (self.N, self.L, self.B + 1) or self.tb.shape != self.tf.shape:
            raise ValueError("tf, tb must be [N][L][B+1]")
        if self.act.shape != (self.L,) or self.w.shape != (self.L,) or self.bw.shape != (self.N, self.N):
            raise ValueError("act, w must be [L] and bw [N][N]")
        c = ast_plan_problem()
        c.L, c.N, c.B, c.M, c.block = self.L, self.N, self.B, self.M, int(block)
        c.mod_factor, c.opt_factor = float(mod_factor), float(opt_factor)
        for name in ("tf", "tb", "a", "act", "w", "u", "bw"):
            setattr(c, "host_" + name, getattr(self, name).ctypes.data_as(_dp))
        self.fixed = None if fixed is None else _d(fixed)
        if self.fixed is not None:
            if self.fixed.shape != (self.L,):
                raise ValueError("fixed must be [L]")
            c.host_fixed = self.fixed.ctypes.data_as(_dp)
        self.c = c


def stage_memory(pr, lo, hi, K, beta):
    lib, out = _lib(), C.c_double()
    _check(lib, lib.asteroid_plan_stage_memory(C.byref(pr.c), lo, hi, K, beta, C.byref(out)))
    return out.value


def allocate(pr, lo, hi, group, K):
    """Alg. 1.  ({device: samples}, E_f, E_b), or None when the micro-batch does not fit."""
    lib = _lib()
    g = len(group)
    G = (C.c_int32 * g)(*group)
    y = (C.c_int32 * g)()
    Ef, Eb, ok = C.c_double(), C.c_double(), C.c_int32()
    _check(lib, lib.asteroid_plan_allocate(C.byref(pr.c), lo, hi, G, g, K, y, C.byref(Ef), C.byref(Eb), C.byref(ok)))
    if not ok.value:
        return None
    return {d: int(v) for d, v in zip(group, y)}, Ef.value, Eb.value


def round_latency(Ef, Eb, Ta, M):
    """Eq. (4)-(6).  (latency, dominant step)."""
    lib = _lib()
    Ef, Eb, Ta = _d(Ef), _d(Eb), _d(Ta)
    lat, dm = C.c_double(), C.c_int32()
    _check(lib, lib.asteroid_plan_round_latency(len(Ef), Ef.ctypes.data_as(_dp), Eb.ctypes.data_as(_dp),
                                                Ta.ctypes.data_as(_dp), M, C.byref(lat), C.byref(dm)))
    return lat.value, dm.value


def plan_hpp(pr):
    """Alg. 2.  (latency, stages, y): stages = [(lo, hi, [device ids])] first stage first,
    y = {device: samples per micro-batch}; (inf, None, None) when nothing fits."""
    lib = _lib()
    N = pr.N
    P, lat = C.c_int32(), C.c_double()
    lo = (C.c_int32 * (N + 1))()
    nd = (C.c_int32 * N)()
    order = (C.c_int32 * N)()
    y = (C.c_int32 * N)()
    _check(lib, lib.asteroid_plan_hpp(C.byref(pr.c), C.byref(P), lo, nd, order, y, C.byref(lat)))
    if P.value == 0:
        return lat.value, None, None
    stages, first = [], 0
    for k in range(P.value):
        stages.append((int(lo[k]), int(lo[k + 1]), [int(order[i]) for i in range(first, first + nd[k])]))
        first += nd[k]
    return lat.value, stages, {d: int(y[d]) for d in range(N)}
