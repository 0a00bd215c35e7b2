"""ctypes binding of the C ABI (include/asteroid.h); same names, argument marshalling only."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

STATUS = {0: "AST_OK", -1: "AST_EINVAL", -2: "AST_ESTATE", -3: "AST_ENOMEM", -4: "AST_EHIP",
          -5: "AST_EUNSUPPORTED"}
KINDS = {"conv2d": 0, "batchnorm2d": 1, "relu": 2, "relu6": 3, "res_begin": 4, "res_add": 5,
         "global_avgpool": 6, "linear": 7, "softmax_ce": 8, "maxpool2x2": 9, "layernorm": 10,
         "mha": 11, "gelu": 12, "swish": 13, "sigmoid": 14, "se_begin": 15, "se_scale": 16, "res_swap": 17, "maxpool3x3s2": 18}
DTYPES = {"f32": 0, "bf16": 1}
LAYOUTS = {"nchw": 0, "nhwc": 1, "bsd": 2}


class AsteroidError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("%s: %s" % (STATUS.get(status, status), msg))
        self.status = status


class ast_layer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("p", C.c_int32 * 8), ("eps", C.c_float)]


class ast_stage_cfg(C.Structure):
    _fields_ = [("B", C.c_int32), ("M", C.c_int32), ("K", C.c_int32), ("in_shape", C.c_int32 * 4),
                ("dtype", C.c_int32), ("layout", C.c_int32), ("needs_input_grad", C.c_int32)]


def lib_path():
    return os.path.join(_HERE, "libasteroid_stage.so")


def load_library():
    """Load libasteroid_stage.so (built in-tree by build.py); raises if it is missing."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError("HIP library not built: %s is missing (run __graft_entry__.build())" % path)
    try:
        # The caller's tensors and streams come from PyTorch, whose wheel carries its own HIP
        # runtime: load it first so that this library binds to the same runtime instance (a
        # second instance loaded beforehand sees no device once PyTorch initialises its own).
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(path)
    vp, i32, f32p, szp = C.c_void_p, C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_size_t)
    lib.asteroid_stage_create.argtypes = [C.POINTER(ast_layer), i32, C.POINTER(ast_stage_cfg), vp, C.POINTER(vp)]
    lib.asteroid_stage_forward.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.asteroid_stage_set_forward_stream.argtypes = [vp, vp]
    lib.asteroid_stream_create.argtypes = [C.POINTER(vp)]
    lib.asteroid_stream_destroy.argtypes = [vp]
    lib.asteroid_stage_backward.argtypes = [vp, i32, vp, vp]
    lib.asteroid_stage_backward_static.argtypes = [vp, i32, vp, vp]
    lib.asteroid_stage_step.argtypes = [vp, C.c_float, C.c_float]
    lib.asteroid_stage_destroy.argtypes = [vp]
    lib.asteroid_stage_destroy.restype = None
    lib.asteroid_stage_num_params.argtypes = [vp]
    lib.asteroid_stage_num_params.restype = C.c_size_t
    for n in ("set_params", "get_params", "get_grads", "set_velocity", "get_velocity"):
        getattr(lib, "asteroid_stage_" + n).argtypes = [vp, f32p]
    lib.asteroid_stage_memory.argtypes = [vp, szp, szp, szp, szp]
    lib.asteroid_stage_plan_memory.argtypes = [C.POINTER(ast_layer), i32, C.POINTER(ast_stage_cfg), szp, szp, szp, szp]
    lib.asteroid_stage_debug_activation.argtypes = [vp, i32, i32, f32p, szp]
    lib.asteroid_stage_profile_begin.argtypes = [vp, C.c_char_p, i32]
    lib.asteroid_stage_profile_end.argtypes = [vp]
    lib.asteroid_stage_profile_entry.argtypes = [vp, i32, C.c_char_p, C.c_size_t, C.POINTER(i32), C.POINTER(C.c_double)]
    lib.asteroid_last_error.restype = C.c_char_p
    lib.asteroid_kp.argtypes = [i32, i32]
    lib.asteroid_kp.restype = i32
    _LIB = lib
    return lib


def _check(lib, status):
    if status != 0:
        raise AsteroidError(status, lib.asteroid_last_error().decode())


def _marshal_layers(layers):
    arr = (ast_layer * len(layers))()
    for a, L in zip(arr, layers):
        k = L["kind"]
        a.kind = KINDS[k]
        a.eps = float(L.get("eps", 0.0))
        if k == "conv2d":
            vals = [L["cin"], L["cout"], L["k"], L["stride"], L["pad"], L["groups"], int(L["bias"])]
        elif k == "linear":
            vals = [L["cin"], L["cout"], int(L["bias"])]
        elif k == "batchnorm2d":
            vals = [L["c"]]
        elif k == "layernorm":
            vals = [L["d"]]
        elif k == "mha":
            vals = [L["d"], L["heads"]]
        else:
            vals = []
        for i, v in enumerate(vals):
            a.p[i] = int(v)
    return arr


def _marshal_cfg(B, M, K, in_shape, dtype, layout, needs_input_grad):
    cfg = ast_stage_cfg()
    cfg.B, cfg.M, cfg.K = B, M, K
    for i, v in enumerate(in_shape):
        cfg.in_shape[i] = int(v)
    cfg.dtype = DTYPES[dtype]
    cfg.layout = LAYOUTS[layout]
    cfg.needs_input_grad = int(bool(needs_input_grad))
    return cfg


def stream_create():
    """A new non-blocking HIP stream of default priority; returns its handle (an int)."""
    lib = load_library()
    h = C.c_void_p()
    _check(lib, lib.asteroid_stream_create(C.byref(h)))
    return h.value


def stream_destroy(handle):
    lib = load_library()
    _check(lib, lib.asteroid_stream_destroy(C.c_void_p(handle or 0)))


def kp(P, p):
    return load_library().asteroid_kp(P, p)


def plan_memory(layers, B, M, K, in_shape, dtype="f32", layout="nchw", needs_input_grad=True):
    """(mod, opt, act_per_mb, workspace) bytes of a stage, without building it (no GPU needed)."""
    lib = load_library()
    arr = _marshal_layers(layers)
    cfg = _marshal_cfg(B, M, K, in_shape, dtype, layout, needs_input_grad)
    out = [C.c_size_t() for _ in range(4)]
    _check(lib, lib.asteroid_stage_plan_memory(arr, len(layers), C.byref(cfg), *[C.byref(o) for o in out]))
    return tuple(o.value for o in out)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class Stage:
    """One pipeline stage on one GPU.  Tensors passed to forward/backward are torch CUDA
    tensors (contiguous, in the stage's layout and dtype); only their data pointers cross."""

    def __init__(self, layers, B, M, K, in_shape, dtype="f32", layout="nchw", needs_input_grad=True,
                 stream=None):
        self.lib = load_library()
        self.layers = list(layers)
        self.B, self.M, self.K = B, M, K
        self.dtype, self.layout = dtype, layout
        arr = _marshal_layers(layers)
        cfg = _marshal_cfg(B, M, K, in_shape, dtype, layout, needs_input_grad)
        h = C.c_void_p()
        _check(self.lib, self.lib.asteroid_stage_create(arr, len(layers), C.byref(cfg),
                                                        C.c_void_p(stream or 0), C.byref(h)))
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.asteroid_stage_destroy(self.h)
            self.h = None

    __del__ = close

    def forward(self, mb, x, labels=None, y=None, loss=None):
        _check(self.lib, self.lib.asteroid_stage_forward(self.h, mb, _ptr(x), _ptr(labels), _ptr(y), _ptr(loss)))

    def set_forward_stream(self, stream):
        _check(self.lib, self.lib.asteroid_stage_set_forward_stream(self.h, C.c_void_p(stream or 0)))

    def backward(self, mb, dy=None, dx=None):
        _check(self.lib, self.lib.asteroid_stage_backward(self.h, mb, _ptr(dy), _ptr(dx)))

    def backward_static(self, mb, dy=None, dx=None):
        _check(self.lib, self.lib.asteroid_stage_backward_static(self.h, mb, _ptr(dy), _ptr(dx)))

    def step(self, lr, momentum):
        _check(self.lib, self.lib.asteroid_stage_step(self.h, lr, momentum))

    @property
    def num_params(self):
        return self.lib.asteroid_stage_num_params(self.h)

    def _get(self, name):
        out = np.empty(self.num_params, np.float32)
        _check(self.lib, getattr(self.lib, "asteroid_stage_" + name)(self.h, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def _set(self, name, flat):
        flat = np.ascontiguousarray(flat, np.float32)
        assert flat.size == self.num_params
        _check(self.lib, getattr(self.lib, "asteroid_stage_" + name)(self.h, flat.ctypes.data_as(C.POINTER(C.c_float))))

    def set_params(self, flat):
        self._set("set_params", flat)

    def get_params(self):
        return self._get("get_params")

    def get_grads(self):
        return self._get("get_grads")

    def set_velocity(self, flat):
        self._set("set_velocity", flat)

    def get_velocity(self):
        return self._get("get_velocity")

    def memory(self):
        out = [C.c_size_t() for _ in range(4)]
        _check(self.lib, self.lib.asteroid_stage_memory(self.h, *[C.byref(o) for o in out]))
        return tuple(o.value for o in out)

    def profile_begin(self, kernel_filter="", max_launches=4096):
        _check(self.lib, self.lib.asteroid_stage_profile_begin(self.h, kernel_filter.encode(), max_launches))

    def profile_end(self):
        """{kernel name: (launches, total_ms)} of the launches recorded since profile_begin."""
        _check(self.lib, self.lib.asteroid_stage_profile_end(self.h))
        out, i = {}, 0
        buf = C.create_string_buffer(256)
        n, ms = C.c_int32(), C.c_double()
        while self.lib.asteroid_stage_profile_entry(self.h, i, buf, 256, C.byref(n), C.byref(ms)) == 0:
            out[buf.value.decode()] = (n.value, ms.value)
            i += 1
        return out

    def debug_activation(self, mb, layer):
        n = C.c_size_t()
        _check(self.lib, self.lib.asteroid_stage_debug_activation(self.h, mb, layer, None, C.byref(n)))
        out = np.empty(n.value, np.float32)
        _check(self.lib, self.lib.asteroid_stage_debug_activation(
            self.h, mb, layer, out.ctypes.data_as(C.POINTER(C.c_float)), C.byref(n)))
        return out
