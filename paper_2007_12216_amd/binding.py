"""ctypes binding with the same names as include/rnswino.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "librnswino.so")

MATRIX_AT, MATRIX_G, MATRIX_BT = 0, 1, 2
STAGE_U, STAGE_V, STAGE_O = 0, 1, 2
FLAG_ALLOW_UNCHECKED_RANGE, FLAG_HOST_ONLY, FLAG_GEMM_BLOCK_64X16 = 1, 2, 4

EXPORTED_SYMBOLS = (
    "rnswino_plan", "rnswino_plan_destroy", "rnswino_output_dims", "rnswino_filter_bytes",
    "rnswino_workspace_bytes", "rnswino_filter_transform", "rnswino_conv2d", "rnswino_conv2d_requant",
    "rnswino_conv2d_events", "rnswino_conv2d_static",
    "rnswino_direct_filter_bytes", "rnswino_direct_workspace_bytes", "rnswino_direct_filter_pack", "rnswino_direct_conv2d",
    "rnswino_requant_pool",
    "rnswino_plan_get_matrix", "rnswino_plan_get_table", "rnswino_plan_get_mrc_inverse", "rnswino_plan_dynamic_range",
    "rnswino_plan_describe", "rnswino_kernel_variants", "rnswino_debug_empty_launch",
    "rnswino_debug_stage", "rnswino_strerror",
)


class RnsWinoError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {rnswino_strerror(code)} ({code})")


class _Desc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("C", ctypes.c_int32), ("K", ctypes.c_int32), ("H", ctypes.c_int32),
                ("W", ctypes.c_int32), ("r", ctypes.c_int32), ("m", ctypes.c_int32), ("pad", ctypes.c_int32),
                ("stride", ctypes.c_int32), ("n_moduli", ctypes.c_int32), ("moduli", ctypes.c_uint32 * 8),
                ("flags", ctypes.c_uint32), ("output_bound", ctypes.c_uint64)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def lib():
    """Load librnswino.so (built in-tree).  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2007_12216_amd.build` "
                              "(or __graft_entry__.build())")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64, u32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32
        L.rnswino_plan.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(_Desc)]
        L.rnswino_plan.restype = ctypes.c_int
        L.rnswino_plan_destroy.argtypes = [vp]
        L.rnswino_plan_destroy.restype = ctypes.c_int
        L.rnswino_output_dims.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.rnswino_output_dims.restype = ctypes.c_int
        L.rnswino_filter_bytes.argtypes = [vp]
        L.rnswino_filter_bytes.restype = ctypes.c_size_t
        L.rnswino_workspace_bytes.argtypes = [vp]
        L.rnswino_workspace_bytes.restype = ctypes.c_size_t
        L.rnswino_filter_transform.argtypes = [vp, vp, vp, vp]
        L.rnswino_filter_transform.restype = ctypes.c_int
        L.rnswino_conv2d.argtypes = [vp, vp, vp, vp, vp, vp]
        L.rnswino_conv2d.restype = ctypes.c_int
        L.rnswino_conv2d_requant.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp]
        L.rnswino_conv2d_requant.restype = ctypes.c_int
        L.rnswino_conv2d_events.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.POINTER(vp)]
        L.rnswino_conv2d_events.restype = ctypes.c_int
        L.rnswino_conv2d_static.argtypes = [vp, vp, vp, vp, vp]
        L.rnswino_conv2d_static.restype = ctypes.c_int
        L.rnswino_direct_filter_bytes.argtypes = [i32, i32, i32]
        L.rnswino_direct_filter_bytes.restype = ctypes.c_size_t
        L.rnswino_direct_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
        L.rnswino_direct_workspace_bytes.restype = ctypes.c_size_t
        L.rnswino_direct_filter_pack.argtypes = [vp, vp, i32, i32, i32, vp]
        L.rnswino_direct_filter_pack.restype = ctypes.c_int
        L.rnswino_direct_conv2d.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp]
        L.rnswino_direct_conv2d.restype = ctypes.c_int
        L.rnswino_requant_pool.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp]
        L.rnswino_requant_pool.restype = ctypes.c_int
        L.rnswino_plan_get_matrix.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp]
        L.rnswino_plan_get_matrix.restype = ctypes.c_int
        L.rnswino_plan_get_table.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t]
        L.rnswino_plan_get_table.restype = ctypes.c_int64
        L.rnswino_plan_get_mrc_inverse.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(u32)]
        L.rnswino_plan_get_mrc_inverse.restype = ctypes.c_int
        L.rnswino_plan_describe.argtypes = [vp, i32, ctypes.c_char_p, ctypes.c_size_t]
        L.rnswino_plan_describe.restype = i64
        L.rnswino_debug_empty_launch.argtypes = [u32, u32, vp, vp, vp]
        L.rnswino_debug_empty_launch.restype = ctypes.c_int
        L.rnswino_kernel_variants.argtypes = [ctypes.c_char_p, ctypes.c_size_t]
        L.rnswino_kernel_variants.restype = i64
        L.rnswino_plan_dynamic_range.argtypes = [vp]
        L.rnswino_plan_dynamic_range.restype = i64
        L.rnswino_debug_stage.argtypes = [vp, ctypes.c_int, vp, vp]
        L.rnswino_debug_stage.restype = ctypes.c_int
        L.rnswino_strerror.argtypes = [ctypes.c_int]
        L.rnswino_strerror.restype = ctypes.c_char_p
        _lib = L
    return _lib


def rnswino_strerror(code: int) -> str:
    return lib().rnswino_strerror(int(code)).decode()


def _check(code: int, what: str):
    if code != 0:
        raise RnsWinoError(code, what)


class Plan:
    """Owner of one rnswino_plan_t* (destroyed with the object)."""

    def __init__(self, handle, desc):
        self.handle = handle
        self.N, self.C, self.K, self.H, self.W = desc.N, desc.C, desc.K, desc.H, desc.W
        self.r, self.m, self.pad = desc.r, desc.m, desc.pad
        self.t = desc.m + desc.r - 1
        self.moduli = tuple(desc.moduli[i] for i in range(desc.n_moduli))
        self.Ho, self.Wo = rnswino_output_dims(self)
        self.th, self.tw = -(-self.Ho // self.m), -(-self.Wo // self.m)
        self.T = self.N * self.th * self.tw

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None:
            _lib.rnswino_plan_destroy(h)


def rnswino_plan(N, C, K, H, W, r, m, pad, moduli, flags: int = 0, stride: int = 1, output_bound: int = 0) -> Plan:
    d = _Desc()
    d.N, d.C, d.K, d.H, d.W, d.r, d.m, d.pad, d.stride = N, C, K, H, W, r, m, pad, stride
    d.n_moduli = len(moduli)
    if len(moduli) <= 8:
        for i, p in enumerate(moduli):
            d.moduli[i] = p
    d.flags = flags
    d.output_bound = int(output_bound)
    out = ctypes.c_void_p()
    _check(lib().rnswino_plan(ctypes.byref(out), ctypes.byref(d)), "rnswino_plan")
    return Plan(out, d)


def rnswino_plan_destroy(plan: Plan) -> None:
    h, plan.handle = plan.handle, None
    if h:
        _check(lib().rnswino_plan_destroy(h), "rnswino_plan_destroy")


def rnswino_output_dims(plan: Plan):
    ho, wo = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().rnswino_output_dims(plan.handle, ctypes.byref(ho), ctypes.byref(wo)), "rnswino_output_dims")
    return ho.value, wo.value


def rnswino_filter_bytes(plan: Plan) -> int:
    return int(lib().rnswino_filter_bytes(plan.handle))


def rnswino_workspace_bytes(plan: Plan) -> int:
    return int(lib().rnswino_workspace_bytes(plan.handle))


def _ptr(obj) -> int:
    """Device (or host) address of a torch tensor / numpy array / raw int."""
    if isinstance(obj, int):
        return obj
    if hasattr(obj, "data_ptr"):
        return obj.data_ptr()
    return obj.ctypes.data


def rnswino_filter_transform(plan: Plan, w_dev, U_dev, stream: int = 0) -> None:
    _check(lib().rnswino_filter_transform(plan.handle, _ptr(w_dev), _ptr(U_dev), stream), "rnswino_filter_transform")


def rnswino_conv2d(plan: Plan, x_dev, U_dev, y_dev, workspace_dev, stream: int = 0) -> None:
    _check(lib().rnswino_conv2d(plan.handle, _ptr(x_dev), _ptr(U_dev), _ptr(y_dev), _ptr(workspace_dev), stream),
           "rnswino_conv2d")


def rnswino_conv2d_requant(plan: Plan, x_dev, U_dev, a_dev, shift: int, pool: bool, workspace_dev, stream: int = 0) -> None:
    _check(lib().rnswino_conv2d_requant(plan.handle, _ptr(x_dev), _ptr(U_dev), _ptr(a_dev), shift, int(bool(pool)),
                                        _ptr(workspace_dev), stream), "rnswino_conv2d_requant")


def rnswino_conv2d_events(plan: Plan, x_dev, U_dev, y_dev, workspace_dev, stream: int, events) -> None:
    """events: six hipEvent_t handles (ints): (start, stop) of the three kernels."""
    arr = (ctypes.c_void_p * 6)(*[int(e) for e in events])
    _check(lib().rnswino_conv2d_events(plan.handle, _ptr(x_dev), _ptr(U_dev), _ptr(y_dev), _ptr(workspace_dev), stream, arr),
           "rnswino_conv2d_events")


STATIC_WORKSPACE_BYTES = 16 << 20


def rnswino_conv2d_static(plan: Plan, x_dev, U_dev, y_dev, stream: int = 0) -> None:
    _check(lib().rnswino_conv2d_static(plan.handle, _ptr(x_dev), _ptr(U_dev), _ptr(y_dev), stream), "rnswino_conv2d_static")


def rnswino_direct_filter_bytes(C: int, K: int, r: int) -> int:
    return int(lib().rnswino_direct_filter_bytes(C, K, r))


def rnswino_direct_workspace_bytes(N: int, C: int, H: int, W: int, pad: int) -> int:
    return int(lib().rnswino_direct_workspace_bytes(N, C, H, W, pad))


def rnswino_direct_filter_pack(w_dev, wt_dev, C: int, K: int, r: int, stream: int = 0) -> None:
    _check(lib().rnswino_direct_filter_pack(_ptr(w_dev), _ptr(wt_dev), C, K, r, stream), "rnswino_direct_filter_pack")


def rnswino_direct_conv2d(x_dev, wt_dev, y_dev, N, C, K, H, W, r, pad, workspace_dev, stream: int = 0) -> None:
    _check(lib().rnswino_direct_conv2d(_ptr(x_dev), _ptr(wt_dev), _ptr(y_dev), N, C, K, H, W, r, pad, _ptr(workspace_dev), stream),
           "rnswino_direct_conv2d")


def rnswino_requant_pool(y_dev, a_dev, planes: int, H: int, W: int, shift: int, pool: bool, stream: int = 0) -> None:
    _check(lib().rnswino_requant_pool(_ptr(y_dev), _ptr(a_dev), planes, H, W, shift, int(bool(pool)), stream),
           "rnswino_requant_pool")


def rnswino_plan_get_matrix(plan: Plan, which: int, modulus_idx: int) -> np.ndarray:
    shape = {MATRIX_AT: (plan.m, plan.t), MATRIX_G: (plan.t, plan.r), MATRIX_BT: (plan.t, plan.t)}.get(which, (1, 1))
    out = np.zeros(shape, dtype=np.int32)
    _check(lib().rnswino_plan_get_matrix(plan.handle, which, modulus_idx, out.ctypes.data), "rnswino_plan_get_matrix")
    return out


TABLE_INPUT, TABLE_INVERSE = 0, 1


def rnswino_plan_get_table(plan: Plan, which: int, modulus_idx: int) -> np.ndarray:
    """Kronecker table of one modulus in the kernels' fragment order: int8 [blocks][steps][planes][64][16]."""
    n = lib().rnswino_plan_get_table(plan.handle, which, modulus_idx, None, 0)
    _check(int(min(n, 0)), "rnswino_plan_get_table")
    out = np.zeros(int(n), dtype=np.int8)
    _check(int(min(lib().rnswino_plan_get_table(plan.handle, which, modulus_idx, out.ctypes.data, out.nbytes), 0)),
           "rnswino_plan_get_table")
    return out.reshape(-1, 64, 16)


def rnswino_plan_get_mrc_inverse(plan: Plan, l: int, j: int) -> int:
    v = ctypes.c_uint32()
    _check(lib().rnswino_plan_get_mrc_inverse(plan.handle, l, j, ctypes.byref(v)), "rnswino_plan_get_mrc_inverse")
    return v.value


def rnswino_plan_describe(plan: Plan, output_mode: int = 0) -> dict:
    """The library's report of what it launches for this plan: {"kernels": [names in launch order], "grids": [...],
    "conversion": ..., "text": the raw report}."""
    n = lib().rnswino_plan_describe(plan.handle, output_mode, None, 0)
    _check(int(min(n, 0)), "rnswino_plan_describe")
    buf = ctypes.create_string_buffer(int(n))
    _check(int(min(lib().rnswino_plan_describe(plan.handle, output_mode, buf, int(n)), 0)), "rnswino_plan_describe")
    text = buf.value.decode()
    kernels, grids, conversion = [], [], None
    for line in text.splitlines():
        if line.startswith("conversion="):
            conversion = line.split("=", 1)[1]
        elif line:
            name, _, rest = line.partition("> ")
            kernels.append(name + ">")
            grids.append(rest)
    return {"kernels": kernels, "grids": grids, "conversion": conversion, "text": text}


def rnswino_debug_empty_launch(grid_x: int, grid_y: int, stream: int = 0, start_event: int = 0, stop_event: int = 0) -> None:
    _check(lib().rnswino_debug_empty_launch(grid_x, grid_y, stream, start_event or None, stop_event or None),
           "rnswino_debug_empty_launch")


def rnswino_kernel_variants() -> list:
    """Names of every kernel instantiation of the three hot stages the library can launch."""
    n = int(lib().rnswino_kernel_variants(None, 0))
    buf = ctypes.create_string_buffer(n)
    lib().rnswino_kernel_variants(buf, n)
    return [l for l in buf.value.decode().splitlines() if l]


def rnswino_plan_dynamic_range(plan: Plan) -> int:
    return int(lib().rnswino_plan_dynamic_range(plan.handle))


def rnswino_debug_stage(plan: Plan, stage: int, src_dev) -> np.ndarray:
    n, P2 = len(plan.moduli), plan.t * plan.t
    shape = {STAGE_U: (n, P2, plan.K, plan.C), STAGE_V: (n, P2, plan.T, plan.C), STAGE_O: (n, P2, plan.K, plan.T)}[stage]
    out = np.empty(shape, dtype=np.int32)
    _check(lib().rnswino_debug_stage(plan.handle, stage, _ptr(src_dev), out.ctypes.data), "rnswino_debug_stage")
    return out
