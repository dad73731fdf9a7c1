"""ctypes binding of the C ABI declared in include/heatkv.h (same names, argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libheatkv.so")

F32, BF16 = 0, 1
VARIANT_HEATKV, VARIANT_BINARY, VARIANT_NAIVE, VARIANT_BINARY_NAIVE = 0, 1, 2, 3
SET_G, SET_E, SET_A = 0, 1, 2
KV_NATIVE, KV_FP8_E4M3 = 0, 1
_DTYPES = {"f32": F32, "bf16": BF16}


class HeatKVError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"heatkv error {code}: {msg}")
        self.code = code


class _CShape(C.Structure):
    _fields_ = [("L", C.c_int32), ("H", C.c_int32), ("d", C.c_int32), ("K", C.c_int32),
                ("batch", C.c_int32), ("dtype", C.c_int32), ("t", C.POINTER(C.c_int32))]


_lib = None
_torch = None


def library_path():
    return _LIB_PATH


def lib():
    """Loads libheatkv.so; there is no fallback when it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is not built; run `python -m paper_2605_14877_amd.build`")
    # The library must share PyTorch's HIP runtime (streams and device pointers cross the boundary):
    # importing torch first makes its libamdhip64.so.7 the one the dynamic linker binds us to.
    import torch
    global _torch
    _torch = torch
    L = C.CDLL(_LIB_PATH)
    vp, i32p, u8p, f32p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_uint8), C.POINTER(C.c_float)
    sp = C.POINTER(_CShape)
    L.heatkv_last_error.restype = C.c_char_p
    L.heatkv_last_error.argtypes = []
    L.heatkv_calibrate_workspace_bytes.restype = C.c_size_t
    L.heatkv_calibrate_workspace_bytes.argtypes = [sp, C.c_int]
    L.heatkv_calibrate.restype = C.c_int
    L.heatkv_calibrate.argtypes = [sp, C.c_int, C.c_int, vp, vp, C.c_float, vp, vp, C.c_size_t, vp]
    L.heatkv_calibrate_static.restype = C.c_int
    L.heatkv_calibrate_static.argtypes = [sp, C.c_int, C.c_int, vp, vp, C.c_float, vp, vp]
    L.heatkv_calibrate_accumulate.restype = C.c_int
    L.heatkv_calibrate_accumulate.argtypes = [sp, C.c_int, C.c_int, vp, vp, C.c_float, C.c_float, vp, vp, vp,
                                              C.c_size_t, vp]
    L.heatkv_calibrate_scales_workspace_bytes.restype = C.c_size_t
    L.heatkv_calibrate_scales_workspace_bytes.argtypes = [sp, C.c_int, i32p]
    L.heatkv_calibrate_scales_accumulate.restype = C.c_int
    L.heatkv_calibrate_scales_accumulate.argtypes = [sp, C.c_int, C.c_int, i32p, C.POINTER(vp), C.POINTER(vp),
                                                     C.c_float, C.c_float, vp, C.POINTER(vp), vp, C.c_size_t, vp]
    L.heatkv_accumulate_beta.restype = C.c_int
    L.heatkv_accumulate_beta.argtypes = [sp, C.c_int, C.c_int, vp, C.c_float, vp, vp]
    L.heatkv_build_schedule.restype = C.c_int
    L.heatkv_build_schedule.argtypes = [sp, f32p, C.c_uint64, C.c_int, C.c_int, C.POINTER(vp)]
    L.heatkv_load_schedule.restype = C.c_int
    L.heatkv_load_schedule.argtypes = [sp, u8p, C.POINTER(vp)]
    L.heatkv_build_schedule_kv.restype = C.c_int
    L.heatkv_build_schedule_kv.argtypes = [sp, f32p, C.c_uint64, C.c_int, C.c_int, C.c_int, C.POINTER(vp)]
    L.heatkv_load_schedule_kv.restype = C.c_int
    L.heatkv_load_schedule_kv.argtypes = [sp, u8p, C.c_int, C.POINTER(vp)]
    L.heatkv_plan_kv_format.restype = C.c_int
    L.heatkv_plan_kv_format.argtypes = [vp]
    L.heatkv_plan_destroy.restype = None
    L.heatkv_plan_destroy.argtypes = [vp]
    L.heatkv_plan_upload.restype = C.c_int
    L.heatkv_plan_upload.argtypes = [vp]
    L.heatkv_plan_budget_tokens.restype = C.c_int64
    L.heatkv_plan_budget_tokens.argtypes = [vp]
    L.heatkv_plan_N.restype = C.c_int
    L.heatkv_plan_N.argtypes = [vp, i32p]
    L.heatkv_plan_order.restype = C.c_int
    L.heatkv_plan_order.argtypes = [vp, C.c_int, i32p]
    L.heatkv_plan_sets.restype = C.c_int
    L.heatkv_plan_sets.argtypes = [vp, C.c_int, C.c_int, u8p]
    L.heatkv_plan_retained.restype = C.c_int
    L.heatkv_plan_retained.argtypes = [vp, C.c_int, C.c_int, C.c_int, i32p, i32p]
    L.heatkv_plan_arena_tokens.restype = C.c_int64
    L.heatkv_plan_arena_tokens.argtypes = [vp]
    L.heatkv_plan_arena_bytes.restype = C.c_size_t
    L.heatkv_plan_arena_bytes.argtypes = [vp]
    L.heatkv_plan_runs.restype = C.c_int
    L.heatkv_plan_runs.argtypes = [vp, C.c_int, C.c_int, i32p, i32p]
    L.heatkv_plan_live_tokens.restype = C.c_int64
    L.heatkv_plan_live_tokens.argtypes = [vp, C.c_int, C.c_int]
    L.heatkv_append_scale.restype = C.c_int
    L.heatkv_append_scale.argtypes = [vp, C.c_int, C.c_int, vp, vp, vp, vp, vp]
    L.heatkv_attend_workspace_bytes.restype = C.c_size_t
    L.heatkv_attend_workspace_bytes.argtypes = [vp, C.c_int, C.c_int]
    L.heatkv_attend_scale.restype = C.c_int
    L.heatkv_attend_scale.argtypes = [vp, C.c_int, C.c_int, vp, vp, vp, vp, vp, C.c_float, vp, vp, C.c_size_t, vp]
    L.heatkv_attend_append_scale.restype = C.c_int
    L.heatkv_attend_append_scale.argtypes = [vp, C.c_int, C.c_int, vp, vp, vp, vp, vp, C.c_float, vp, vp, C.c_size_t, vp]
    f64p = C.POINTER(C.c_double)
    L.heatkv_head_scores.restype = C.c_int
    L.heatkv_head_scores.argtypes = [sp, f32p, C.c_int, C.c_int, f64p]
    L.heatkv_rank_dispersion.restype = C.c_int
    L.heatkv_rank_dispersion.argtypes = [sp, f32p, C.c_int, C.c_int, C.c_int, f64p]
    _lib = L
    return L


def _check(rc):
    if rc != 0:
        raise HeatKVError(rc, lib().heatkv_last_error().decode())


def _i32p(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


class Shape:
    """Problem shape (Sec. 3.1 notation); keeps the token list alive for the C struct."""

    def __init__(self, L, H, d, t, batch, dtype):
        self.L, self.H, self.d, self.batch = int(L), int(H), int(d), int(batch)
        self.t = np.ascontiguousarray(t, dtype=np.int32)
        self.K = int(self.t.size)
        self.dtype = _DTYPES[dtype] if isinstance(dtype, str) else int(dtype)
        self.c_struct = _CShape(self.L, self.H, self.d, self.K, self.batch, self.dtype, _i32p(self.t))

    @property
    def ref(self):
        return C.byref(self.c_struct)

    @property
    def elem_size(self):
        return 2 if self.dtype == BF16 else 4


def _ptr(x):
    """Device (or host) address of a torch tensor / numpy array / None."""
    if x is None:
        return None
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    if not x.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return x.data_ptr()


# The kernels trust the sizes the plan / shape imply, so the operands are checked here, on the host, before
# any pointer crosses the boundary: a wrong tensor becomes a Python error, not a memory fault on the GPU.
def _check_tensor(x, name, shape=None, dtype_code=None, min_bytes=None):
    if x is None:
        return
    torch = _torch
    if not isinstance(x, torch.Tensor):
        raise TypeError(f"{name}: expected a torch tensor")
    if not x.is_cuda:
        raise ValueError(f"{name}: expected a device tensor")
    if not x.is_contiguous():
        raise ValueError(f"{name}: tensor must be contiguous")
    if shape is not None and x.shape != shape:
        raise ValueError(f"{name}: shape {tuple(x.shape)} does not match {tuple(shape)}")
    if dtype_code is not None and x.dtype is not (torch.bfloat16 if dtype_code == BF16 else torch.float32):
        raise ValueError(f"{name}: dtype {x.dtype} does not match the plan's")
    if min_bytes is not None and x.numel() * x.element_size() < min_bytes:
        raise ValueError(f"{name}: {x.numel() * x.element_size()} bytes, at least {min_bytes} needed")


def _check_scale_operands(plan, layer, k, named, arenas):
    sh = plan.shape
    if not (0 <= layer < sh.L and 0 <= k < sh.K):
        return  # the library reports the index error
    cur = plan.scale_shapes[k]
    dt = sh.dtype
    for name, x in named:
        _check_tensor(x, name, cur, dt)
    nbytes = plan.arena_bytes_cached
    for name, x in arenas:
        _check_tensor(x, name, None, None, nbytes)


def _check_calibrate_operands(shape, k1, q, k_all, mass, beta):
    if not 0 <= k1 < shape.K:
        return
    t_k, c_k = int(shape.t[k1]), int(shape.t[: k1 + 1].sum())
    _check_tensor(q, "q", (shape.batch, shape.H, t_k, shape.d), shape.dtype)
    _check_tensor(k_all, "k_all", (shape.batch, shape.H, c_k, shape.d), shape.dtype)
    _check_tensor(mass, "mass", (shape.batch, shape.H, shape.K), F32)
    _check_tensor(beta, "beta", (shape.L, shape.H, shape.K, shape.K), F32)


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


class Plan:
    """Owner of a heatkv_plan handle."""

    def __init__(self, handle, shape):
        self.handle = C.c_void_p(handle)
        self.shape = shape
        # what the per-scale tensors and the arenas must look like (checked by the wrappers on every call)
        self.scale_shapes = [(shape.batch, shape.H, int(t), shape.d) for t in shape.t]
        self.arena_bytes_cached = int(lib().heatkv_plan_arena_bytes(self.handle))

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.heatkv_plan_destroy(self.handle)
            self.handle = None

    # --- inspection -----------------------------------------------------
    @property
    def budget_tokens(self):
        return int(lib().heatkv_plan_budget_tokens(self.handle))

    @property
    def kv_format(self):
        return int(lib().heatkv_plan_kv_format(self.handle))

    @property
    def arena_tokens(self):
        return int(lib().heatkv_plan_arena_tokens(self.handle))

    @property
    def arena_bytes(self):
        return int(lib().heatkv_plan_arena_bytes(self.handle))

    def N(self):
        out = np.zeros(max(self.shape.K - 1, 0), dtype=np.int32)
        _check(lib().heatkv_plan_N(self.handle, _i32p(out)))
        return out

    def order(self, i):
        out = np.zeros(self.shape.L * self.shape.H, dtype=np.int32)
        _check(lib().heatkv_plan_order(self.handle, i, _i32p(out)))
        return out

    def sets(self, k, which):
        out = np.zeros((self.shape.K, self.shape.L * self.shape.H), dtype=np.uint8)
        _check(lib().heatkv_plan_sets(self.handle, k, which, out.ctypes.data_as(C.POINTER(C.c_uint8))))
        return out

    def retained(self, k, layer, head):
        n = C.c_int32(0)
        _check(lib().heatkv_plan_retained(self.handle, k, layer, head, None, C.byref(n)))
        out = np.zeros(n.value, dtype=np.int32)
        if n.value:
            _check(lib().heatkv_plan_retained(self.handle, k, layer, head, _i32p(out), C.byref(n)))
        return out

    def runs(self, k, layer):
        row = np.zeros(self.shape.H, dtype=np.int32)
        ln = np.zeros(self.shape.H, dtype=np.int32)
        _check(lib().heatkv_plan_runs(self.handle, k, layer, _i32p(row), _i32p(ln)))
        return row, ln

    def live_tokens(self, k, layer):
        return int(lib().heatkv_plan_live_tokens(self.handle, k, layer))

    def upload(self):
        _check(lib().heatkv_plan_upload(self.handle))

    def attend_workspace_bytes(self, layer, k):
        return int(lib().heatkv_attend_workspace_bytes(self.handle, layer, k))


def heatkv_build_schedule(shape, beta, budget_bytes_per_seq, sinks, variant=VARIANT_HEATKV, kv_format=KV_NATIVE):
    """kv_format != KV_NATIVE goes through heatkv_build_schedule_kv."""
    beta = np.ascontiguousarray(beta, dtype=np.float32)
    assert beta.shape == (shape.L, shape.H, shape.K, shape.K)
    h = C.c_void_p()
    bp = beta.ctypes.data_as(C.POINTER(C.c_float))
    if kv_format == KV_NATIVE:
        _check(lib().heatkv_build_schedule(shape.ref, bp, int(budget_bytes_per_seq), int(sinks), int(variant),
                                           C.byref(h)))
    else:
        _check(lib().heatkv_build_schedule_kv(shape.ref, bp, int(budget_bytes_per_seq), int(sinks), int(variant),
                                              int(kv_format), C.byref(h)))
    return Plan(h.value, shape)


heatkv_build_schedule_kv = heatkv_build_schedule


def heatkv_load_schedule(shape, present, kv_format=KV_NATIVE):
    present = np.ascontiguousarray(present, dtype=np.uint8)
    assert present.shape == (shape.K, shape.L, shape.H, shape.K)
    h = C.c_void_p()
    pp = present.ctypes.data_as(C.POINTER(C.c_uint8))
    if kv_format == KV_NATIVE:
        _check(lib().heatkv_load_schedule(shape.ref, pp, C.byref(h)))
    else:
        _check(lib().heatkv_load_schedule_kv(shape.ref, pp, int(kv_format), C.byref(h)))
    return Plan(h.value, shape)


heatkv_load_schedule_kv = heatkv_load_schedule


def calibrate_workspace_bytes(shape, k1):
    return int(lib().heatkv_calibrate_workspace_bytes(shape.ref, k1))


def heatkv_calibrate(shape, layer, k1, q, k_all, sm_scale, mass, ws, stream=None):
    _check_calibrate_operands(shape, k1, q, k_all, mass, None)
    _check_tensor(ws, "ws")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(lib().heatkv_calibrate(shape.ref, layer, k1, _ptr(q), _ptr(k_all), float(sm_scale), _ptr(mass),
                                  _ptr(ws), ws_bytes, _stream() if stream is None else stream))


calibrate = heatkv_calibrate


def heatkv_calibrate_static(shape, layer, k1, q, k_all, sm_scale, mass, stream=None):
    """heatkv_calibrate with the library's static workspace: no allocation, no workspace argument."""
    _check_calibrate_operands(shape, k1, q, k_all, mass, None)
    _check(lib().heatkv_calibrate_static(shape.ref, layer, k1, _ptr(q), _ptr(k_all), float(sm_scale), _ptr(mass),
                                         _stream() if stream is None else stream))


def heatkv_accumulate_beta(shape, layer, k1, mass, weight, beta, stream=None):
    _check_calibrate_operands(shape, k1, None, None, mass, beta)
    _check(lib().heatkv_accumulate_beta(shape.ref, layer, k1, _ptr(mass), float(weight), _ptr(beta),
                                        _stream() if stream is None else stream))


def heatkv_append_scale(plan, layer, k, k_new, v_new, k_arena, v_arena, stream=None):
    _check_scale_operands(plan, layer, k, (("k_new", k_new), ("v_new", v_new)),
                          (("k_arena", k_arena), ("v_arena", v_arena)))
    _check(lib().heatkv_append_scale(plan.handle, layer, k, _ptr(k_new), _ptr(v_new), _ptr(k_arena), _ptr(v_arena),
                                     _stream() if stream is None else stream))


def heatkv_attend_scale(plan, layer, k, q, k_cur, v_cur, k_arena, v_arena, sm_scale, out, ws=None, stream=None):
    _check_scale_operands(plan, layer, k, (("q", q), ("k_cur", k_cur), ("v_cur", v_cur), ("out", out)),
                          (("k_arena", k_arena), ("v_arena", v_arena)))
    _check_tensor(ws, "ws")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(lib().heatkv_attend_scale(plan.handle, layer, k, _ptr(q), _ptr(k_cur), _ptr(v_cur), _ptr(k_arena),
                                     _ptr(v_arena), float(sm_scale), _ptr(out), _ptr(ws), ws_bytes,
                                     _stream() if stream is None else stream))


def heatkv_attend_append_scale(plan, layer, k, q, k_cur, v_cur, k_arena, v_arena, sm_scale, out, ws=None, stream=None):
    _check_scale_operands(plan, layer, k, (("q", q), ("k_cur", k_cur), ("v_cur", v_cur), ("out", out)),
                          (("k_arena", k_arena), ("v_arena", v_arena)))
    _check_tensor(ws, "ws")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(lib().heatkv_attend_append_scale(plan.handle, layer, k, _ptr(q), _ptr(k_cur), _ptr(v_cur), _ptr(k_arena),
                                            _ptr(v_arena), float(sm_scale), _ptr(out), _ptr(ws), ws_bytes,
                                            _stream() if stream is None else stream))


def heatkv_calibrate_accumulate(shape, layer, k1, q, k_all, sm_scale, weight, beta, mass, ws, stream=None):
    _check_calibrate_operands(shape, k1, q, k_all, mass, beta)
    _check_tensor(ws, "ws")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(lib().heatkv_calibrate_accumulate(shape.ref, layer, k1, _ptr(q), _ptr(k_all), float(sm_scale),
                                             float(weight), _ptr(beta), _ptr(mass), _ptr(ws), ws_bytes,
                                             _stream() if stream is None else stream))


def calibrate_scales_workspace_bytes(shape, k1_list):
    k1 = (C.c_int32 * len(k1_list))(*[int(k) for k in k1_list])
    return int(lib().heatkv_calibrate_scales_workspace_bytes(shape.ref, len(k1_list), k1))


def heatkv_calibrate_scales_accumulate(shape, layer, k1_list, q_list, k_all_list, sm_scale, weight, beta, mass_list,
                                       ws, stream=None):
    """Eq. 2 masses of several query scales and their dataset average in one launch (see include/heatkv.h).
    q_list / k_all_list: one tensor per entry of k1_list; mass_list: None or one tensor-or-None per entry."""
    n = len(k1_list)
    if len(q_list) != n or len(k_all_list) != n or (mass_list is not None and len(mass_list) != n):
        raise ValueError("k1_list, q_list, k_all_list and mass_list must have the same length")
    for i, k1 in enumerate(k1_list):
        _check_calibrate_operands(shape, int(k1), q_list[i], k_all_list[i],
                                  None if mass_list is None else mass_list[i], beta)
    _check_tensor(ws, "ws")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    k1 = (C.c_int32 * n)(*[int(k) for k in k1_list])
    qp = (C.c_void_p * n)(*[_ptr(x) for x in q_list])
    kp = (C.c_void_p * n)(*[_ptr(x) for x in k_all_list])
    mp = None if mass_list is None else (C.c_void_p * n)(*[_ptr(x) for x in mass_list])
    _check(lib().heatkv_calibrate_scales_accumulate(shape.ref, layer, n, k1, qp, kp, float(sm_scale), float(weight),
                                                    _ptr(beta), mp, _ptr(ws), ws_bytes,
                                                    _stream() if stream is None else stream))


def heatkv_head_scores(shape, beta, sinks, variant=VARIANT_HEATKV):
    """[K][T] fp64 scores behind the orders (Eq. 3 / Eq. 4 sums); beta: host [L,H,K,K] float32."""
    beta = np.ascontiguousarray(beta, dtype=np.float32)
    out = np.zeros((shape.K, shape.L * shape.H), dtype=np.float64)
    _check(lib().heatkv_head_scores(shape.ref, beta.ctypes.data_as(C.POINTER(C.c_float)), int(sinks), int(variant),
                                    out.ctypes.data_as(C.POINTER(C.c_double))))
    return out


def heatkv_rank_dispersion(shape, betas, sinks, variant=VARIANT_HEATKV):
    """[K] fp64 rank-position dispersion over runs (App. C); betas: host [runs,L,H,K,K] float32."""
    betas = np.ascontiguousarray(betas, dtype=np.float32)
    out = np.zeros(shape.K, dtype=np.float64)
    _check(lib().heatkv_rank_dispersion(shape.ref, betas.ctypes.data_as(C.POINTER(C.c_float)), int(betas.shape[0]),
                                        int(sinks), int(variant), out.ctypes.data_as(C.POINTER(C.c_double))))
    return out
