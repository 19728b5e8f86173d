"""ctypes binding of the C ABI declared in include/muon.h.

Argument marshalling only: every arithmetic step of the Muon update runs inside the
HIP library.  PyTorch is used by callers for device memory and streams; this module
touches tensors only to read ``data_ptr()`` / shape / dtype.

The library is loaded from the package directory (built in-tree by ``build.py``).
There is no fallback: a missing library is an ImportError at first use.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Iterable, List, Optional, Sequence

MUON_F32, MUON_BF16 = 0, 1
MUON_BF16X2, MUON_BF16X3 = 2, 3     # Newton-Schulz arithmetic only: sums of two / three bf16 planes
NS_DTYPES = {"f32": MUON_F32, "bf16": MUON_BF16, "bf16x2": MUON_BF16X2, "bf16x3": MUON_BF16X3}
MUON_SCALE_ADJUSTED_LR, MUON_SCALE_BASELINE, MUON_SCALE_UPDATE_NORM = 0, 1, 2
MUON_OK = 0
STATUS_NAMES = {
    0: "MUON_OK", -1: "MUON_E_INVALID_ARG", -2: "MUON_E_UNSUPPORTED_DTYPE", -3: "MUON_E_SHAPE_MISMATCH",
    -4: "MUON_E_WORKSPACE_TOO_SMALL", -5: "MUON_E_HIP", -6: "MUON_E_NOT_RESIDENT", -7: "MUON_E_MISALIGNED", -8: "MUON_E_NO_MEMORY", -9: "MUON_E_STATIC_LIMIT",
}

EXPORTS = (
    "muon_default_hparams", "muon_workspace_bytes", "muon_init", "muon_step", "muon_debug_read_update",
    "muon_plan_describe", "muon_plan_chunks", "muon_destroy", "muon_status_string", "muon_last_hip_error",
    "muon_profile_enable", "muon_profile_read", "muon_adamw_step", "muon_probe_mfma_rate",
    "muon_plan_only", "muon_plan_tiles", "muon_step_static",
)
PROF_NAMES = ("momentum_norm_cast", "norm_finalize", "gram", "poly", "apply_poly", "weight_update", "update_rms")


class muon_param(C.Structure):
    _fields_ = [("w", C.c_void_p), ("g", C.c_void_p), ("m", C.c_void_p),
                ("rows", C.c_int64), ("cols", C.c_int64), ("w_dtype", C.c_int32), ("g_dtype", C.c_int32)]


class muon_hparams(C.Structure):
    _fields_ = [("lr", C.c_double), ("weight_decay", C.c_double), ("momentum", C.c_double),
                ("a", C.c_double), ("b", C.c_double), ("c", C.c_double),
                ("rms_scale", C.c_double), ("eps", C.c_double),
                ("ns_steps", C.c_int32), ("nesterov", C.c_int32),
                ("scale_mode", C.c_int32), ("reserved", C.c_int32), ("hidden_size", C.c_double),
                ("coeff_schedule", C.POINTER(C.c_double))]


class muon_adamw_param(C.Structure):
    _fields_ = [("p", C.c_void_p), ("g", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p),
                ("numel", C.c_int64), ("p_dtype", C.c_int32), ("g_dtype", C.c_int32)]


class muon_adamw_hparams(C.Structure):
    _fields_ = [("lr", C.c_double), ("weight_decay", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double), ("step", C.c_int64)]


class MuonError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = f"{where}: {STATUS_NAMES.get(status, status)}"
        try:
            msg += f" ({lib().muon_status_string(status).decode()})"
            if status == -5:
                msg += f" hipError={lib().muon_last_hip_error()}"
        except Exception:  # pragma: no cover
            pass
        super().__init__(msg)


_LIB = None


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmuon_hip.so")


def lib() -> C.CDLL:
    """Loads the HIP library (once).  Raises ImportError when it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2502_16982_amd.build` "
                          "(there is no CPU fallback)")
    L = C.CDLL(path)
    P = C.POINTER
    L.muon_default_hparams.argtypes = [P(muon_hparams)]
    L.muon_default_hparams.restype = C.c_int
    L.muon_workspace_bytes.argtypes = [P(muon_param), C.c_int32, C.c_int32, C.c_size_t, P(C.c_size_t)]
    L.muon_workspace_bytes.restype = C.c_int
    L.muon_init.argtypes = [P(C.c_void_p), P(muon_param), C.c_int32, C.c_int32, C.c_void_p, C.c_size_t]
    L.muon_init.restype = C.c_int
    L.muon_step.argtypes = [C.c_void_p, P(muon_param), C.c_int32, P(muon_hparams), C.c_void_p, C.c_void_p]
    L.muon_step.restype = C.c_int
    L.muon_step_static.argtypes = [P(muon_param), C.c_int32, C.c_int32, P(muon_hparams), C.c_void_p, C.c_void_p]
    L.muon_step_static.restype = C.c_int
    L.muon_debug_read_update.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]
    L.muon_debug_read_update.restype = C.c_int
    L.muon_plan_describe.argtypes = [C.c_void_p, C.c_int32, P(C.c_int64), C.c_int32]
    L.muon_plan_describe.restype = C.c_int
    L.muon_plan_chunks.argtypes = [C.c_void_p]
    L.muon_plan_chunks.restype = C.c_int
    L.muon_destroy.argtypes = [C.c_void_p]
    L.muon_destroy.restype = None
    L.muon_status_string.argtypes = [C.c_int]
    L.muon_status_string.restype = C.c_char_p
    L.muon_last_hip_error.argtypes = []
    L.muon_last_hip_error.restype = C.c_int
    L.muon_adamw_step.argtypes = [P(muon_adamw_param), C.c_int32, P(muon_adamw_hparams), C.c_void_p]
    L.muon_adamw_step.restype = C.c_int
    L.muon_profile_enable.argtypes = [C.c_void_p, C.c_int]
    L.muon_profile_enable.restype = C.c_int
    L.muon_profile_read.argtypes = [C.c_void_p, P(C.c_double), P(C.c_int64), C.c_int]
    L.muon_profile_read.restype = C.c_int
    L.muon_probe_mfma_rate.argtypes = [C.c_int, C.c_int, P(C.c_double), P(C.c_double)]
    L.muon_probe_mfma_rate.restype = C.c_int
    L.muon_plan_only.argtypes = [P(C.c_void_p), P(muon_param), C.c_int32, C.c_int32, C.c_size_t]
    L.muon_plan_only.restype = C.c_int
    L.muon_plan_tiles.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, P(C.c_int32), C.c_int32]
    L.muon_plan_tiles.restype = C.c_int
    _LIB = L
    return L


def _check(status: int, where: str) -> None:
    if status != MUON_OK:
        raise MuonError(status, where)


def muon_probe_mfma_rate(random_operands: bool = True, iters: int = 40000) -> dict:
    """Sustained bf16 matrix-core rate with register-resident operands: {"tflops", "clock_mhz"}."""
    tf, mhz = C.c_double(0.0), C.c_double(0.0)
    _check(lib().muon_probe_mfma_rate(1 if random_operands else 0, int(iters), C.byref(tf), C.byref(mhz)),
           "muon_probe_mfma_rate")
    return {"tflops": tf.value, "clock_mhz": mhz.value}


def dtype_code(torch_dtype) -> int:
    import torch
    if torch_dtype == torch.float32:
        return MUON_F32
    if torch_dtype == torch.bfloat16:
        return MUON_BF16
    raise MuonError(-2, f"dtype {torch_dtype}")


def default_hparams(**overrides) -> muon_hparams:
    hp = muon_hparams()
    _check(lib().muon_default_hparams(C.byref(hp)), "muon_default_hparams")
    for k, v in overrides.items():
        if not hasattr(hp, k):
            raise AttributeError(k)
        if k == "coeff_schedule":
            set_coeff_schedule(hp, v)
        else:
            setattr(hp, k, v)
    return hp


def set_coeff_schedule(hp: muon_hparams, schedule) -> None:
    """Attach per-iteration (a, b, c) triples (or None) to hp; sets ns_steps to their number.  The host array is
    kept alive by hp itself."""
    if schedule is None:
        hp.coeff_schedule = C.POINTER(C.c_double)()
        hp._schedule_keepalive = None
        return
    flat = [float(x) for triple in schedule for x in triple]
    if len(flat) % 3 or any(len(t) != 3 for t in schedule):
        raise ValueError("schedule must be a sequence of (a, b, c) triples")
    arr = (C.c_double * len(flat))(*flat)
    hp._schedule_keepalive = arr
    hp.coeff_schedule = C.cast(arr, C.POINTER(C.c_double))
    hp.ns_steps = len(flat) // 3


def param_array(shapes: Sequence[Sequence[int]], w_dtypes: Sequence[int], g_dtypes: Sequence[int]):
    arr = (muon_param * len(shapes))()
    for i, (r, c) in enumerate(shapes):
        arr[i].rows, arr[i].cols = int(r), int(c)
        arr[i].w_dtype, arr[i].g_dtype = int(w_dtypes[i]), int(g_dtypes[i])
    return arr


def muon_workspace_bytes(params, n: int, ns_dtype: int, max_bytes: int = 0) -> int:
    out = C.c_size_t(0)
    _check(lib().muon_workspace_bytes(params, n, ns_dtype, max_bytes, C.byref(out)), "muon_workspace_bytes")
    return int(out.value)


def muon_init(params, n: int, ns_dtype: int, workspace_ptr: int, workspace_bytes: int) -> C.c_void_p:
    ctx = C.c_void_p(None)
    _check(lib().muon_init(C.byref(ctx), params, n, ns_dtype, C.c_void_p(workspace_ptr), workspace_bytes), "muon_init")
    return ctx


def muon_step(ctx, params, n: int, hp: muon_hparams, stream_ptr: int = 0, update_rms_ptr: int = 0) -> None:
    _check(lib().muon_step(ctx, params, n, C.byref(hp), C.c_void_p(stream_ptr), C.c_void_p(update_rms_ptr)), "muon_step")


def muon_step_static(params, n: int, ns_dtype: int, hp: muon_hparams, stream_ptr: int = 0, update_rms_ptr: int = 0) -> None:
    """One step with the workspace inside the library (no device allocation anywhere in the call)."""
    _check(lib().muon_step_static(params, n, ns_dtype, C.byref(hp), C.c_void_p(stream_ptr), C.c_void_p(update_rms_ptr)),
           "muon_step_static")


def muon_debug_read_update(ctx, index: int, dst_ptr: int, dst_dtype: int, stream_ptr: int = 0) -> None:
    _check(lib().muon_debug_read_update(ctx, index, C.c_void_p(dst_ptr), dst_dtype, C.c_void_p(stream_ptr)),
           "muon_debug_read_update")


def muon_plan_describe(ctx, index: int) -> dict:
    buf = (C.c_int64 * 8)()
    k = lib().muon_plan_describe(ctx, index, buf, 8)
    if k < 0:
        raise MuonError(k, "muon_plan_describe")
    keys = ("m", "n", "transposed", "m_pad", "n_pad", "chunk", "tile_m", "tile_n")
    return dict(zip(keys, [int(v) for v in buf[:k]]))


def muon_plan_chunks(ctx) -> int:
    k = lib().muon_plan_chunks(ctx)
    if k < 0:
        raise MuonError(k, "muon_plan_chunks")
    return k


def muon_plan_only(params, n: int, ns_dtype: int, workspace_bytes: int) -> C.c_void_p:
    """Host-only launch plan (no device is touched); release with muon_destroy."""
    ctx = C.c_void_p(None)
    _check(lib().muon_plan_only(C.byref(ctx), params, n, ns_dtype, workspace_bytes), "muon_plan_only")
    return ctx


PLAN_PRODUCTS = {"gram": 0, "poly": 1, "apply": 2, "apply_last": 3}


def muon_plan_tiles(ctx, chunk: int, product: str, level: int) -> list:
    """Tile table of one grouped launch of a host-only plan: [(matrix, row0, col0, rows, cols, computed_blocks), ...]; offsets and extents in elements, blocks of 32 x 32."""
    count = lib().muon_plan_tiles(ctx, chunk, PLAN_PRODUCTS[product], level, None, 0)
    if count < 0:
        raise MuonError(count, "muon_plan_tiles")
    buf = (C.c_int32 * (6 * max(count, 1)))()
    got = lib().muon_plan_tiles(ctx, chunk, PLAN_PRODUCTS[product], level, buf, count)
    if got != count:
        raise MuonError(got if got < 0 else -1, "muon_plan_tiles")
    return [tuple(buf[6 * i:6 * i + 6]) for i in range(count)]


def muon_profile_enable(ctx, enable: bool) -> None:
    _check(lib().muon_profile_enable(ctx, int(bool(enable))), "muon_profile_enable")


def muon_profile_read(ctx, reset: bool = False) -> dict:
    """{kernel class: (milliseconds, launches)} accumulated since the last reset."""
    ms = (C.c_double * len(PROF_NAMES))()
    cnt = (C.c_int64 * len(PROF_NAMES))()
    _check(lib().muon_profile_read(ctx, ms, cnt, int(bool(reset))), "muon_profile_read")
    return {name: (float(ms[i]), int(cnt[i])) for i, name in enumerate(PROF_NAMES)}


def muon_adamw_step(tensors, *, lr: float, weight_decay: float, beta1: float = 0.9, beta2: float = 0.95,
                    eps: float = 1e-8, step: int = 1, stream_ptr: int = 0) -> None:
    """tensors: iterable of (p, g, m, v) torch tensors of one size each (any shape, contiguous)."""
    tensors = [tuple(t) for t in tensors]
    arr = (muon_adamw_param * max(len(tensors), 1))()
    for i, (p, g, m, v) in enumerate(tensors):
        if not (p.is_contiguous() and g.is_contiguous() and m.is_contiguous() and v.is_contiguous()):
            raise MuonError(-1, f"tensor {i}: buffers must be contiguous")
        if not (p.numel() == g.numel() == m.numel() == v.numel()):
            raise MuonError(-1, f"tensor {i}: p, g, m, v must have one size")
        if dtype_code(m.dtype) != MUON_F32 or dtype_code(v.dtype) != MUON_F32:
            raise MuonError(-2, f"tensor {i}: moments must be fp32")
        a = arr[i]
        a.p, a.g, a.m, a.v = p.data_ptr(), g.data_ptr(), m.data_ptr(), v.data_ptr()
        a.numel = p.numel()
        a.p_dtype, a.g_dtype = dtype_code(p.dtype), dtype_code(g.dtype)
    hp = muon_adamw_hparams(lr, weight_decay, beta1, beta2, eps, step)
    _check(lib().muon_adamw_step(arr, len(tensors), C.byref(hp), C.c_void_p(stream_ptr)), "muon_adamw_step")


def muon_destroy(ctx) -> None:
    lib().muon_destroy(ctx)


class MuonStepper:
    """Convenience holder: one context + workspace for a fixed list of (W, G, M) torch tensors.

    Marshals pointers and calls the C ABI; owns the workspace tensor.
    """

    def __init__(self, tensors: Iterable[tuple], ns_dtype: str = "bf16", max_workspace_bytes: int = 0):
        import torch
        self.tensors: List[tuple] = [tuple(t) for t in tensors]
        if not self.tensors:
            raise MuonError(-1, "empty parameter list")
        if ns_dtype not in NS_DTYPES:
            raise ValueError(f"ns_dtype must be one of {sorted(NS_DTYPES)}")
        self.ns_dtype = NS_DTYPES[ns_dtype]
        self.n = len(self.tensors)
        self.params = (muon_param * self.n)()
        self.device = self.tensors[0][0].device
        self.set_tensors(self.tensors)
        nbytes = muon_workspace_bytes(self.params, self.n, self.ns_dtype, max_workspace_bytes)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.workspace_bytes = nbytes
        self.ctx = muon_init(self.params, self.n, self.ns_dtype, self.workspace.data_ptr(), nbytes)

    def set_tensors(self, tensors) -> None:
        self.tensors = [tuple(t) for t in tensors]
        for i, (w, g, m) in enumerate(self.tensors):
            if w.dim() != 2 or g.shape != w.shape or m.shape != w.shape:
                raise MuonError(-1, f"matrix {i}: W, G, M must be 2-D and of one shape")
            if not (w.is_contiguous() and g.is_contiguous() and m.is_contiguous()):
                raise MuonError(-1, f"matrix {i}: buffers must be contiguous")
            p = self.params[i]
            p.w, p.g, p.m = w.data_ptr(), g.data_ptr(), m.data_ptr()
            p.rows, p.cols = w.shape
            p.w_dtype, p.g_dtype = dtype_code(w.dtype), dtype_code(g.dtype)
            if dtype_code(m.dtype) != MUON_F32:
                raise MuonError(-2, f"matrix {i}: momentum must be fp32")

    def step(self, hp: muon_hparams, stream=None, update_rms=None) -> None:
        import torch
        s = stream if stream is not None else torch.cuda.current_stream(self.device)
        muon_step(self.ctx, self.params, self.n, hp, s.cuda_stream,
                  0 if update_rms is None else update_rms.data_ptr())

    def read_update(self, index: int, dtype=None):
        import torch
        w = self.tensors[index][0]
        dtype = dtype or torch.float32
        out = torch.empty(w.shape, dtype=dtype, device=self.device)
        muon_debug_read_update(self.ctx, index, out.data_ptr(), dtype_code(dtype),
                               torch.cuda.current_stream(self.device).cuda_stream)
        return out

    def close(self) -> None:
        if getattr(self, "ctx", None) is not None:
            muon_destroy(self.ctx)
            self.ctx = None

    def __del__(self):  # pragma: no cover
        try:
            self.close()
        except Exception:
            pass
