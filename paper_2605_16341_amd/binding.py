"""ctypes binding of liborthdion.so: the same entry points as include/orthdion.h, plus a thin
convenience class.  Argument marshalling only - every step of the method runs in the HIP
kernels.  There is no CPU fallback: a missing library is an error."""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liborthdion.so")

ORTHDION_OK = 0
ORTHDION_E_INVALID_ARG = -1
ORTHDION_E_NULL_PTR = -2
ORTHDION_E_BAD_SHAPE = -3
ORTHDION_E_WORKSPACE_TOO_SMALL = -4
ORTHDION_E_MISALIGNED = -5
ORTHDION_E_HIP = -6
ORTHDION_E_NO_STEP = -7
ORTHDION_E_NO_MEMORY = -8

ORTHDION_F32, ORTHDION_BF16 = 0, 1
ORTHDION_QR, ORTHDION_COLNORM = 0, 1
ORTHDION_EF_DION, ORTHDION_EF_PAPER, ORTHDION_EF_POLYAK = 0, 1, 2
ORTHDION_PREC_AUTO, ORTHDION_PREC_FAST, ORTHDION_PREC_EXACT = 0, 1, 2

EXPORTS = ["orthdion_create", "orthdion_workspace_bytes", "orthdion_set_lr", "orthdion_set_mu",
           "orthdion_set_variant", "orthdion_step", "orthdion_get_info", "orthdion_workspace_layout",
           "orthdion_profile_begin", "orthdion_profile_end", "orthdion_set_diagnostics",
           "orthdion_get_diagnostics", "orthdion_rank_policy", "orthdion_resize_q", "orthdion_strerror",
           "orthdion_destroy", "orthdion_step_static", "orthdion_static_scratch_bytes", "orthdion_get_warnings",
           "orthdion_get_groups"]

DIAG = ["b_norm", "r_norm", "tracking_error", "residual_ratio", "inner", "nu", "erank", "g_norm"]
ORTHDION_NDIAG = len(DIAG)

PHASES = ["stats", "proj", "proj_reduce", "gram_left", "chol_left", "orth_left", "guard_left", "finish_left", "back",
          "back_reduce", "gram_right", "chol_right", "orth_right", "guard_right", "finish_right", "efx"]
ORTHDION_NPHASE = len(PHASES)


class orthdion_matdesc(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int64), ("n", ctypes.c_int64), ("r", ctypes.c_int32),
                ("ldx", ctypes.c_int64), ("ldg", ctypes.c_int64), ("ldm", ctypes.c_int64)]


class orthdion_config(ctypes.Structure):
    _fields_ = [("x_dtype", ctypes.c_int), ("g_dtype", ctypes.c_int), ("variant", ctypes.c_int),
                ("ef", ctypes.c_int), ("precision", ctypes.c_int), ("mu", ctypes.c_float),
                ("lr", ctypes.c_float), ("groups", ctypes.c_int32)]


_lib: Optional[ctypes.CDLL] = None


def _share_torch_hip_runtime() -> None:
    """PyTorch wheels ship their own copy of the HIP runtime (same SONAME as ROCm's).  Device
    pointers and streams are only meaningful inside one runtime instance, so when this
    library is loaded before torch it must bind to torch's copy, not to /opt/rocm's: map
    torch's copy first and the loader resolves our dependency to it by SONAME."""
    import importlib.util
    try:
        spec = importlib.util.find_spec("torch")
    except (ImportError, ValueError):
        spec = None
    if spec is None or not spec.submodule_search_locations:
        return
    cand = os.path.join(list(spec.submodule_search_locations)[0], "lib", "libamdhip64.so")
    if os.path.exists(cand):
        ctypes.CDLL(cand, mode=ctypes.RTLD_GLOBAL)


def load() -> ctypes.CDLL:
    """Loads the in-tree library (built by build.py); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_16341_amd.build` "
                           "(there is no fallback path)")
    _share_torch_hip_runtime()
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    lib.orthdion_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(orthdion_matdesc), ctypes.c_int32,
                                    ctypes.POINTER(orthdion_config)]
    lib.orthdion_create.restype = ctypes.c_int
    lib.orthdion_workspace_bytes.argtypes = [vp]
    lib.orthdion_workspace_bytes.restype = sz
    lib.orthdion_get_groups.argtypes = [vp]
    lib.orthdion_get_groups.restype = ctypes.c_int32
    lib.orthdion_set_lr.argtypes = [vp, ctypes.c_float]
    lib.orthdion_set_lr.restype = ctypes.c_int
    lib.orthdion_set_mu.argtypes = [vp, ctypes.c_float]
    lib.orthdion_set_mu.restype = ctypes.c_int
    lib.orthdion_set_variant.argtypes = [vp, ctypes.c_int]
    lib.orthdion_set_variant.restype = ctypes.c_int
    lib.orthdion_step.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                  ctypes.POINTER(vp), vp, sz, vp]
    lib.orthdion_step.restype = ctypes.c_int
    lib.orthdion_step_static.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                         ctypes.POINTER(vp), vp]
    lib.orthdion_step_static.restype = ctypes.c_int
    lib.orthdion_static_scratch_bytes.argtypes = []
    lib.orthdion_static_scratch_bytes.restype = sz
    lib.orthdion_get_info.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), vp]
    lib.orthdion_get_info.restype = ctypes.c_int
    lib.orthdion_get_warnings.argtypes = [vp, ctypes.POINTER(ctypes.c_uint32), vp]
    lib.orthdion_get_warnings.restype = ctypes.c_int
    lib.orthdion_workspace_layout.argtypes = [vp, ctypes.c_int32] + [ctypes.POINTER(sz)] * 6
    lib.orthdion_workspace_layout.restype = ctypes.c_int
    lib.orthdion_profile_begin.argtypes = [vp, ctypes.c_uint32, ctypes.c_int32]
    lib.orthdion_profile_begin.restype = ctypes.c_int
    lib.orthdion_profile_end.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int32)]
    lib.orthdion_profile_end.restype = ctypes.c_int
    lib.orthdion_set_diagnostics.argtypes = [vp, ctypes.c_int32]
    lib.orthdion_set_diagnostics.restype = ctypes.c_int
    lib.orthdion_get_diagnostics.argtypes = [vp, ctypes.POINTER(ctypes.c_float), vp]
    lib.orthdion_get_diagnostics.restype = ctypes.c_int
    lib.orthdion_rank_policy.argtypes = [ctypes.c_float, ctypes.c_float, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_float, ctypes.c_float, ctypes.POINTER(ctypes.c_float),
                                         ctypes.POINTER(ctypes.c_int32)]
    lib.orthdion_rank_policy.restype = ctypes.c_int
    lib.orthdion_resize_q.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, vp, ctypes.c_int32, vp, vp]
    lib.orthdion_resize_q.restype = ctypes.c_int
    lib.orthdion_strerror.argtypes = [ctypes.c_int]
    lib.orthdion_strerror.restype = ctypes.c_char_p
    lib.orthdion_destroy.argtypes = [vp]
    lib.orthdion_destroy.restype = ctypes.c_int
    _lib = lib
    return lib


class OrthDionError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"orthdion status {status}: {orthdion_strerror(status)}")


def orthdion_strerror(status: int) -> str:
    return load().orthdion_strerror(int(status)).decode()


def _check(status: int) -> None:
    if status != ORTHDION_OK:
        raise OrthDionError(status)


def orthdion_create(shapes: Sequence[Sequence[int]], r, x_dtype: int, g_dtype: int, variant: int = ORTHDION_QR,
                    ef: int = ORTHDION_EF_DION, precision: int = ORTHDION_PREC_AUTO, mu: float = 0.95,
                    lr: float = 0.01, lds: Optional[Sequence[Sequence[int]]] = None, groups: int = 0) -> int:
    """`shapes` is a list of (m, n); `r` one rank or one per matrix; `lds` optional
    (ldx, ldg, ldm) per matrix (default n); `groups` 0 (the library chooses), 1 or 2.  Returns
    the opaque handle as an int."""
    lib = load()
    nmat = len(shapes)
    ranks = [int(r)] * nmat if isinstance(r, int) else [int(v) for v in r]
    descs = (orthdion_matdesc * max(nmat, 1))()
    for i, (m, n) in enumerate(shapes):
        ld = lds[i] if lds is not None else (n, n, n)
        descs[i] = orthdion_matdesc(int(m), int(n), ranks[i], int(ld[0]), int(ld[1]), int(ld[2]))
    cfg = orthdion_config(int(x_dtype), int(g_dtype), int(variant), int(ef), int(precision), float(mu), float(lr), int(groups))
    handle = ctypes.c_void_p()
    _check(lib.orthdion_create(ctypes.byref(handle), descs, nmat, ctypes.byref(cfg)))
    return handle.value


def orthdion_workspace_bytes(handle: int) -> int:
    return int(load().orthdion_workspace_bytes(handle))


def orthdion_get_groups(handle: int) -> int:
    return int(load().orthdion_get_groups(handle))


def orthdion_set_lr(handle: int, lr: float) -> None:
    _check(load().orthdion_set_lr(handle, float(lr)))


def orthdion_set_mu(handle: int, mu: float) -> None:
    _check(load().orthdion_set_mu(handle, float(mu)))


def orthdion_set_variant(handle: int, variant: int) -> None:
    _check(load().orthdion_set_variant(handle, int(variant)))


def _ptr_array(ptrs: Sequence[int]):
    arr = (ctypes.c_void_p * len(ptrs))()
    for i, p in enumerate(ptrs):
        arr[i] = p
    return arr


def orthdion_step(handle: int, X: Sequence[int], G: Sequence[int], M: Sequence[int], Q: Sequence[int],
                  workspace: int, workspace_bytes: int, stream: int = 0) -> None:
    """X, G, M, Q: device addresses (ints), one per matrix; `stream` a hipStream_t as int."""
    _check(load().orthdion_step(handle, _ptr_array(X), _ptr_array(G), _ptr_array(M), _ptr_array(Q),
                                ctypes.c_void_p(workspace), workspace_bytes, ctypes.c_void_p(stream)))


def orthdion_step_static(handle: int, X: Sequence[int], G: Sequence[int], M: Sequence[int], Q: Sequence[int],
                         stream: int = 0) -> None:
    """orthdion_step on the library's own device scratch (no workspace argument)."""
    _check(load().orthdion_step_static(handle, _ptr_array(X), _ptr_array(G), _ptr_array(M), _ptr_array(Q),
                                       ctypes.c_void_p(stream)))


def orthdion_static_scratch_bytes() -> int:
    return int(load().orthdion_static_scratch_bytes())


def orthdion_get_info(handle: int, nmat: int, stream: int = 0) -> List[int]:
    out = (ctypes.c_int32 * nmat)()
    _check(load().orthdion_get_info(handle, out, ctypes.c_void_p(stream)))
    return list(out)


WARN_B_CLIPPED, WARN_R_CLIPPED, WARN_B_SCALE_BLIND, WARN_WAIT_EXPIRED = 1, 2, 4, 8


def orthdion_get_warnings(handle: int, nmat: int, stream: int = 0) -> List[int]:
    out = (ctypes.c_uint32 * nmat)()
    _check(load().orthdion_get_warnings(handle, out, ctypes.c_void_p(stream)))
    return list(out)


def orthdion_workspace_layout(handle: int, index: int) -> dict:
    vals = [ctypes.c_size_t() for _ in range(6)]
    _check(load().orthdion_workspace_layout(handle, int(index), *[ctypes.byref(v) for v in vals]))
    keys = ["P", "R", "T_P1", "T_P2", "T_Q1", "T_Q2"]
    return {k: int(v.value) for k, v in zip(keys, vals)}


def orthdion_profile_begin(handle: int, phase_mask: int, max_steps: int) -> None:
    _check(load().orthdion_profile_begin(handle, int(phase_mask), int(max_steps)))


def orthdion_profile_end(handle: int) -> dict:
    """{phase name: (total milliseconds, intervals)} for the phases that were bracketed."""
    ms = (ctypes.c_float * ORTHDION_NPHASE)()
    cnt = (ctypes.c_int32 * ORTHDION_NPHASE)()
    _check(load().orthdion_profile_end(handle, ms, cnt))
    return {PHASES[i]: (float(ms[i]), int(cnt[i])) for i in range(ORTHDION_NPHASE) if cnt[i] > 0}


def orthdion_set_diagnostics(handle: int, enable: bool) -> None:
    _check(load().orthdion_set_diagnostics(handle, 1 if enable else 0))


def orthdion_get_diagnostics(handle: int, nmat: int, stream: int = 0) -> List[dict]:
    """One {name: value} dict per matrix for the most recent step (names in DIAG)."""
    out = (ctypes.c_float * (nmat * ORTHDION_NDIAG))()
    _check(load().orthdion_get_diagnostics(handle, out, ctypes.c_void_p(stream)))
    return [{DIAG[k]: float(out[i * ORTHDION_NDIAG + k]) for k in range(ORTHDION_NDIAG)} for i in range(nmat)]


def orthdion_rank_policy(e_t: float, ema_prev: float, r_min: int, r_max: int, alpha: float, gamma: float):
    """(new EMA, next rank) of the adaptive-rank rule."""
    ema, nxt = ctypes.c_float(), ctypes.c_int32()
    _check(load().orthdion_rank_policy(float(e_t), float(ema_prev), int(r_min), int(r_max), float(alpha),
                                       float(gamma), ctypes.byref(ema), ctypes.byref(nxt)))
    return float(ema.value), int(nxt.value)


def orthdion_resize_q(q_old: int, n: int, r_old: int, q_new: int, r_new: int, pad: int = 0, stream: int = 0) -> None:
    """Device addresses as ints; `pad` may be 0 only when the rank does not grow."""
    _check(load().orthdion_resize_q(ctypes.c_void_p(q_old), int(n), int(r_old), ctypes.c_void_p(q_new), int(r_new),
                                    ctypes.c_void_p(pad or None), ctypes.c_void_p(stream)))


def orthdion_destroy(handle: int) -> None:
    _check(load().orthdion_destroy(handle))


class OrthDion:
    """Owns a handle and a torch-allocated workspace; `step` takes lists of torch tensors
    (device memory and the current stream come from torch; nothing else does)."""

    def __init__(self, shapes, r, x_dtype="bf16", g_dtype=None, variant="qr", ef="dion", precision="auto",
                 mu=0.95, lr=0.01, device="cuda:0", groups=0):
        import torch
        g_dtype = g_dtype or x_dtype
        dt = {"f32": ORTHDION_F32, "bf16": ORTHDION_BF16}
        self.shapes = [tuple(s) for s in shapes]
        self.nmat = len(self.shapes)
        self.r = r
        self._x_dtype = {"f32": torch.float32, "bf16": torch.bfloat16}[x_dtype]
        self._g_dtype = {"f32": torch.float32, "bf16": torch.bfloat16}[g_dtype]
        self.handle = orthdion_create(self.shapes, r, dt[x_dtype], dt[g_dtype],
                                      {"qr": ORTHDION_QR, "colnorm": ORTHDION_COLNORM}[variant],
                                      {"dion": ORTHDION_EF_DION, "paper": ORTHDION_EF_PAPER, "polyak": ORTHDION_EF_POLYAK}[ef],
                                      {"auto": ORTHDION_PREC_AUTO, "fast": ORTHDION_PREC_FAST,
                                       "exact": ORTHDION_PREC_EXACT}[precision], mu, lr, groups=groups)
        self.workspace_bytes = orthdion_workspace_bytes(self.handle)
        self.groups = orthdion_get_groups(self.handle)
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=device)
        self._torch = torch

    def _check_buffers(self, X, G, M, Q) -> None:
        """The library sees raw addresses only: a tensor of the wrong type, shape or layout
        would be read and written out of bounds, so it is refused here."""
        torch = self._torch
        for name, seq in (("X", X), ("G", G), ("M", M), ("Q", Q)):
            if len(seq) != self.nmat:
                raise ValueError(f"{name}: expected {self.nmat} tensors, got {len(seq)}")
        for i, (m, n) in enumerate(self.shapes):
            r = self.r if isinstance(self.r, int) else self.r[i]
            want = {"X": ((m, n), self._x_dtype), "G": ((m, n), self._g_dtype), "M": ((m, n), torch.float32),
                    "Q": ((n, r), torch.float32)}
            for name, t in (("X", X[i]), ("G", G[i]), ("M", M[i]), ("Q", Q[i])):
                shape, dtype = want[name]
                if not t.is_cuda or tuple(t.shape) != shape or t.dtype != dtype or not t.is_contiguous():
                    raise ValueError(f"{name}[{i}]: need a contiguous {dtype} device tensor of shape {shape}, got "
                                     f"{t.dtype} {tuple(t.shape)} on {t.device}, contiguous={t.is_contiguous()}")

    def step(self, X, G, M, Q, stream=None) -> None:
        torch = self._torch
        self._check_buffers(X, G, M, Q)
        st = stream if stream is not None else torch.cuda.current_stream().cuda_stream
        orthdion_step(self.handle, [t.data_ptr() for t in X], [t.data_ptr() for t in G],
                      [t.data_ptr() for t in M], [t.data_ptr() for t in Q],
                      self.workspace.data_ptr(), self.workspace_bytes, st)

    def info(self, stream=None) -> List[int]:
        st = stream if stream is not None else self._torch.cuda.current_stream().cuda_stream
        return orthdion_get_info(self.handle, self.nmat, st)

    def warnings(self, stream=None) -> List[int]:
        st = stream if stream is not None else self._torch.cuda.current_stream().cuda_stream
        return orthdion_get_warnings(self.handle, self.nmat, st)

    def set_diagnostics(self, enable: bool) -> None:
        orthdion_set_diagnostics(self.handle, enable)

    def diagnostics(self, stream=None) -> List[dict]:
        st = stream if stream is not None else self._torch.cuda.current_stream().cuda_stream
        return orthdion_get_diagnostics(self.handle, self.nmat, st)

    def debug_factors(self, index: int) -> dict:
        """P, R and the triangular factors the last step left in the workspace (copies)."""
        torch = self._torch
        lay = orthdion_workspace_layout(self.handle, index)
        m, n = self.shapes[index]
        r = self.r if isinstance(self.r, int) else self.r[index]
        out = {}
        for key, (rows, cols) in {"P": (m, r), "R": (n, r), "T_P1": (r, r), "T_P2": (r, r), "T_Q1": (r, r),
                                  "T_Q2": (r, r)}.items():
            nbytes = rows * cols * 4
            out[key] = self.workspace[lay[key]:lay[key] + nbytes].view(torch.float32).reshape(rows, cols).clone()
        return out

    def set_lr(self, lr: float) -> None:
        orthdion_set_lr(self.handle, lr)

    def set_mu(self, mu: float) -> None:
        orthdion_set_mu(self.handle, mu)

    def set_variant(self, variant: str) -> None:
        orthdion_set_variant(self.handle, {"qr": ORTHDION_QR, "colnorm": ORTHDION_COLNORM}[variant])

    def close(self) -> None:
        if self.handle:
            orthdion_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
