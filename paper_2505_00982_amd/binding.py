"""ctypes binding of libfosi_hip.so: argument marshalling only.

torch supplies device memory (tensor.data_ptr()) and the HIP stream; every
step of the path runs inside the library's kernels.  There is no fallback: if
the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Callable, Optional, Tuple

import numpy as np
import torch  # imported first on purpose: the library binds to the HIP runtime torch has loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libfosi_hip.so"
_lib = None

STATUS = {0: "OK", -1: "INVALID_ARG", -2: "BAD_LAYOUT", -3: "RANK", -4: "NONFINITE", -5: "HIP", -6: "NOMEM",
          -7: "CALLBACK", -8: "LIMIT"}
PROF = {"hvp_project": 0, "hvp_expand": 1, "reorth_dot": 2, "reorth_sub": 3, "normalise": 4, "ritz_vectors": 5,
        "step": 6, "admm": 7, "hvp_ggn": 8, "hvp_other": 9, "step_project": 10, "step_complement": 11, "step_apply": 12,
        "traffic_model": 13}

EXPORTS = [
    "fosi_ctx_create", "fosi_ctx_destroy", "fosi_ctx_synchronize", "fosi_last_error", "fosi_status_string",
    "hvp_planted_create", "hvp_diag_create", "hvp_softmax_ggn_create", "hvp_softmax_ggn_bf16_create", "hvp_callback_create", "hvp_apply",
    "hvp_destroy", "fosi_workspace_bytes", "fosi_lanczos", "fosi_lanczos_begin", "fosi_lanczos_end", "fosi_graph_stats", "fosi_lanczos_second_passes",
    "fosi_lanczos_row_sharded", "fosi_lanczos_steps", "fosi_tridiag_eigh", "fosi_ritz", "fosi_step", "fosi_step_noalloc", "fosi_step_adamw", "fosi_admm_begin",
    "fosi_admm_end", "fosi_traffic_model", "fosi_profile_enable", "fosi_profile_reset", "fosi_profile_read",
]


class FosiError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"fosi status {status} ({STATUS.get(status, '?')}): {message}")
        self.status = status


class _LanczosOpts(C.Structure):
    _fields_ = [("reorth_mode", C.c_int32), ("breakdown_tol", C.c_double), ("graph_mode", C.c_int32),
                ("reorth_eta", C.c_double)]


class _StepParams(C.Structure):
    _fields_ = [("alpha", C.c_float), ("lr", C.c_float), ("momentum", C.c_float), ("sigma", C.c_float),
                ("curv_mode", C.c_int32)]


class _AdamwParams(C.Structure):
    _fields_ = [("alpha", C.c_float), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float), ("sigma", C.c_float), ("curv_mode", C.c_int32)]


HVP_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p)


def library_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library() -> C.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it with `python -m paper_2505_00982_amd.build` (there is no CPU fallback)")
    lib = C.CDLL(path)
    vp, i64, i32, dp = C.c_void_p, C.c_int64, C.c_int32, C.POINTER(C.c_double)
    lib.fosi_ctx_create.argtypes = [C.POINTER(vp), C.c_int, vp]
    lib.fosi_ctx_destroy.argtypes = [vp]
    lib.fosi_ctx_synchronize.argtypes = [vp]
    lib.fosi_last_error.argtypes = [vp]
    lib.fosi_last_error.restype = C.c_char_p
    lib.fosi_status_string.argtypes = [i32]
    lib.fosi_status_string.restype = C.c_char_p
    lib.hvp_planted_create.argtypes = [vp, i64, C.c_int, vp, i64, vp, C.c_float, C.POINTER(vp)]
    lib.hvp_diag_create.argtypes = [vp, i64, vp, C.POINTER(vp)]
    lib.hvp_softmax_ggn_create.argtypes = [vp, C.c_int, C.c_int, C.c_int, vp, vp, C.POINTER(vp)]
    lib.hvp_softmax_ggn_bf16_create.argtypes = [vp, C.c_int, C.c_int, C.c_int, vp, vp, C.POINTER(vp)]
    lib.hvp_callback_create.argtypes = [vp, i64, HVP_FN, vp, C.POINTER(vp)]
    lib.hvp_apply.argtypes = [vp, vp, vp]
    lib.hvp_destroy.argtypes = [vp]
    lib.fosi_lanczos.argtypes = [vp, vp, i64, C.c_int, vp, i64, dp, dp, C.POINTER(i32), C.POINTER(_LanczosOpts)]
    lib.fosi_lanczos_begin.argtypes = [vp, vp, i64, C.c_int, vp, i64, C.POINTER(_LanczosOpts)]
    lib.fosi_lanczos_end.argtypes = [vp, dp, dp, C.POINTER(i32)]
    lib.fosi_lanczos_row_sharded.argtypes = [vp, vp, i64, C.c_int, C.c_int, vp, i64, dp, dp, C.POINTER(i32),
                                             C.POINTER(_LanczosOpts)]
    lib.fosi_workspace_bytes.argtypes = [i64, C.c_int, C.c_int]
    lib.fosi_workspace_bytes.restype = C.c_size_t
    lib.fosi_graph_stats.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.fosi_lanczos_second_passes.argtypes = [vp, C.POINTER(C.c_int32)]
    lib.fosi_lanczos_steps.argtypes = [i64, C.c_int, C.c_int]
    lib.fosi_tridiag_eigh.argtypes = [C.c_int, dp, dp, dp, dp]
    lib.fosi_ritz.argtypes = [vp, i64, C.c_int, vp, i64, dp, dp, C.c_int, C.c_int, vp, i64, dp, dp]
    lib.fosi_step.argtypes = [vp, i64, C.c_int, vp, i64, dp, vp, vp, vp, vp, C.POINTER(_StepParams)]
    lib.fosi_step_noalloc.argtypes = [vp, i64, C.c_int, vp, i64, dp, vp, vp, vp, vp, C.POINTER(_StepParams)]
    lib.fosi_step_adamw.argtypes = [vp, i64, C.c_int, vp, i64, dp, vp, vp, vp, vp, vp, vp, i64, C.POINTER(_AdamwParams)]
    lib.fosi_admm_begin.argtypes = [vp, i64, C.c_float, vp, vp, vp]
    lib.fosi_admm_end.argtypes = [vp, i64, C.c_float, vp, vp, vp]
    lib.fosi_traffic_model.argtypes = [vp, i64, vp, i64, C.c_int, vp, i64, C.c_int]
    lib.fosi_profile_enable.argtypes = [vp, C.c_int]
    lib.fosi_profile_reset.argtypes = [vp]
    lib.fosi_profile_read.argtypes = [vp, C.c_int, C.POINTER(i64), dp, dp]
    for name in EXPORTS:
        if name not in ("fosi_last_error", "fosi_status_string", "fosi_workspace_bytes"):
            getattr(lib, name).restype = i32
    _lib = lib
    return lib


def _dptr(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if t.dtype != torch.float32 or not t.is_cuda:
        raise TypeError("expected an fp32 device tensor")
    return t.data_ptr()


@dataclass
class StepParams:
    alpha: float = 0.1
    lr: float = 0.01
    momentum: float = 0.9
    sigma: float = 5e-4
    curv_mode: int = 0


class ColMajor:
    """n x cols fp32 column-major matrix in one flat device tensor with leading dimension ld."""

    def __init__(self, n: int, cols: int, ld: Optional[int] = None, device="cuda:0", buf: Optional[torch.Tensor] = None):
        self.n, self.cols = int(n), int(cols)
        self.ld = int(ld) if ld is not None else (self.n + 63) // 64 * 64
        if buf is None:
            buf = torch.zeros(self.ld * max(self.cols, 1), dtype=torch.float32, device=device)
        self.buf = buf

    @classmethod
    def from_numpy(cls, A: np.ndarray, ld: Optional[int] = None, device="cuda:0", extra_cols: int = 0) -> "ColMajor":
        n, c = A.shape
        M = cls(n, c + extra_cols, ld, device)
        host = np.zeros((c + extra_cols, M.ld), dtype=np.float32)
        host[:c, :n] = np.asarray(A, dtype=np.float32).T
        M.buf.copy_(torch.from_numpy(host.reshape(-1)))
        return M

    def col(self, j: int) -> torch.Tensor:
        return self.buf[j * self.ld: j * self.ld + self.n]

    def to_numpy(self, cols: Optional[int] = None) -> np.ndarray:
        c = self.cols if cols is None else cols
        return self.buf[: c * self.ld].reshape(c, self.ld)[:, : self.n].T.cpu().numpy()

    @property
    def ptr(self) -> int:
        return self.buf.data_ptr()


class Context:
    def __init__(self, device: int = 0, stream: Optional[torch.cuda.Stream] = None):
        self.lib = load_library()
        self.device = int(device)
        if stream is None:
            stream = torch.cuda.current_stream(self.device)
        self.stream = stream
        h = C.c_void_p()
        st = self.lib.fosi_ctx_create(C.byref(h), self.device, C.c_void_p(stream.cuda_stream))
        if st != 0:
            raise FosiError(st, "fosi_ctx_create failed")
        self.handle = h

    def check(self, st: int):
        if st != 0:
            raise FosiError(st, self.lib.fosi_last_error(self.handle).decode())

    def synchronize(self):
        self.check(self.lib.fosi_ctx_synchronize(self.handle))

    def close(self):
        if getattr(self, "handle", None):
            self.lib.fosi_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- operators
    def hvp_planted(self, U: ColMajor, lam: torch.Tensor, shift: float) -> "Hvp":
        h = C.c_void_p()
        self.check(self.lib.hvp_planted_create(self.handle, U.n, U.cols, U.ptr, U.ld, _ptr(lam), float(shift), C.byref(h)))
        return Hvp(self, h, U.n, keep=(U, lam))

    def hvp_diag(self, d: torch.Tensor) -> "Hvp":
        h = C.c_void_p()
        self.check(self.lib.hvp_diag_create(self.handle, d.numel(), _ptr(d), C.byref(h)))
        return Hvp(self, h, d.numel(), keep=(d,))

    def hvp_softmax_ggn(self, X: torch.Tensor, W: torch.Tensor) -> "Hvp":
        B, d = X.shape
        d2, Cc = W.shape
        assert d == d2 and X.is_contiguous() and W.is_contiguous()
        h = C.c_void_p()
        self.check(self.lib.hvp_softmax_ggn_create(self.handle, B, d, Cc, _ptr(X), _ptr(W), C.byref(h)))
        return Hvp(self, h, d * Cc, keep=(X, W))

    def hvp_softmax_ggn_bf16(self, X: torch.Tensor, W: torch.Tensor) -> "Hvp":
        """X: B x d torch.bfloat16 (the operator is defined by exactly these values), W: d x C float32."""
        B, d = X.shape
        d2, Cc = W.shape
        assert X.dtype == torch.bfloat16 and W.dtype == torch.float32
        assert d == d2 and X.is_contiguous() and W.is_contiguous()
        h = C.c_void_p()
        assert X.is_cuda
        self.check(self.lib.hvp_softmax_ggn_bf16_create(self.handle, B, d, Cc, X.data_ptr(), _ptr(W), C.byref(h)))
        return Hvp(self, h, d * Cc, keep=(X, W))

    def hvp_callback(self, n: int, fn: Callable[[int, int, int], int]) -> "Hvp":
        """fn(v_ptr, hv_ptr, stream_ptr) -> 0 on success; the pointers are raw device addresses."""
        def tramp(_user, v, hv, stream):
            try:
                return int(fn(v, hv, stream))
            except Exception:
                return 1
        cb = HVP_FN(tramp)
        h = C.c_void_p()
        self.check(self.lib.hvp_callback_create(self.handle, n, cb, None, C.byref(h)))
        return Hvp(self, h, n, keep=(cb, fn))

    # -- timers
    def profile_enable(self, on=True):
        """True / False: every kernel class / none; a class name or a list of names: only those classes."""
        if isinstance(on, str):
            on = [on]
        if isinstance(on, (list, tuple)):
            mask = 0
            for name in on:
                mask |= 1 << (PROF[name] + 1)
            on = mask
        self.check(self.lib.fosi_profile_enable(self.handle, int(on)))

    def profile_reset(self):
        self.check(self.lib.fosi_profile_reset(self.handle))

    def profile_read(self, cls) -> Tuple[int, float, float]:
        if isinstance(cls, str):
            cls = PROF[cls]
        n, ms, by = C.c_int64(), C.c_double(), C.c_double()
        self.check(self.lib.fosi_profile_read(self.handle, cls, C.byref(n), C.byref(ms), C.byref(by)))
        return n.value, ms.value, by.value

    def workspace_bytes(self, n: int = 1, m: int = 1, r_v: int = 0) -> int:
        """Device memory a context holds for itself for sizes (n, m, r_v); the same for every admissible size."""
        return int(self.lib.fosi_workspace_bytes(n, m, r_v))

    def graph_stats(self) -> Tuple[int, int]:
        """(captures, replays) of HIP graphs by fosi_lanczos on this context."""
        c, r = C.c_int64(), C.c_int64()
        self.check(self.lib.fosi_graph_stats(self.handle, C.byref(c), C.byref(r)))
        return c.value, r.value


class Hvp:
    def __init__(self, ctx: Context, handle, n: int, keep=()):
        self.ctx, self.handle, self.n, self._keep = ctx, handle, int(n), keep

    def apply(self, v: torch.Tensor, hv: torch.Tensor):
        self.ctx.check(self.ctx.lib.hvp_apply(self.handle, _ptr(v), _ptr(hv)))

    def close(self):
        if self.handle:
            self.ctx.lib.hvp_destroy(self.handle)
            self.handle = None


REORTH_SINGLE, REORTH_TWICE, REORTH_LOCAL_FULL, REORTH_SELECTIVE = 1, 2, 3, 4
GRAPH_OFF, GRAPH_ON = 0, 1


def fosi_lanczos(ctx: Context, op: Hvp, Q: ColMajor, m: int, reorth_mode: int = 0,
                 breakdown_tol: float = 1e-6, graph_mode: int = 0,
                 reorth_eta: float = 0.0) -> Tuple[np.ndarray, np.ndarray, int]:
    """Q.col(0) holds the start vector.  reorth_mode 0 = library default; graph_mode 1 = capture the
    run into a HIP graph and replay it (0, default: eager launches); reorth_eta: threshold of the second pass
    of REORTH_SELECTIVE (0 = 1/sqrt 2).  Returns (alpha, beta, m_eff)."""
    alpha, beta = np.zeros(m), np.zeros(m)
    m_eff = C.c_int32(0)
    opts = _LanczosOpts(reorth_mode, breakdown_tol, graph_mode, reorth_eta)
    ctx.check(ctx.lib.fosi_lanczos(ctx.handle, op.handle, Q.n, m, Q.ptr, Q.ld, _dptr(alpha), _dptr(beta),
                                   C.byref(m_eff), C.byref(opts)))
    return alpha, beta, int(m_eff.value)


def fosi_lanczos_begin(ctx: Context, op: Hvp, Q: ColMajor, m: int, reorth_mode: int = 0, breakdown_tol: float = 1e-6,
                       graph_mode: int = 0, reorth_eta: float = 0.0) -> int:
    """Enqueues the whole run on the context's stream without waiting for the GPU; returns m for fosi_lanczos_end."""
    opts = _LanczosOpts(reorth_mode, breakdown_tol, graph_mode, reorth_eta)
    ctx.check(ctx.lib.fosi_lanczos_begin(ctx.handle, op.handle, Q.n, m, Q.ptr, Q.ld, C.byref(opts)))
    return m


def fosi_lanczos_end(ctx: Context, m: int) -> Tuple[np.ndarray, np.ndarray, int]:
    """Waits for the run started by fosi_lanczos_begin(..., m); returns (alpha, beta, m_eff)."""
    alpha, beta = np.zeros(m), np.zeros(m)
    m_eff = C.c_int32(0)
    ctx.check(ctx.lib.fosi_lanczos_end(ctx.handle, _dptr(alpha), _dptr(beta), C.byref(m_eff)))
    return alpha, beta, int(m_eff.value)


def fosi_lanczos_row_sharded(ctx: Context, op: Hvp, Q: ColMajor, m: int, shards: int, reorth_mode: int = 0,
                             breakdown_tol: float = 1e-6) -> Tuple[np.ndarray, np.ndarray, int]:
    """Algorithm 2 emulated on one GPU with `shards` row blocks.  Same contract as fosi_lanczos."""
    alpha, beta = np.zeros(m), np.zeros(m)
    m_eff = C.c_int32(0)
    opts = _LanczosOpts(reorth_mode, breakdown_tol, 0, 0.0)
    ctx.check(ctx.lib.fosi_lanczos_row_sharded(ctx.handle, op.handle, Q.n, m, shards, Q.ptr, Q.ld, _dptr(alpha),
                                               _dptr(beta), C.byref(m_eff), C.byref(opts)))
    return alpha, beta, int(m_eff.value)


def fosi_lanczos_second_passes(ctx: Context) -> int:
    """Steps of the context's last completed run in which REORTH_SELECTIVE took its second pass."""
    c = C.c_int32(0)
    ctx.check(ctx.lib.fosi_lanczos_second_passes(ctx.handle, C.byref(c)))
    return int(c.value)


def fosi_lanczos_steps(n: int, k: int, l: int) -> int:
    return int(load_library().fosi_lanczos_steps(n, k, l))


def fosi_tridiag_eigh(alpha: np.ndarray, beta: np.ndarray, vectors: bool = True):
    lib = load_library()
    a = np.ascontiguousarray(alpha, dtype=np.float64)
    m = a.shape[0]
    b = np.zeros(max(m, 1))
    b[: max(m - 1, 0)] = np.asarray(beta, dtype=np.float64)[: max(m - 1, 0)]
    ev = np.zeros(m)
    Z = np.zeros((m, m), order="F") if vectors else None
    st = lib.fosi_tridiag_eigh(m, _dptr(a), _dptr(b), _dptr(ev), _dptr(Z) if vectors else None)
    if st != 0:
        raise FosiError(st, "fosi_tridiag_eigh failed")
    return (ev, Z) if vectors else ev


def fosi_ritz(ctx: Context, Q: ColMajor, m_eff: int, alpha: np.ndarray, beta: np.ndarray, k: int, l: int,
              V: ColMajor) -> Tuple[np.ndarray, np.ndarray]:
    """Writes the k+l Ritz vectors into V; returns (evals, resid)."""
    a = np.ascontiguousarray(alpha, dtype=np.float64)
    b = np.ascontiguousarray(beta, dtype=np.float64)
    evals, resid = np.zeros(max(k + l, 1)), np.zeros(max(k + l, 1))
    ctx.check(ctx.lib.fosi_ritz(ctx.handle, Q.n, m_eff, Q.ptr, Q.ld, _dptr(a), _dptr(b), k, l, V.ptr, V.ld,
                                _dptr(evals), _dptr(resid)))
    return evals[: k + l], resid[: k + l]


def fosi_step(ctx: Context, V: Optional[ColMajor], r_v: int, evals: Optional[np.ndarray], g: torch.Tensor,
              pi: Optional[torch.Tensor], mom: torch.Tensor, w: torch.Tensor, p: StepParams):
    n = w.numel()
    ev = np.ascontiguousarray(evals, dtype=np.float64) if r_v > 0 else np.zeros(1)
    sp = _StepParams(p.alpha, p.lr, p.momentum, p.sigma, p.curv_mode)
    ctx.check(ctx.lib.fosi_step(ctx.handle, n, r_v, V.ptr if r_v > 0 else None, V.ld if r_v > 0 else 0, _dptr(ev),
                                _ptr(g), _ptr(pi), _ptr(mom), _ptr(w), C.byref(sp)))


def fosi_step_noalloc(stream: Optional[torch.cuda.Stream], V: Optional[ColMajor], r_v: int, evals: Optional[np.ndarray],
                      g: torch.Tensor, pi: Optional[torch.Tensor], mom: torch.Tensor, w: torch.Tensor, p: StepParams):
    """fosi_step without a context and without any allocation (static device scratch); r_v <= 64.  `stream` None:
    torch's current stream on the current device."""
    lib = load_library()
    n = w.numel()
    if stream is None:
        stream = torch.cuda.current_stream()
    ev = np.ascontiguousarray(evals, dtype=np.float64) if r_v > 0 else np.zeros(1)
    sp = _StepParams(p.alpha, p.lr, p.momentum, p.sigma, p.curv_mode)
    st = lib.fosi_step_noalloc(C.c_void_p(stream.cuda_stream), n, r_v, V.ptr if r_v > 0 else None, V.ld if r_v > 0 else 0,
                               _dptr(ev), _ptr(g), _ptr(pi), _ptr(mom), _ptr(w), C.byref(sp))
    if st != 0:
        raise FosiError(st, lib.fosi_status_string(st).decode())


@dataclass
class AdamwParams:
    alpha: float = 0.1
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.05
    sigma: float = 5e-4
    curv_mode: int = 0


def fosi_step_adamw(ctx: Context, V: Optional[ColMajor], r_v: int, evals: Optional[np.ndarray], g: torch.Tensor,
                    pi: Optional[torch.Tensor], exp_avg: torch.Tensor, exp_avg_sq: torch.Tensor, work: torch.Tensor,
                    w: torch.Tensor, step_index: int, p: AdamwParams):
    n = w.numel()
    ev = np.ascontiguousarray(evals, dtype=np.float64) if r_v > 0 else np.zeros(1)
    ap = _AdamwParams(p.alpha, p.lr, p.beta1, p.beta2, p.eps, p.weight_decay, p.sigma, p.curv_mode)
    ctx.check(ctx.lib.fosi_step_adamw(ctx.handle, n, r_v, V.ptr if r_v > 0 else None, V.ld if r_v > 0 else 0, _dptr(ev),
                                      _ptr(g), _ptr(pi), _ptr(exp_avg), _ptr(exp_avg_sq), _ptr(work), _ptr(w),
                                      int(step_index), C.byref(ap)))


def fosi_admm_begin(ctx: Context, sigma: float, pi: torch.Tensor, w_anchor: torch.Tensor, wa: torch.Tensor):
    ctx.check(ctx.lib.fosi_admm_begin(ctx.handle, wa.numel(), float(sigma), _ptr(pi), _ptr(w_anchor), _ptr(wa)))


def fosi_admm_end(ctx: Context, sigma: float, w_anchor: torch.Tensor, wa: torch.Tensor, pi: torch.Tensor):
    ctx.check(ctx.lib.fosi_admm_end(ctx.handle, wa.numel(), float(sigma), _ptr(w_anchor), _ptr(wa), _ptr(pi)))


def fosi_traffic_model(ctx: Context, A: Optional[ColMajor], cols_in: int, B: Optional[ColMajor], cols_out: int, n: int):
    """Memory-only model of a sweep (measurement aid): cols_in columns of A read, cols_out columns of B written."""
    ctx.check(ctx.lib.fosi_traffic_model(ctx.handle, int(n), A.ptr if A is not None else None, A.ld if A is not None else 0,
                                         int(cols_in), B.ptr if B is not None else None, B.ld if B is not None else 0,
                                         int(cols_out)))
