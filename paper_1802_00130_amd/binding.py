"""ctypes binding of libdn.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; torch is used to own device
memory and to name the stream.  There is no CPU fallback: if libdn.so is missing or does not
load, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

DN_FULL = 0
DN_BLOCKDIAG = 1
DN_PARTITION = 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[ctypes.CDLL] = None

_c_float_p = ctypes.c_void_p  # device pointers travel as integers


class NewtonParams(ctypes.Structure):
    """dn_newton_params of include/dn.h."""
    _fields_ = [("lam", ctypes.c_double), ("sigma", ctypes.c_double), ("eta", ctypes.c_double),
                ("eps", ctypes.c_double), ("drop", ctypes.c_double), ("boost", ctypes.c_double),
                ("cg_max", ctypes.c_int), ("mode", ctypes.c_int), ("combine", ctypes.c_int),
                ("max_trials", ctypes.c_int), ("cg_min", ctypes.c_int), ("r_percent", ctypes.c_double),
                ("reuse_forward", ctypes.c_int)]


class NewtonStats(ctypes.Structure):
    """dn_newton_stats of include/dn.h."""
    _fields_ = [("f_old", ctypes.c_double), ("f_new", ctypes.c_double), ("alpha", ctypes.c_double),
                ("beta1", ctypes.c_double), ("beta2", ctypes.c_double), ("rho", ctypes.c_double),
                ("gTd", ctypes.c_double), ("dGd", ctypes.c_double), ("cg_iters", ctypes.c_int),
                ("f_evals", ctypes.c_int)]


class DnError(RuntimeError):
    def __init__(self, code: int, where: str, hip: int = 0):
        self.code = code
        msg = f"{where}: {load_library().dn_strerror(code).decode()} (code {code}"
        msg += f", hip error {hip})" if hip else ")"
        super().__init__(msg)


def lib_path() -> str:
    return os.path.join(_HERE, "libdn.so")


def load_library() -> ctypes.CDLL:
    """Load libdn.so built in-tree (paper_1802_00130_amd/build.py); raise if it is not there."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not built: run `python -m paper_1802_00130_amd.build` "
                                "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(path)
    vp, i, d, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_double, ctypes.c_size_t
    P = ctypes.POINTER
    sig = {
        "dn_strerror": (ctypes.c_char_p, [i]),
        "dn_create": (i, [P(vp), i, P(i), d, i, i]),
        "dn_destroy": (None, [vp]),
        "dn_num_params": (sz, [vp]),
        "dn_workspace_bytes": (sz, [vp]),
        "dn_product_slices": (i, [vp, i]),
        "dn_gemm_large_tiles": (i, [i, P(i), P(i), P(i), P(i)]),
        "dn_bind": (i, [vp, vp, sz, vp]),
        "dn_forward": (i, [vp, vp, vp, vp, i, P(d), vp]),
        "dn_forward_static": (i, [i, P(i), d, vp, vp, vp, i, vp, P(d), vp]),
        "dn_grad": (i, [vp, vp, vp, vp, i, vp, P(d)]),
        "dn_jacobian_prep": (i, [vp, vp, vp, i, vp, i]),
        "dn_jacobian_read": (i, [vp, i, vp]),
        "dn_gn_matvec": (i, [vp, vp, vp, i]),
        "dn_gn_matvec_rop": (i, [vp, vp, vp]),
        "dn_cg": (i, [vp, vp, d, d, i, i, vp, P(i), P(d)]),
        "dn_cg_sync": (i, [vp, vp, d, d, i, i, i, d, vp, P(i), P(d)]),
        "dn_set_split": (i, [vp, P(i)]),
        "dn_num_partitions": (i, [vp]),
        "dn_newton_step": (i, [vp, vp, vp, vp, i, vp, i, vp, P(NewtonParams), P(NewtonStats)]),
        "dn_set_stream_passes": (i, [vp, i]),
        "dn_set_spin_limit": (i, [vp, ctypes.c_uint]),
        "dn_sync_status": (i, [vp]),
        "dn_profile_enable": (i, [vp, i]),
        "dn_profile_select": (i, [vp, ctypes.c_ulonglong]),
        "dn_profile_reset": (i, [vp]),
        "dn_profile_num_classes": (i, []),
        "dn_profile_class_name": (ctypes.c_char_p, [i]),
        "dn_profile_read": (i, [vp, i, P(d), P(ctypes.c_longlong)]),
        "dn_profile_band_phases": (i, [vp, i]),
        "dn_profile_band_read": (i, [vp, P(d), P(d)]),
        "dn_last_hip_error": (i, [vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _LIB = lib
    return lib


EXPORTED_SYMBOLS = (
    "dn_strerror", "dn_create", "dn_destroy", "dn_num_params", "dn_workspace_bytes", "dn_product_slices", "dn_gemm_large_tiles", "dn_bind",
    "dn_forward",
    "dn_forward_static", "dn_grad", "dn_jacobian_prep", "dn_jacobian_read", "dn_gn_matvec", "dn_gn_matvec_rop", "dn_cg", "dn_cg_sync",
    "dn_set_split", "dn_num_partitions", "dn_newton_step", "dn_set_stream_passes", "dn_set_spin_limit",
    "dn_sync_status", "dn_profile_enable", "dn_profile_select", "dn_profile_reset", "dn_profile_num_classes",
    "dn_profile_class_name", "dn_profile_read", "dn_profile_band_phases", "dn_profile_band_read", "dn_last_hip_error",
)


def _dev_f32(t: torch.Tensor, name: str, numel: Optional[int] = None) -> int:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError(f"{name}: need a contiguous float32 device tensor")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"{name}: expected {numel} elements, got {t.numel()}")
    return t.data_ptr()


class Context:
    """Owns a dn_ctx and the torch tensor that backs its workspace."""

    def __init__(self, dims: Sequence[int], C: float, l_max: int, s_max: int,
                 device: str = "cuda:0", stream: Optional[torch.cuda.Stream] = None):
        self._lib = load_library()
        self.dims = tuple(int(x) for x in dims)
        self.L = len(self.dims) - 1
        self._h = ctypes.c_void_p()
        arr = (ctypes.c_int * len(self.dims))(*self.dims)
        rc = self._lib.dn_create(ctypes.byref(self._h), self.L, arr, float(C), int(l_max), int(s_max))
        if rc != 0:
            raise DnError(rc, "dn_create")
        self.n = int(self._lib.dn_num_params(self._h))
        self.device = torch.device(device)
        self.workspace_bytes = int(self._lib.dn_workspace_bytes(self._h))
        self.workspace = torch.zeros(self.workspace_bytes // 4 + 64, dtype=torch.float32, device=self.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        rc = self._lib.dn_bind(self._h, self._ws_ptr, self.workspace_bytes, self.stream.cuda_stream)
        self._check(rc, "dn_bind")
        self.s = 0

    def _check(self, rc: int, where: str) -> None:
        if rc != 0:
            raise DnError(rc, where, int(self._lib.dn_last_hip_error(self._h)))

    def close(self) -> None:
        if getattr(self, "_h", None) and self._h.value:
            self._lib.dn_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):  # pragma: no cover
        try:
            self.close()
        except Exception:
            pass

    def set_split(self, groups: Sequence[int]) -> int:
        """Split structure for DN_PARTITION (neuron groups per layer, Section 3.1); returns the partition count."""
        arr = (ctypes.c_int * len(self.dims))(*[int(x) for x in groups])
        if len(groups) != len(self.dims):
            raise ValueError("one group count per layer, input layer included")
        self._check(self._lib.dn_set_split(self._h, arr), "dn_set_split")
        return int(self._lib.dn_num_partitions(self._h))

    def num_systems(self, mode: int) -> int:
        if mode == DN_PARTITION:
            return int(self._lib.dn_num_partitions(self._h))
        return self.L if mode == DN_BLOCKDIAG else 1

    # -- single-pass (team) kernel controls --------------------------------------------------
    def set_stream_passes(self, passes: int) -> None:
        """0: automatic (one read of the stored blocks where available); 2: always the two-pass kernels."""
        self._check(self._lib.dn_set_stream_passes(self._h, int(passes)), "dn_set_stream_passes")

    def set_spin_limit(self, polls: int) -> None:
        self._check(self._lib.dn_set_spin_limit(self._h, int(polls)), "dn_set_spin_limit")

    def sync_status(self) -> int:
        """Wait for the stream; returns the library's status code (0, or DN_ETIMEOUT = -6) without raising."""
        return int(self._lib.dn_sync_status(self._h))

    def rebind(self) -> None:
        """Bind the same workspace again (clears a reported time-out and the stored Jacobian)."""
        self._check(self._lib.dn_bind(self._h, self._ws_ptr, self.workspace_bytes, self.stream.cuda_stream), "dn_bind")
        self.s = 0

    # -- profiling ---------------------------------------------------------------------------
    def profile_enable(self, on: bool) -> None:
        self._check(self._lib.dn_profile_enable(self._h, int(on)), "dn_profile_enable")

    def profile_select(self, names=None) -> None:
        """Bracket only the named kernel classes (None = all)."""
        mask = 0
        for k in range(self._lib.dn_profile_num_classes()):
            if names is None or self._lib.dn_profile_class_name(k).decode() in names:
                mask |= 1 << k
        self._check(self._lib.dn_profile_select(self._h, mask), "dn_profile_select")

    def profile_reset(self) -> None:
        self._check(self._lib.dn_profile_reset(self._h), "dn_profile_reset")

    def profile_band_phases(self, on: bool) -> None:
        """Phase clocks of the single-pass kernel for wide outputs on or off."""
        self._check(self._lib.dn_profile_band_phases(self._h, int(on)), "dn_profile_band_phases")

    def profile_band_read(self) -> dict:
        """Mean shader-clock cycles per band of the last clocked launch: loading, waiting for the exchange, rest."""
        cyc = (ctypes.c_double * 3)()
        bands = ctypes.c_double()
        self._check(self._lib.dn_profile_band_read(self._h, cyc, ctypes.byref(bands)), "dn_profile_band_read")
        return {"load_cycles": cyc[0], "exchange_wait_cycles": cyc[1], "transposed_product_cycles": cyc[2],
                "bands_per_work_group": bands.value}

    def profile_read(self) -> dict:
        out = {}
        for k in range(self._lib.dn_profile_num_classes()):
            ms, cnt = ctypes.c_double(), ctypes.c_longlong()
            self._check(self._lib.dn_profile_read(self._h, k, ctypes.byref(ms), ctypes.byref(cnt)), "dn_profile_read")
            out[self._lib.dn_profile_class_name(k).decode()] = (ms.value, cnt.value)
        return out


def dn_forward(ctx: Context, theta: torch.Tensor, X: torch.Tensor, Y: torch.Tensor,
               ZL: Optional[torch.Tensor] = None) -> float:
    """f(theta) on all rows of X, Y (Section 2.1 objective)."""
    l = X.shape[0]
    f = ctypes.c_double()
    zl = 0 if ZL is None else _dev_f32(ZL, "ZL", l * ctx.dims[-1])
    rc = ctx._lib.dn_forward(ctx._h, _dev_f32(theta, "theta", ctx.n), _dev_f32(X, "X", l * ctx.dims[0]),
                             _dev_f32(Y, "Y", l * ctx.dims[-1]), l, ctypes.byref(f), zl)
    ctx._check(rc, "dn_forward")
    return f.value


STATIC_SCRATCH_BYTES = 32 << 20


def dn_forward_static(dims: Sequence[int], C: float, theta: torch.Tensor, X: torch.Tensor, Y: torch.Tensor,
                      ZL: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> float:
    """f(theta) as dn_forward, through the entry point that allocates nothing (no context, no workspace: the
    library's fixed scratch).  Raises DnError with code -7 when the problem exceeds that scratch."""
    lib = load_library()
    dims = tuple(int(x) for x in dims)
    l = X.shape[0]
    n = sum(dims[m - 1] * dims[m] + dims[m] for m in range(1, len(dims)))
    arr = (ctypes.c_int * len(dims))(*dims)
    f = ctypes.c_double()
    zl = 0 if ZL is None else _dev_f32(ZL, "ZL", l * dims[-1])
    st = stream if stream is not None else torch.cuda.current_stream(X.device)
    rc = lib.dn_forward_static(len(dims) - 1, arr, float(C), _dev_f32(theta, "theta", n),
                               _dev_f32(X, "X", l * dims[0]), _dev_f32(Y, "Y", l * dims[-1]), l, st.cuda_stream,
                               ctypes.byref(f), zl)
    if rc != 0:
        raise DnError(rc, "dn_forward_static")
    return f.value


def dn_grad(ctx: Context, theta: torch.Tensor, X: torch.Tensor, Y: torch.Tensor, g: torch.Tensor,
            want_f: bool = True) -> Optional[float]:
    """g = grad f(theta) (Section 2.2 back-propagation); returns f when want_f."""
    l = X.shape[0]
    f = ctypes.c_double()
    rc = ctx._lib.dn_grad(ctx._h, _dev_f32(theta, "theta", ctx.n), _dev_f32(X, "X", l * ctx.dims[0]),
                          _dev_f32(Y, "Y", l * ctx.dims[-1]), l, _dev_f32(g, "g", ctx.n),
                          ctypes.byref(f) if want_f else None)
    ctx._check(rc, "dn_grad")
    return f.value if want_f else None


def dn_jacobian_prep(ctx: Context, theta: torch.Tensor, X: torch.Tensor, S: torch.Tensor) -> None:
    """Store dz^L/ds^m for the rows S of X (Section 3.3)."""
    if not (S.is_cuda and S.dtype == torch.int32 and S.is_contiguous()):
        raise TypeError("S: need a contiguous int32 device tensor")
    l = X.shape[0]
    rc = ctx._lib.dn_jacobian_prep(ctx._h, _dev_f32(theta, "theta", ctx.n), _dev_f32(X, "X", l * ctx.dims[0]), l,
                                   S.data_ptr(), S.numel())
    ctx._check(rc, "dn_jacobian_prep")
    ctx.s = S.numel()


def dn_jacobian_read(ctx: Context, m: int, P_out: torch.Tensor) -> None:
    rc = ctx._lib.dn_jacobian_read(ctx._h, int(m), _dev_f32(P_out, "P_out", ctx.s * ctx.dims[-1] * ctx.dims[m]))
    ctx._check(rc, "dn_jacobian_read")


def dn_gn_matvec(ctx: Context, v: torch.Tensor, out: torch.Tensor, mode: int = DN_FULL) -> None:
    """out = G^S v, full or per-layer block-diagonal (Sections 4.1-4.3)."""
    rc = ctx._lib.dn_gn_matvec(ctx._h, _dev_f32(v, "v", ctx.n), _dev_f32(out, "out", ctx.n), int(mode))
    ctx._check(rc, "dn_gn_matvec")


def dn_gn_matvec_rop(ctx: Context, v: torch.Tensor, out: torch.Tensor) -> None:
    """out = G^S v without the stored blocks (forward-mode pass, then back-propagation; Section 2.2's alternative)."""
    rc = ctx._lib.dn_gn_matvec_rop(ctx._h, _dev_f32(v, "v", ctx.n), _dev_f32(out, "out", ctx.n))
    ctx._check(rc, "dn_gn_matvec_rop")


def dn_cg(ctx: Context, g: torch.Tensor, lam: float, sigma: float, max_iter: int, mode: int,
          d: torch.Tensor) -> Tuple[int, list]:
    """CG on (G^S + lam I) d = -g; returns (iterations, residual norms)."""
    iters = ctypes.c_int()
    nres = ctx.num_systems(mode)
    res = (ctypes.c_double * max(nres, 1))()
    rc = ctx._lib.dn_cg(ctx._h, _dev_f32(g, "g", ctx.n), float(lam), float(sigma), int(max_iter), int(mode),
                        _dev_f32(d, "d", ctx.n), ctypes.byref(iters), res)
    ctx._check(rc, "dn_cg")
    return iters.value, [res[k] for k in range(nres)]


def dn_cg_sync(ctx: Context, g: torch.Tensor, lam: float, sigma: float, max_iter: int, cg_min: int,
               r_percent: float, d: torch.Tensor, mode: int = DN_BLOCKDIAG) -> Tuple[int, list]:
    """CG on independent systems with the joint early termination of Section 4.4; returns (iterations,
    residual norms)."""
    iters = ctypes.c_int()
    nres = max(ctx.num_systems(mode), 1)
    res = (ctypes.c_double * nres)()
    rc = ctx._lib.dn_cg_sync(ctx._h, _dev_f32(g, "g", ctx.n), float(lam), float(sigma), int(max_iter), int(mode),
                             int(cg_min), float(r_percent), _dev_f32(d, "d", ctx.n), ctypes.byref(iters), res)
    ctx._check(rc, "dn_cg_sync")
    return iters.value, [res[k] for k in range(nres)]


def dn_newton_step(ctx: Context, theta: torch.Tensor, X: torch.Tensor, Y: torch.Tensor, S: torch.Tensor,
                   d_prev: torch.Tensor, lam: float, cg_max: int, sigma: float = 1e-3, eta: float = 1e-4,
                   eps: float = 1e-5, drop: float = 2.0 / 3.0, boost: float = 1.5, mode: int = DN_FULL,
                   combine: bool = True, max_trials: int = 30, cg_min: int = 0, r_percent: float = 0.0,
                   reuse_forward: bool = False) -> dict:
    """One outer Newton iteration (Section 4.5): theta and d_prev are updated in place; returns the
    statistics of the step and the next lambda under key "lam".  reuse_forward: theta, X and Y are exactly as
    the previous dn_newton_step on this context left them (the gradient then skips its forward pass)."""
    if not (S.is_cuda and S.dtype == torch.int32 and S.is_contiguous()):
        raise TypeError("S: need a contiguous int32 device tensor")
    l = X.shape[0]
    prm = NewtonParams(float(lam), float(sigma), float(eta), float(eps), float(drop), float(boost), int(cg_max),
                       int(mode), int(bool(combine)), int(max_trials), int(cg_min), float(r_percent),
                       int(bool(reuse_forward)))
    st = NewtonStats()
    rc = ctx._lib.dn_newton_step(ctx._h, _dev_f32(theta, "theta", ctx.n), _dev_f32(X, "X", l * ctx.dims[0]),
                                 _dev_f32(Y, "Y", l * ctx.dims[-1]), l, S.data_ptr(), S.numel(),
                                 _dev_f32(d_prev, "d_prev", ctx.n), ctypes.byref(prm), ctypes.byref(st))
    ctx._check(rc, "dn_newton_step")
    ctx.s = S.numel()
    out = {name: getattr(st, name) for name, _ in NewtonStats._fields_}
    out["beta"] = (st.beta1, st.beta2)
    out["lam"] = prm.lam
    return out
