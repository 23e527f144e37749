"""Thin ctypes binding of libprac (include/prac.h): argument marshalling only.

Every method mirrors the C entry point of the same name, takes torch tensors
that live on the context's device (PyTorch supplies device memory and the
stream, nothing else) and raises PracError on a non-zero status.  There is no
CPU fallback: if libprac.so is missing, import of the library fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libprac.so")

PRAC_F32, PRAC_BF16 = 0, 1
PRAC_REFRESH_PRINCIPAL, PRAC_REFRESH_RANDOM = 1, 2
C_ROWMAJOR, C_PACKED = 0, 1
TUNE_CTDY_SPLITS, TUNE_PROFILE_STRIDE, TUNE_WGRAD_ONE_LAUNCH, TUNE_WGRAD_TAIL = 1, 2, 3, 4
KERNEL_KINDS = {"compress": 1, "ct_dy": 2, "t_reduce": 3, "p_t": 4, "gram": 5, "fused_fwd": 6, "reconstruct": 7,
                "weight_grad": 8, "sum_p_t": 9}
STATUS = {0: "PRAC_OK", -1: "PRAC_EINVAL", -2: "PRAC_ENOMEM", -3: "PRAC_EHIP",
          -4: "PRAC_ENUMERIC", -5: "PRAC_EUNSUPPORTED", -6: "PRAC_ENOCTX", -7: "PRAC_ETOOBIG"}
STATIC_SCRATCH_BYTES = 48 << 20

EXPORTS = ["prac_create", "prac_destroy", "prac_set_stream", "prac_sync_status", "prac_strerror",
           "prac_last_hip_error", "prac_profile_select", "prac_profile_read", "prac_profile_read_each", "prac_set_tuning",
           "prac_compressed_bytes", "prac_unpack_compressed", "prac_philox_words", "prac_philox_normal", "prac_gram",
           "prac_basis_lp_bytes", "prac_pack_basis", "prac_fit_basis", "prac_compress",
           "prac_compress_fused_fwd", "prac_weight_grad", "prac_weight_grad_shared", "prac_reconstruct",
           "prac_workspace_bytes", "prac_reserve_workspace", "prac_debug_fit_slab_margin", "prac_weight_grad_static"]
OPS = {"gram": 1, "fit_basis": 2, "compress": 3, "fused_fwd": 4, "weight_grad": 5, "reconstruct": 6}


class PracError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS.get(status, status)}")


class FitOpts(C.Structure):
    _fields_ = [("iters", C.c_int), ("oversample", C.c_int), ("row_stride", C.c_int64),
                ("warm_start", C.c_int)]


class CallShape(C.Structure):
    """prac_call_shape of include/prac.h."""
    _fields_ = [("op", C.c_int), ("dt", C.c_int), ("odt", C.c_int), ("N", C.c_int64), ("d", C.c_int64),
                ("k", C.c_int), ("r", C.c_int), ("n_out", C.c_int), ("m", C.c_int64 * 4), ("c_layout", C.c_int),
                ("have_p_lp", C.c_int), ("generic", C.c_int), ("refresh", C.c_int), ("fit", FitOpts)]


def call_shape(op: str, N: int, d: int, k: int, r: int, m=(), dt: int = PRAC_BF16, odt: int = PRAC_BF16,
               c_layout: int = C_PACKED, have_p_lp: bool = True, generic: bool = False, refresh: int = 3,
               iters: int = 0, oversample: int = 0, row_stride: int = 0, warm_start: bool = False) -> CallShape:
    sh = CallShape()
    sh.op, sh.dt, sh.odt, sh.N, sh.d, sh.k, sh.r = OPS[op], dt, odt, N, d, k, r
    sh.n_out = len(m)
    for i, v in enumerate(m):
        sh.m[i] = v
    sh.c_layout, sh.have_p_lp, sh.generic, sh.refresh = c_layout, int(have_p_lp), int(generic), refresh
    sh.fit = FitOpts(iters, oversample, row_stride, 1 if warm_start else 0)
    return sh


_lib = None


def load_library() -> C.CDLL:
    """Load libprac.so (built by `python -m paper_2602_23111_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2602_23111_amd.build`")
    lib = C.CDLL(_LIB_PATH)
    vp, i64, i32, u64, u32, f32 = C.c_void_p, C.c_int64, C.c_int, C.c_uint64, C.c_uint32, C.c_float
    sig = {
        "prac_create": (i32, [C.POINTER(vp), i32, vp]),
        "prac_destroy": (i32, [vp]),
        "prac_set_stream": (i32, [vp, vp]),
        "prac_sync_status": (i32, [vp]),
        "prac_strerror": (C.c_char_p, [i32]),
        "prac_last_hip_error": (i32, [vp]),
        "prac_profile_select": (i32, [vp, i32]),
        "prac_profile_read": (i32, [vp, C.POINTER(C.c_double), C.POINTER(i64)]),
        "prac_profile_read_each": (i32, [vp, C.POINTER(C.c_float), i64, C.POINTER(i64)]),
        "prac_set_tuning": (i32, [vp, i32, i32]),
        "prac_compressed_bytes": (C.c_size_t, [i64, i32, i32, i32, i64]),
        "prac_unpack_compressed": (i32, [vp, vp, i64, i32, vp, i64]),
        "prac_philox_words": (i32, [vp, u64, u64, u32, vp, i64]),
        "prac_philox_normal": (i32, [vp, u64, u64, u32, vp, i64]),
        "prac_gram": (i32, [vp, vp, i32, i64, i64, i64, i64, vp, i64]),
        "prac_basis_lp_bytes": (C.c_size_t, [i64, i32]),
        "prac_pack_basis": (i32, [vp, vp, i64, i64, i32, vp]),
        "prac_fit_basis": (i32, [vp, vp, i32, i64, i64, i64, i32, i32, u64, u64, i32,
                                 C.POINTER(FitOpts), vp, i64, vp, C.POINTER(f32)]),
        "prac_compress": (i32, [vp, vp, i32, i64, i64, i64, vp, vp, i64, i32, vp, i64, i32]),
        "prac_compress_fused_fwd": (i32, [vp, vp, i32, i64, i64, i64, vp, i64, i64, i32, vp, vp, i64,
                                          i32, vp, i64, vp, i64, i32]),
        "prac_weight_grad": (i32, [vp, vp, vp, i32, i64, i64, i64, i32, i64, vp, vp, i64, i64, i32, i32,
                                   f32, vp, i32, i64, f32]),
        "prac_reconstruct": (i32, [vp, vp, i32, i64, i64, i32, vp, i64, i64, i32, i32, f32, vp, i64]),
        "prac_weight_grad_static": (i32, [vp, vp, vp, i32, i64, i64, i64, i32, i64, vp, vp, i64, i64, i32, i32,
                                          f32, vp, i32, i64, f32]),
        "prac_workspace_bytes": (C.c_size_t, [vp, C.POINTER(CallShape)]),
        "prac_reserve_workspace": (i32, [vp, C.c_size_t]),
        "prac_debug_fit_slab_margin": (i64, [C.POINTER(CallShape)]),
        "prac_weight_grad_shared": (i32, [vp, vp, i32, i64, i64, i32, i32, C.POINTER(vp), C.POINTER(i64),
                                          C.POINTER(i64), vp, vp, i64, i64, i32, i32, f32, C.POINTER(vp), i32,
                                          C.POINTER(i64), f32]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PRAC_F32
    if t.dtype == torch.bfloat16:
        return PRAC_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _mat(t: torch.Tensor):
    """(pointer, rows, cols, leading dimension) of a row-major 2-D tensor view."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("expected a row-major 2-D tensor (unit column stride)")
    return t.data_ptr(), t.shape[0], t.shape[1], (t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1]))


def _check(rc: int, where: str):
    if rc != 0:
        raise PracError(rc, where)


class Prac:
    """One libprac context bound to a device and to torch's current stream."""

    def __init__(self, device: int = 0, stream: torch.cuda.Stream | None = None):
        self.lib = load_library()
        self.device = device
        torch.cuda.set_device(device)
        st = stream if stream is not None else torch.cuda.current_stream(device)
        self._stream = st
        h = C.c_void_p()
        _check(self.lib.prac_create(C.byref(h), device, C.c_void_p(st.cuda_stream)), "prac_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self.lib.prac_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_stream(self, stream: torch.cuda.Stream):
        self._stream = stream
        _check(self.lib.prac_set_stream(self._h, C.c_void_p(stream.cuda_stream)), "prac_set_stream")

    def sync_status(self):
        _check(self.lib.prac_sync_status(self._h), "prac_sync_status")

    # ---- scratch sizing
    def workspace_bytes(self, shape: CallShape) -> int:
        return int(self.lib.prac_workspace_bytes(self._h, C.byref(shape)))

    def reserve_workspace(self, nbytes: int):
        _check(self.lib.prac_reserve_workspace(self._h, nbytes), "prac_reserve_workspace")

    # ---- per-kernel timing hook
    def profile_select(self, kind: int):
        _check(self.lib.prac_profile_select(self._h, kind), "prac_profile_select")

    def profile_read(self):
        """(total milliseconds, launches) of the selected kernel since the last read."""
        ms, n = C.c_double(0.0), C.c_int64(0)
        _check(self.lib.prac_profile_read(self._h, C.byref(ms), C.byref(n)), "prac_profile_read")
        return float(ms.value), int(n.value)

    def profile_read_each(self, cap: int = 1 << 16):
        """Per-launch milliseconds (a list, launch order) of the selected kernel since the last read."""
        buf, n = (C.c_float * cap)(), C.c_int64(0)
        _check(self.lib.prac_profile_read_each(self._h, buf, cap, C.byref(n)), "prac_profile_read_each")
        return [float(buf[i]) for i in range(min(cap, int(n.value)))]

    # ---- Gaussian draw
    def philox_words(self, seed: int, draw: int, stream: int, n: int) -> torch.Tensor:
        out = torch.empty(n, dtype=torch.int32, device=f"cuda:{self.device}")
        _check(self.lib.prac_philox_words(self._h, seed, draw, stream, out.data_ptr(), n), "prac_philox_words")
        return out

    def philox_normal(self, seed: int, draw: int, stream: int, n: int) -> torch.Tensor:
        out = torch.empty(n, dtype=torch.float32, device=f"cuda:{self.device}")
        _check(self.lib.prac_philox_normal(self._h, seed, draw, stream, out.data_ptr(), n), "prac_philox_normal")
        return out

    # ---- Gram
    def gram(self, X: torch.Tensor, row_stride: int = 1, out: torch.Tensor | None = None) -> torch.Tensor:
        px, N, d, ldx = _mat(X)
        G = out if out is not None else torch.empty((d, d), dtype=torch.float32, device=X.device)
        pg, _, _, ldg = _mat(G)
        _check(self.lib.prac_gram(self._h, px, _dt(X), N, d, ldx, row_stride, pg, ldg), "prac_gram")
        return G

    # ---- basis
    def basis_lp_bytes(self, d: int, c: int) -> int:
        return int(self.lib.prac_basis_lp_bytes(d, c))

    def pack_basis(self, P: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
        pp, d, c, ldp = _mat(P)
        lp = out if out is not None else torch.zeros(self.basis_lp_bytes(d, c), dtype=torch.uint8, device=P.device)
        _check(self.lib.prac_pack_basis(self._h, pp, d, ldp, c, lp.data_ptr()), "prac_pack_basis")
        return lp

    def fit_basis(self, X: torch.Tensor | None, k: int, r: int, seed: int, draw: int,
                  refresh: int = PRAC_REFRESH_PRINCIPAL | PRAC_REFRESH_RANDOM, P: torch.Tensor | None = None,
                  d: int | None = None, iters: int = 0, oversample: int = 0, row_stride: int = 0,
                  warm_start: bool = False, pack: bool = True, P_lp: torch.Tensor | None = None):
        """Returns (P, P_lp or None, scale).  P_lp: an existing packed-basis buffer to write into."""
        if X is not None:
            px, N, dx, ldx = _mat(X)
            xdt, dev = _dt(X), X.device
        else:
            px, N, dx, ldx, xdt, dev = None, 0, d, d, PRAC_F32, P.device
        if P is None:
            P = torch.zeros((dx, k + r), dtype=torch.float32, device=dev)
        pp, _, _, ldp = _mat(P)
        if P_lp is not None:
            lp, pack = P_lp, True
        else:
            lp = torch.zeros(self.basis_lp_bytes(dx, k + r), dtype=torch.uint8, device=dev) if pack else None
        opts = FitOpts(iters, oversample, row_stride, 1 if warm_start else 0)
        scale = C.c_float(0.0)
        _check(self.lib.prac_fit_basis(self._h, px, xdt, N, dx, ldx, k, r, seed, draw, refresh, C.byref(opts),
                                       pp, ldp, lp.data_ptr() if pack else None, C.byref(scale)), "prac_fit_basis")
        return P, lp, float(scale.value)

    # ---- compress
    def set_tuning(self, key: int, value: int):
        _check(self.lib.prac_set_tuning(self._h, key, value), "prac_set_tuning")

    def compressed_bytes(self, N: int, c: int, dtype: torch.dtype = torch.bfloat16, layout: int = C_PACKED,
                         ldc: int = 0) -> int:
        return int(self.lib.prac_compressed_bytes(N, c, PRAC_BF16 if dtype == torch.bfloat16 else PRAC_F32,
                                                  layout, ldc))

    def _c_out(self, N, c, X, out, layout):
        """(tensor, pointer, ldc) of the compressed activation in the requested layout."""
        if layout == C_PACKED:
            Cm = out if out is not None else torch.empty(self.compressed_bytes(N, c) // 2, dtype=torch.bfloat16,
                                                         device=X.device)
            return Cm, Cm.data_ptr(), 0
        Cm = out if out is not None else torch.empty((N, c), dtype=X.dtype, device=X.device)
        pc, _, _, ldc = _mat(Cm)
        return Cm, pc, ldc

    def compress(self, X: torch.Tensor, P: torch.Tensor, P_lp: torch.Tensor | None = None,
                 out: torch.Tensor | None = None, layout: int = C_ROWMAJOR) -> torch.Tensor:
        px, N, d, ldx = _mat(X)
        pp, _, c, ldp = _mat(P)
        Cm, pc, ldc = self._c_out(N, c, X, out, layout)
        _check(self.lib.prac_compress(self._h, px, _dt(X), N, d, ldx, pp, P_lp.data_ptr() if P_lp is not None else None,
                                      ldp, c, pc, ldc, layout), "prac_compress")
        return Cm

    def unpack_compressed(self, Cpk: torch.Tensor, N: int, c: int, out: torch.Tensor | None = None) -> torch.Tensor:
        Cm = out if out is not None else torch.empty((N, c), dtype=torch.bfloat16, device=Cpk.device)
        pc, _, _, ldc = _mat(Cm)
        _check(self.lib.prac_unpack_compressed(self._h, Cpk.data_ptr(), N, c, pc, ldc), "prac_unpack_compressed")
        return Cm

    def compress_fused_fwd(self, X: torch.Tensor, W: torch.Tensor, P: torch.Tensor, w_layout: int = 0,
                           P_lp: torch.Tensor | None = None, Y: torch.Tensor | None = None,
                           out: torch.Tensor | None = None, layout: int = C_ROWMAJOR):
        px, N, d, ldx = _mat(X)
        pw, w0, w1, ldw = _mat(W)
        m = w1 if w_layout == 0 else w0
        pp, _, c, ldp = _mat(P)
        Ym = Y if Y is not None else torch.empty((N, m), dtype=X.dtype, device=X.device)
        py, _, _, ldy = _mat(Ym)
        Cm, pc, ldc = self._c_out(N, c, X, out, layout)
        _check(self.lib.prac_compress_fused_fwd(self._h, px, _dt(X), N, d, ldx, pw, m, ldw, w_layout, pp,
                                                P_lp.data_ptr() if P_lp is not None else None, ldp, c, py, ldy,
                                                pc, ldc, layout), "prac_compress_fused_fwd")
        return Ym, Cm

    # ---- weight gradient
    def weight_grad(self, Cm: torch.Tensor, dY: torch.Tensor, P: torch.Tensor, k: int, r: int, scale: float,
                    P_lp: torch.Tensor | None = None, out: torch.Tensor | None = None,
                    out_dtype: torch.dtype = torch.float32, beta: float = 0.0,
                    layout: int = C_ROWMAJOR, static: bool = False) -> torch.Tensor:
        """Cm: N x (k+r) row-major, or the flat packed buffer when layout == C_PACKED.
        static=True calls prac_weight_grad_static (then `out` must be given: this binding allocates nothing
        on that path either)."""
        py, N, m, lddy = _mat(dY)
        pp, d, _, ldp = _mat(P)
        if layout == C_PACKED:
            pc, ldc, cdt = Cm.data_ptr(), 0, PRAC_BF16
        else:
            pc, _, _, ldc = _mat(Cm)
            cdt = _dt(Cm)
        if static and out is None:
            raise ValueError("weight_grad(static=True) needs `out`")
        dW = out if out is not None else torch.empty((d, m), dtype=out_dtype, device=dY.device)
        pw, _, _, lddw = _mat(dW)
        fn = self.lib.prac_weight_grad_static if static else self.lib.prac_weight_grad
        _check(fn(self._h, pc, py, cdt, N, m, ldc, layout, lddy, pp, P_lp.data_ptr() if P_lp is not None else None,
                  d, ldp, k, r, scale, pw, _dt(dW), lddw, beta),
               "prac_weight_grad_static" if static else "prac_weight_grad")
        return dW

    def weight_grad_shared(self, Cm: torch.Tensor, dYs, P: torch.Tensor, k: int, r: int, scale: float,
                           P_lp: torch.Tensor | None = None, outs=None, out_dtype: torch.dtype = torch.float32,
                           beta: float = 0.0, layout: int = C_ROWMAJOR, N: int | None = None):
        """Weight gradients of several layers that share one compressed activation: list of dW_h."""
        n = len(dYs)
        pp, d, _, ldp = _mat(P)
        if layout == C_PACKED:
            pc, ldc, cdt = Cm.data_ptr(), 0, PRAC_BF16
        else:
            pc, _, _, ldc = _mat(Cm)
            cdt = _dt(Cm)
        ys = [_mat(y) for y in dYs]
        Nn = ys[0][1]
        if outs is None:
            outs = [torch.empty((d, y[2]), dtype=out_dtype, device=dYs[0].device) for y in ys]
        ws = [_mat(w) for w in outs]
        arr_p = (C.c_void_p * n)
        arr_i = (C.c_int64 * n)
        _check(self.lib.prac_weight_grad_shared(
            self._h, pc, cdt, Nn, ldc, layout, n, arr_p(*[y[0] for y in ys]), arr_i(*[y[2] for y in ys]),
            arr_i(*[y[3] for y in ys]), pp, P_lp.data_ptr() if P_lp is not None else None, d, ldp, k, r, scale,
            arr_p(*[w[0] for w in ws]), _dt(outs[0]), arr_i(*[w[3] for w in ws]), beta), "prac_weight_grad_shared")
        return outs

    # ---- reconstruction
    def reconstruct(self, Cm: torch.Tensor, P: torch.Tensor, k: int, r: int, scale: float, N: int | None = None,
                    out: torch.Tensor | None = None, layout: int = C_ROWMAJOR) -> torch.Tensor:
        """Xh = C[:, :k] Q1^T + scale * C[:, k:] Q2^T.  Cm: N x (k+r) row-major, or the flat packed
        buffer (then N must be given) when layout == C_PACKED."""
        pp, d, _, ldp = _mat(P)
        if layout == C_PACKED:
            pc, ldc, cdt, dt = Cm.data_ptr(), 0, PRAC_BF16, torch.bfloat16
        else:
            pc, N, _, ldc = _mat(Cm)
            cdt, dt = _dt(Cm), Cm.dtype
        Xh = out if out is not None else torch.empty((N, d), dtype=dt, device=Cm.device)
        px, _, _, ldxh = _mat(Xh)
        _check(self.lib.prac_reconstruct(self._h, pc, cdt, N, ldc, layout, pp, d, ldp, k, r, scale, px, ldxh),
               "prac_reconstruct")
        return Xh
