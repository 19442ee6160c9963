"""Python binding of libaser.so: the MI355X implementation of ASER's per-layer calibration path.

Argument marshalling only.  Every function has the name and the meaning of the C entry point
declared in include/aser.h; tensors are torch tensors on the GPU (torch provides device memory
and the stream, nothing else) or raw integer device addresses.  There is no CPU fallback: if
the HIP library has not been built, importing the entry points raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libaser.so")

ASER_OK = 0
ASER_ERR_INVALID_ARG = 1
ASER_ERR_SHAPE = 2
ASER_ERR_DTYPE = 3
ASER_ERR_NOT_SPD = 4
ASER_ERR_NO_CONVERGE = 5
ASER_ERR_WORKSPACE = 6
ASER_ERR_HIP = 7

ASER_DTYPE_BF16 = 0
ASER_DTYPE_F32 = 1
ASER_PRECISION_AUTO = 0
ASER_PRECISION_FAST = 1
ASER_PRECISION_EXACT = 2
ASER_CODES_INT8 = 0
ASER_CODES_INT4_PACKED = 1

EXPORTS = (
    "aser_status_string", "aser_create", "aser_destroy", "aser_last_error", "aser_set_workspace", "aser_set_precision",
    "aser_workspace_bytes", "aser_gram_accumulate", "aser_smooth_outliers", "aser_smooth_outliers_noalloc",
    "aser_quantize_rtn",
    "aser_whiten", "aser_error_reconstruct", "aser_svd_plan", "aser_quantize_act_rtn",
    "aser_spectrum_workspace_bytes", "aser_singular_values", "aser_select_rank", "aser_effective_rank",
    "aser_output_error_workspace_bytes", "aser_layer_output_error",
    "aser_forward_workspace_bytes", "aser_compensated_forward", "aser_mfma_rate_probe",
    "aser_error_reconstruct_enqueue", "aser_finish", "aser_calibrate_layers", "aser_pick_concurrent_streams",
    "aser_layer_workspace_bytes", "aser_smoothed_weight", "aser_quant_target",
)


class aser_svd_opts(ctypes.Structure):
    _fields_ = [("block", ctypes.c_int32), ("max_iter", ctypes.c_int32), ("seed", ctypes.c_uint32)]


class aser_layer_desc(ctypes.Structure):
    """Mirror of the C struct of the same name (one layer of aser_calibrate_layers)."""
    _vp, _i64, _i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    _fields_ = [("X", _vp), ("x_dtype", _i32), ("clear_stats", _i32), ("rows", _i64), ("ldx", _i64),
                ("G", _vp), ("ldg", _i64), ("abs_sum", _vp), ("count", _vp),
                ("W", _vp), ("m", _i64), ("n", _i64), ("ldw", _i64), ("f", _i32), ("bits", _i32),
                ("idx", _vp), ("mdiag", _vp),
                ("layout", _i32), ("r", _i32), ("codes", _vp), ("scales", _vp), ("T", _vp), ("ldt", _i64),
                ("damp", ctypes.c_float), ("stats_from", _i32), ("S", _vp), ("lds", _i64),
                ("opts", ctypes.POINTER(aser_svd_opts)), ("L_A", _vp), ("L_B", _vp), ("sigma", _vp),
                ("err", ctypes.c_double), ("n_iter", _i32), ("status", _i32)]


class AserError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("aser status %d (%s): %s" % (status, status_string(status), message))
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads libaser.so built in-tree by paper_2411_07762_amd.build; raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libaser.so is not built: run `python -m paper_2411_07762_amd.build` "
                           "(there is no CPU fallback for the HIP path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float
    lib.aser_status_string.restype = ctypes.c_char_p
    lib.aser_status_string.argtypes = [ctypes.c_int]
    lib.aser_create.restype = ctypes.c_int
    lib.aser_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, vp]
    lib.aser_destroy.restype = ctypes.c_int
    lib.aser_destroy.argtypes = [vp]
    lib.aser_last_error.restype = ctypes.c_char_p
    lib.aser_last_error.argtypes = [vp]
    lib.aser_set_workspace.restype = ctypes.c_int
    lib.aser_set_workspace.argtypes = [vp, vp, ctypes.c_size_t]
    lib.aser_set_precision.restype = ctypes.c_int
    lib.aser_set_precision.argtypes = [vp, ctypes.c_int]
    lib.aser_workspace_bytes.restype = ctypes.c_size_t
    lib.aser_workspace_bytes.argtypes = [i64, i64, i32, ctypes.POINTER(aser_svd_opts)]
    lib.aser_gram_accumulate.restype = ctypes.c_int
    lib.aser_gram_accumulate.argtypes = [vp, vp, ctypes.c_int, i64, i64, i64, vp, i64, vp, vp]
    lib.aser_smooth_outliers.restype = ctypes.c_int
    lib.aser_smooth_outliers.argtypes = [vp, vp, i64, i64, i64, vp, vp, i32, vp, vp, vp, vp]
    lib.aser_smooth_outliers_noalloc.restype = ctypes.c_int
    lib.aser_smooth_outliers_noalloc.argtypes = lib.aser_smooth_outliers.argtypes
    lib.aser_quantize_rtn.restype = ctypes.c_int
    lib.aser_quantize_rtn.argtypes = [vp, vp, i64, i64, i64, vp, vp, i32, i32, i32, vp, vp, vp, i64]
    lib.aser_smoothed_weight.restype = ctypes.c_int
    lib.aser_smoothed_weight.argtypes = [vp, vp, i64, i64, i64, vp, i32, vp, i64]
    lib.aser_quant_target.restype = ctypes.c_int
    lib.aser_quant_target.argtypes = [vp, vp, i64, i64, i64, vp, vp, i64, vp, i64]
    lib.aser_whiten.restype = ctypes.c_int
    lib.aser_whiten.argtypes = [vp, vp, i64, i64, vp, f32, vp, i64, ctypes.POINTER(ctypes.c_int32)]
    lib.aser_error_reconstruct.restype = ctypes.c_int
    lib.aser_error_reconstruct.argtypes = [vp, vp, i64, i64, i64, vp, i64, i32, vp, i32, ctypes.POINTER(aser_svd_opts),
                                           vp, vp, vp, ctypes.POINTER(ctypes.c_double),
                                           ctypes.POINTER(ctypes.c_int32)]
    lib.aser_error_reconstruct_enqueue.restype = ctypes.c_int
    lib.aser_error_reconstruct_enqueue.argtypes = lib.aser_error_reconstruct.argtypes[:-2]
    lib.aser_finish.restype = ctypes.c_int
    lib.aser_finish.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)]
    lib.aser_calibrate_layers.restype = ctypes.c_int
    lib.aser_calibrate_layers.argtypes = [ctypes.POINTER(vp), i32, ctypes.POINTER(aser_layer_desc), i32]
    lib.aser_layer_workspace_bytes.restype = ctypes.c_size_t
    lib.aser_layer_workspace_bytes.argtypes = [ctypes.POINTER(aser_layer_desc)]
    lib.aser_pick_concurrent_streams.restype = ctypes.c_int
    lib.aser_pick_concurrent_streams.argtypes = [i32, ctypes.POINTER(vp), i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.aser_svd_plan.restype = ctypes.c_int
    lib.aser_svd_plan.argtypes = [i64, i64, i32, ctypes.POINTER(aser_svd_opts), ctypes.POINTER(ctypes.c_int32),
                                  ctypes.POINTER(ctypes.c_int32)]
    lib.aser_spectrum_workspace_bytes.restype = ctypes.c_size_t
    lib.aser_spectrum_workspace_bytes.argtypes = [i64, i64, i32]
    lib.aser_singular_values.restype = ctypes.c_int
    lib.aser_singular_values.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp]
    lib.aser_select_rank.restype = ctypes.c_int
    lib.aser_select_rank.argtypes = [vp, vp, i64, ctypes.c_double, ctypes.POINTER(ctypes.c_int32),
                                     ctypes.POINTER(ctypes.c_double)]
    lib.aser_effective_rank.restype = ctypes.c_int
    lib.aser_effective_rank.argtypes = [vp, vp, i64, ctypes.c_double, ctypes.POINTER(ctypes.c_double)]
    lib.aser_output_error_workspace_bytes.restype = ctypes.c_size_t
    lib.aser_output_error_workspace_bytes.argtypes = [i64, i64, i64, i32]
    lib.aser_layer_output_error.restype = ctypes.c_int
    lib.aser_layer_output_error.argtypes = [vp, vp, i64, i64, i64, vp, ctypes.c_int, i64, i64, vp, vp, i32, vp, vp, vp, i32,
                                            i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.aser_forward_workspace_bytes.restype = ctypes.c_size_t
    lib.aser_forward_workspace_bytes.argtypes = [i64, i64, i64, i32]
    lib.aser_compensated_forward.restype = ctypes.c_int
    lib.aser_compensated_forward.argtypes = [vp, vp, vp, i64, i64, vp, i32, vp, i64, vp, vp, i32, i32, vp, i64]
    lib.aser_quantize_act_rtn.restype = ctypes.c_int
    lib.aser_quantize_act_rtn.argtypes = [vp, vp, ctypes.c_int, i64, i64, i64, vp, i32, vp, vp]
    lib.aser_mfma_rate_probe.restype = ctypes.c_int
    lib.aser_mfma_rate_probe.argtypes = [vp, i32, i32, i32, ctypes.POINTER(ctypes.c_double)]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().aser_status_string(int(status)).decode()


# ----------------------------------------------------------------------------------- marshalling
def _ptr(t) -> Optional[int]:
    """Device address of a tensor (or a raw int address, or None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _ld(t, cols: int) -> int:
    if isinstance(t, int) or t is None:
        return cols
    if t.dim() == 1:
        return cols
    if t.stride(-1) != 1:
        raise ValueError("matrices must be row-major with unit column stride")
    return t.stride(0)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return ASER_DTYPE_BF16
    if t.dtype == torch.float32:
        return ASER_DTYPE_F32
    raise TypeError("activations must be bfloat16 or float32")


class Context:
    """Owns an aser_ctx bound to a device and a HIP stream (torch's current stream by default)."""

    def __init__(self, device: int = 0, stream: Optional[int] = None):
        self._lib = load_library()
        if stream is None:
            import torch
            stream = torch.cuda.current_stream(device).cuda_stream
        h = ctypes.c_void_p()
        st = self._lib.aser_create(ctypes.byref(h), int(device), ctypes.c_void_p(stream))
        if st != ASER_OK:
            raise AserError(st, "aser_create failed")
        self.handle = h
        self.device = device
        self._ws = None
        self._ws_bytes = 0

    def close(self):
        if self.handle:
            self._lib.aser_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_precision(self, mode: int):
        self.check(self._lib.aser_set_precision(self.handle, int(mode)))

    def last_error(self) -> str:
        return self._lib.aser_last_error(self.handle).decode()

    def check(self, status: int):
        if status != ASER_OK:
            raise AserError(status, self.last_error())

    def ensure_workspace(self, nbytes: int):
        """Allocates (with torch) and binds a workspace of at least nbytes."""
        import torch
        nbytes = (int(nbytes) + 255) // 256 * 256
        if self._ws is None or self._ws_bytes < nbytes:
            new = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda:%d" % self.device)
            base = new.data_ptr()
            off = (-base) % 256
            # the old tensor stays alive until the library has read what it left pending in it
            st = self._lib.aser_set_workspace(self.handle, ctypes.c_void_p(base + off), nbytes)
            self._ws, self._ws_bytes = new, nbytes
            self.check(st)


def aser_workspace_bytes(m: int, n: int, r: int, opts: Optional[aser_svd_opts] = None) -> int:
    return int(load_library().aser_workspace_bytes(m, n, r, ctypes.byref(opts) if opts is not None else None))


def aser_set_workspace(ctx: Context, dev_ptr, nbytes: int) -> int:
    return ctx._lib.aser_set_workspace(ctx.handle, ctypes.c_void_p(_ptr(dev_ptr)), int(nbytes))


def aser_gram_accumulate(ctx: Context, X, G, abs_sum=None, count=None, *, rows=None, n=None, ldx=None, ldg=None,
                         x_dtype=None) -> int:
    rows = X.shape[0] if rows is None else rows
    n = X.shape[1] if n is None else n
    return ctx._lib.aser_gram_accumulate(
        ctx.handle, _ptr(X), _dtype_code(X) if x_dtype is None else x_dtype, rows, n,
        _ld(X, n) if ldx is None else ldx, _ptr(G), _ld(G, n) if ldg is None else ldg, _ptr(abs_sum), _ptr(count))


def aser_smooth_outliers(ctx: Context, W, abs_sum, count, f: int, idx, mdiag, W_o=None, score=None, *, m=None, n=None,
                         ldw=None) -> int:
    m = W.shape[0] if m is None else m
    n = W.shape[1] if n is None else n
    return ctx._lib.aser_smooth_outliers(ctx.handle, _ptr(W), m, n, _ld(W, n) if ldw is None else ldw, _ptr(abs_sum),
                                         _ptr(count), f, _ptr(idx), _ptr(mdiag), _ptr(W_o), _ptr(score))


def aser_smooth_outliers_noalloc(ctx: Context, W, abs_sum, count, f: int, idx, mdiag, W_o=None, score=None, *, m=None,
                                 n=None, ldw=None) -> int:
    m = W.shape[0] if m is None else m
    n = W.shape[1] if n is None else n
    return ctx._lib.aser_smooth_outliers_noalloc(ctx.handle, _ptr(W), m, n, _ld(W, n) if ldw is None else ldw,
                                                 _ptr(abs_sum), _ptr(count), f, _ptr(idx), _ptr(mdiag), _ptr(W_o),
                                                 _ptr(score))


def aser_quantize_rtn(ctx: Context, W, idx, mdiag, f: int, bits: int, layout: int, codes, scales, T=None, *, m=None,
                      n=None, ldw=None, ldt=None) -> int:
    m = W.shape[0] if m is None else m
    n = W.shape[1] if n is None else n
    return ctx._lib.aser_quantize_rtn(ctx.handle, _ptr(W), m, n, _ld(W, n) if ldw is None else ldw, _ptr(idx),
                                      _ptr(mdiag), f, bits, layout, _ptr(codes), _ptr(scales), _ptr(T),
                                      (_ld(T, n) if T is not None else n) if ldt is None else ldt)


def aser_smoothed_weight(ctx: Context, W, idx, f: int, Ws, *, m=None, n=None, ldw=None, ldws=None) -> int:
    m = W.shape[0] if m is None else m
    n = W.shape[1] if n is None else n
    return ctx._lib.aser_smoothed_weight(ctx.handle, _ptr(W), m, n, _ld(W, n) if ldw is None else ldw, _ptr(idx), f,
                                         _ptr(Ws), _ld(Ws, n) if ldws is None else ldws)


def aser_quant_target(ctx: Context, W, mdiag, Wq, T, *, m=None, n=None, ldw=None, ldq=None, ldt=None) -> int:
    m = W.shape[0] if m is None else m
    n = W.shape[1] if n is None else n
    return ctx._lib.aser_quant_target(ctx.handle, _ptr(W), m, n, _ld(W, n) if ldw is None else ldw, _ptr(mdiag),
                                      _ptr(Wq), _ld(Wq, n) if ldq is None else ldq, _ptr(T),
                                      _ld(T, n) if ldt is None else ldt)


def aser_whiten(ctx: Context, G, mdiag, damp: float, S, *, n=None, ldg=None, lds=None, want_info: bool = True):
    """Returns (status, info).  want_info=False passes info = NULL: no synchronisation, a non-positive
    pivot is reported by the next aser_error_reconstruct on this context (info is returned as None)."""
    n = G.shape[0] if n is None else n
    info = ctypes.c_int32(0)
    st = ctx._lib.aser_whiten(ctx.handle, _ptr(G), _ld(G, n) if ldg is None else ldg, n, _ptr(mdiag), float(damp),
                              _ptr(S), _ld(S, n) if lds is None else lds, ctypes.byref(info) if want_info else None)
    return st, (info.value if want_info else None)


def aser_error_reconstruct(ctx: Context, T, S, r: int, L_A, L_B, sigma, opts: Optional[aser_svd_opts] = None, *,
                           idx=None, f: int = 0, m=None, n=None, ldt=None, lds=None):
    """Returns (status, err, n_iter).  idx, f: the outlier set of aser_smooth_outliers (f = 0: none)."""
    m = T.shape[0] if m is None else m
    n = T.shape[1] if n is None else n
    err = ctypes.c_double(0.0)
    nit = ctypes.c_int32(0)
    st = ctx._lib.aser_error_reconstruct(ctx.handle, _ptr(T), m, n, _ld(T, n) if ldt is None else ldt, _ptr(S),
                                         _ld(S, n) if lds is None else lds, r, _ptr(idx) if f > 0 else None, f,
                                         ctypes.byref(opts) if opts is not None else None, _ptr(L_A), _ptr(L_B),
                                         _ptr(sigma), ctypes.byref(err), ctypes.byref(nit))
    return st, err.value, nit.value


def aser_error_reconstruct_enqueue(ctx: Context, T, S, r: int, L_A, L_B, sigma, opts: Optional[aser_svd_opts] = None, *,
                                   idx=None, f: int = 0, m=None, n=None, ldt=None, lds=None) -> int:
    """aser_error_reconstruct without its wait; aser_finish(ctx) returns the results."""
    m = T.shape[0] if m is None else m
    n = T.shape[1] if n is None else n
    return ctx._lib.aser_error_reconstruct_enqueue(ctx.handle, _ptr(T), m, n, _ld(T, n) if ldt is None else ldt, _ptr(S),
                                                   _ld(S, n) if lds is None else lds, r, _ptr(idx) if f > 0 else None, f,
                                                   ctypes.byref(opts) if opts is not None else None, _ptr(L_A),
                                                   _ptr(L_B), _ptr(sigma))


def aser_finish(ctx: Context):
    """Returns (status, err, n_iter) of the enqueued aser_error_reconstruct."""
    err = ctypes.c_double(0.0)
    nit = ctypes.c_int32(0)
    st = ctx._lib.aser_finish(ctx.handle, ctypes.byref(err), ctypes.byref(nit))
    return st, err.value, nit.value


def aser_svd_plan(m: int, n: int, r: int, opts: Optional[aser_svd_opts] = None):
    """Returns (status, block, iters): what aser_error_reconstruct will use for this shape."""
    b, it = ctypes.c_int32(0), ctypes.c_int32(0)
    st = load_library().aser_svd_plan(m, n, r, ctypes.byref(opts) if opts is not None else None, ctypes.byref(b),
                                      ctypes.byref(it))
    return st, b.value, it.value


def aser_quantize_act_rtn(ctx: Context, X, mdiag, bits: int, codes, scales, *, rows=None, n=None, ldx=None,
                          x_dtype=None) -> int:
    rows = X.shape[0] if rows is None else rows
    n = X.shape[1] if n is None else n
    return ctx._lib.aser_quantize_act_rtn(ctx.handle, _ptr(X), _dtype_code(X) if x_dtype is None else x_dtype, rows, n,
                                          _ld(X, n) if ldx is None else ldx, _ptr(mdiag), bits, _ptr(codes),
                                          _ptr(scales))


def aser_spectrum_workspace_bytes(m: int, n: int, with_s: bool) -> int:
    return int(load_library().aser_spectrum_workspace_bytes(m, n, 1 if with_s else 0))


def aser_singular_values(ctx: Context, T, S, sigma, *, m=None, n=None, ldt=None, lds=None) -> int:
    m = T.shape[0] if m is None else m
    n = T.shape[1] if n is None else n
    return ctx._lib.aser_singular_values(ctx.handle, _ptr(T), m, n, _ld(T, n) if ldt is None else ldt, _ptr(S),
                                         (_ld(S, n) if S is not None else n) if lds is None else lds, _ptr(sigma))


def aser_select_rank(ctx: Context, sigma, alpha: float, *, k=None):
    """Returns (status, r, (sum, share_at_r, share_at_r_plus_1))."""
    k = sigma.shape[0] if k is None else k
    r = ctypes.c_int32(0)
    st3 = (ctypes.c_double * 3)()
    st = ctx._lib.aser_select_rank(ctx.handle, _ptr(sigma), k, float(alpha), ctypes.byref(r), st3)
    return st, r.value, (st3[0], st3[1], st3[2])


def aser_effective_rank(ctx: Context, sigma, eps: float = 1e-12, *, k=None):
    """Returns (status, effective_rank)."""
    k = sigma.shape[0] if k is None else k
    out = ctypes.c_double(0.0)
    st = ctx._lib.aser_effective_rank(ctx.handle, _ptr(sigma), k, float(eps), ctypes.byref(out))
    return st, out.value


def aser_output_error_workspace_bytes(m: int, n: int, rows: int, r: int) -> int:
    return int(load_library().aser_output_error_workspace_bytes(m, n, rows, r))


def aser_layer_output_error(ctx: Context, W, X, mdiag, codes, layout: int, scales, L_A, L_B, r: int, act_bits: int, *,
                            m=None, n=None, ldw=None, rows=None, ldx=None, x_dtype=None):
    """Returns (status, err, ref_norm)."""
    m = W.shape[0] if m is None else m
    n = W.shape[1] if n is None else n
    rows = X.shape[0] if rows is None else rows
    err, ref = ctypes.c_double(0.0), ctypes.c_double(0.0)
    st = ctx._lib.aser_layer_output_error(ctx.handle, _ptr(W), m, n, _ld(W, n) if ldw is None else ldw, _ptr(X),
                                          _dtype_code(X) if x_dtype is None else x_dtype, rows,
                                          _ld(X, n) if ldx is None else ldx, _ptr(mdiag), _ptr(codes), layout,
                                          _ptr(scales), _ptr(L_A), _ptr(L_B), r, act_bits, ctypes.byref(err),
                                          ctypes.byref(ref))
    return st, err.value, ref.value


def aser_forward_workspace_bytes(rows: int, n: int, m: int, r: int) -> int:
    return int(load_library().aser_forward_workspace_bytes(rows, n, m, r))


def aser_compensated_forward(ctx: Context, x_codes, x_scales, w_codes, layout: int, w_scales, L_A, L_B, r: int,
                             lowrank_split: bool, Y, *, rows=None, n=None, m=None, ldy=None) -> int:
    rows = x_codes.shape[0] if rows is None else rows
    n = x_codes.shape[1] if n is None else n
    m = w_scales.shape[0] if m is None else m
    return ctx._lib.aser_compensated_forward(ctx.handle, _ptr(x_codes), _ptr(x_scales), rows, n, _ptr(w_codes), layout,
                                             _ptr(w_scales), m, _ptr(L_A), _ptr(L_B), r, 1 if lowrank_split else 0,
                                             _ptr(Y), _ld(Y, m) if ldy is None else ldy)


# ----------------------------------------------------------------------------------- one layer, end to end
def aser_mfma_rate_probe(ctx: Context, kind: int, workgroups_per_cu: int = 1, iters: int = 20000):
    """(status, 10^12 operations per second) of a pure MFMA loop: kind 0 bf16, kind 1 int8; kinds 2 and 3: the
    same with the operand traffic of a 256 x 256 tile around the instructions (measurement aid)."""
    out = ctypes.c_double(0.0)
    st = ctx._lib.aser_mfma_rate_probe(ctx.handle, int(kind), int(workgroups_per_cu), int(iters), ctypes.byref(out))
    return st, out.value


class LayerBuffers:
    """Device buffers of one layer's calibration state and outputs (allocated with torch)."""

    def __init__(self, m: int, n: int, r: int, f: int, bits: int, packed: bool, device: int = 0,
                 intermediates: bool = True):
        """intermediates=False: no G / abs_sum / count, T and S (aser_calibrate_layers then keeps them in the
        context's workspace while the layer is in flight)."""
        import torch
        dev = "cuda:%d" % device
        self.m, self.n, self.r, self.f, self.bits, self.packed = m, n, r, f, bits, packed
        if not intermediates:
            self._stats = self.G = self.abs_sum = self.count = self.T = self.S = None
            self._outputs(torch, dev)
            return
        # the three statistics share one allocation, so that clearing them is one launch
        g_bytes = (n * n * 4 + 255) // 256 * 256
        a_bytes = (n * 8 + 255) // 256 * 256
        self._stats = torch.zeros(g_bytes + a_bytes + 256, dtype=torch.uint8, device=dev)
        self.G = self._stats[:n * n * 4].view(torch.float32).view(n, n)
        self.abs_sum = self._stats[g_bytes:g_bytes + n * 8].view(torch.float64)
        self.count = self._stats[g_bytes + a_bytes:g_bytes + a_bytes + 8].view(torch.int64)
        self.T = torch.empty((m, n), dtype=torch.float32, device=dev)
        self.S = torch.empty((n, n), dtype=torch.float32, device=dev)
        self._outputs(torch, dev)

    def _outputs(self, torch, dev):
        m, n, r, f, packed = self.m, self.n, self.r, self.f, self.packed
        self.idx = torch.zeros(max(f, 1), dtype=torch.int32, device=dev)
        self.mdiag = torch.empty(n, dtype=torch.float32, device=dev)
        self.codes = torch.empty((m, n // 2 if packed else n), dtype=torch.uint8 if packed else torch.int8, device=dev)
        self.scales = torch.empty(m, dtype=torch.float32, device=dev)
        self.L_A = torch.empty((m, r), dtype=torch.float32, device=dev)
        self.L_B = torch.empty((r, n), dtype=torch.float32, device=dev)
        self.sigma = torch.empty(r, dtype=torch.float32, device=dev)
        self.err = float("nan")

    def reset_statistics(self):
        self._stats.zero_()


def calibrate_layer(ctx: Context, W, X, buf: LayerBuffers, opts: Optional[aser_svd_opts] = None, damp: float = 0.0,
                    accumulate: bool = True):
    """The loop body of Algorithm 1 for one layer: five ABI calls on buffers in `buf`.

    With accumulate=False the Gram statistics already in `buf` are used (layers sharing an input).
    """
    ctx.ensure_workspace(aser_workspace_bytes(buf.m, buf.n, buf.r, opts))
    layout = ASER_CODES_INT4_PACKED if buf.packed else ASER_CODES_INT8
    if accumulate:
        ctx.check(aser_gram_accumulate(ctx, X, buf.G, buf.abs_sum, buf.count))
    ctx.check(aser_smooth_outliers(ctx, W, buf.abs_sum, buf.count, buf.f, buf.idx, buf.mdiag))
    ctx.check(aser_quantize_rtn(ctx, W, buf.idx, buf.mdiag, buf.f, buf.bits, layout, buf.codes, buf.scales, buf.T))
    st, _ = aser_whiten(ctx, buf.G, buf.mdiag, damp, buf.S, want_info=False)   # pivot check at the layer's one sync
    ctx.check(st)
    st, err, _ = aser_error_reconstruct(ctx, buf.T, buf.S, buf.r, buf.L_A, buf.L_B, buf.sigma, opts,
                                        idx=buf.idx, f=buf.f)
    ctx.check(st)
    buf.err = err
    return buf


def layer_desc(W, buf: "LayerBuffers", X=None, clear_stats: bool = False, opts: Optional[aser_svd_opts] = None,
               damp: float = 0.0, stats_from: Optional[int] = None) -> aser_layer_desc:
    """The descriptor of one layer for aser_calibrate_layers from its weight, its buffers and (unless the
    statistics in `buf` are already finished) its activations.  The tensors must outlive the call."""
    d = aser_layer_desc()
    if X is not None:
        d.X, d.x_dtype, d.rows, d.ldx = _ptr(X), _dtype_code(X), X.shape[0], _ld(X, buf.n)
    d.clear_stats = 1 if clear_stats else 0
    d.stats_from = 0 if stats_from is None else stats_from + 1       # index of an earlier layer of the same call
    d.G, d.ldg, d.abs_sum, d.count = _ptr(buf.G), _ld(buf.G, buf.n) if buf.G is not None else 0, _ptr(buf.abs_sum), _ptr(buf.count)
    d.W, d.m, d.n, d.ldw, d.f, d.bits = _ptr(W), buf.m, buf.n, _ld(W, buf.n), buf.f, buf.bits
    d.idx, d.mdiag = _ptr(buf.idx), _ptr(buf.mdiag)
    d.layout = ASER_CODES_INT4_PACKED if buf.packed else ASER_CODES_INT8
    d.r, d.codes, d.scales = buf.r, _ptr(buf.codes), _ptr(buf.scales)
    d.T, d.ldt = _ptr(buf.T), _ld(buf.T, buf.n) if buf.T is not None else 0
    d.damp, d.S, d.lds = damp, _ptr(buf.S), _ld(buf.S, buf.n) if buf.S is not None else 0
    if opts is not None:
        d.opts = ctypes.pointer(opts)
    d.L_A, d.L_B, d.sigma = _ptr(buf.L_A), _ptr(buf.L_B), _ptr(buf.sigma)
    return d


def aser_layer_workspace_bytes(desc: aser_layer_desc) -> int:
    return int(load_library().aser_layer_workspace_bytes(ctypes.byref(desc)))


def aser_calibrate_layers(ctxs, descs) -> int:
    """Runs the layers `descs` (aser_layer_desc) with len(ctxs) of them in flight; per-layer status, err and
    n_iter are left in the descriptors.  Returns the first failing status, or ASER_OK."""
    lib = load_library()
    handles = (ctypes.c_void_p * len(ctxs))(*[c.handle for c in ctxs])
    arr = (aser_layer_desc * len(descs))(*descs)
    st = lib.aser_calibrate_layers(handles, len(ctxs), arr, len(descs))
    for d, a in zip(descs, arr):
        d.err, d.n_iter, d.status = a.err, a.n_iter, a.status
    return st


def aser_pick_concurrent_streams(stream_handles, want: int, device: int = 0):
    """Returns (status, indices): up to `want` of the candidate streams (raw hipStream_t handles) that run
    concurrently with one another."""
    n = len(stream_handles)
    cand = (ctypes.c_void_p * n)(*stream_handles)
    chosen = (ctypes.c_int32 * max(n, 1))()
    cnt = ctypes.c_int32(0)
    st = load_library().aser_pick_concurrent_streams(device, cand, n, want, chosen, ctypes.byref(cnt))
    return st, [chosen[i] for i in range(cnt.value)]
