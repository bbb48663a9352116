"""ctypes binding of include/fobq.h.  Argument marshalling only: torch supplies
device memory and the HIP stream; no arithmetic of the method happens here.
There is no CPU fallback: if libfobq.so is missing the import of the library
fails loudly."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

OK, EINVAL, ENOMEM, EHIP, ENOTPD, ESTATE = 0, -1, -2, -3, -4, -5
ORDER_NATURAL, ORDER_SENSI_DESC, ORDER_CUSTOM = 0, 1, 2
ORDER_ERR_DESC, ORDER_W_DESC, ORDER_SENSI_ASC, ORDER_ERR_ASC, ORDER_W_ASC = 3, 4, 5, 6, 7
ORDER_SENSI_DYNAMIC = 8
STAGES = ("xxt", "finalize", "cholesky", "inverse", "order", "permute", "eliminate", "columns", "emit", "slice")
HESSIAN_FP64, HESSIAN_INT8_SLICES = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    return os.path.join(_HERE, "libfobq.so")


class FobqOpts(ctypes.Structure):
    _fields_ = [("bits", ctypes.c_int32), ("group", ctypes.c_int32),
                ("damp", ctypes.c_double), ("damp_abs", ctypes.c_double),
                ("order", ctypes.c_int32), ("block", ctypes.c_int32),
                ("stop_after", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("perm_in", ctypes.c_void_p)]


class FobqOut(ctypes.Structure):
    _fields_ = [("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("zeros", ctypes.c_void_p),
                ("Q", ctypes.c_void_p), ("perm", ctypes.c_void_p), ("W_work", ctypes.c_void_p),
                ("Hinv_work", ctypes.c_void_p), ("loss", ctypes.c_void_p)]


class FobqLayer(ctypes.Structure):
    _fields_ = [("W", ctypes.c_void_p), ("d_row", ctypes.c_int64), ("d_col", ctypes.c_int64),
                ("H", ctypes.c_void_p), ("out", FobqOut)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libfobq.so (built by paper_2509_05576_amd/build.py).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: build it with `python -m paper_2509_05576_amd.build` "
                                "(there is no fallback implementation)")
    lib = ctypes.CDLL(path)
    vp, i64, i32, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_double
    lib.fobq_create.argtypes = [ctypes.POINTER(vp), i32, vp]
    lib.fobq_destroy.argtypes = [vp]
    lib.fobq_last_error.argtypes = [vp]
    lib.fobq_last_error.restype = ctypes.c_char_p
    lib.fobq_hessian_begin.argtypes = [vp, i64]
    lib.fobq_hessian_set_mode.argtypes = [vp, i32]
    lib.fobq_hessian_accumulate.argtypes = [vp, vp, i64, i64]
    lib.fobq_hessian_accumulate_conv.argtypes = [vp, vp, i64, i64, i64, i64, i32, i32, i32]
    lib.fobq_hessian_finalize.argtypes = [vp, vp]
    lib.fobq_quantize_layer.argtypes = [vp, vp, i64, i64, vp, ctypes.POINTER(FobqOpts), ctypes.POINTER(FobqOut)]
    lib.fobq_quantize_layer_enqueue.argtypes = lib.fobq_quantize_layer.argtypes
    lib.fobq_quantize_layers_batched.argtypes = [vp, i32, ctypes.POINTER(FobqLayer), ctypes.POINTER(FobqOpts)]
    lib.fobq_finish.argtypes = [vp]
    lib.fobq_spd_inverse.argtypes = [vp, vp, i64, vp]
    lib.fobq_sensitivity.argtypes = [vp, vp, i64, i64, vp, ctypes.POINTER(FobqOpts), vp, vp]
    lib.fobq_sensitivity_static.argtypes = lib.fobq_sensitivity.argtypes
    lib.fobq_debug_fail_after.argtypes = [vp, i32]
    lib.fobq_debug_offset_tables.argtypes = [i32, i32, i64, i64, ctypes.POINTER(i32), i64, ctypes.POINTER(i64)]
    lib.fobq_workspace_bytes.argtypes = [vp, ctypes.POINTER(i64)]
    lib.fobq_hessian_form.argtypes = [vp, ctypes.POINTER(i32)]
    lib.fobq_obq_rows.argtypes = [vp, vp, i64, i64, vp, ctypes.POINTER(FobqOpts), i64, i64, vp, vp, vp, vp]
    lib.fobq_probe_int8_matrix_rate.argtypes = [vp, i32, ctypes.POINTER(dbl)]
    lib.fobq_profile_enable.argtypes = [vp, i32]
    lib.fobq_profile_get.argtypes = [vp, i32, ctypes.POINTER(dbl), ctypes.POINTER(i64)]
    lib.fobq_profile_reset.argtypes = [vp]
    for name in ("fobq_create", "fobq_destroy", "fobq_hessian_begin", "fobq_hessian_set_mode", "fobq_hessian_accumulate",
                 "fobq_hessian_accumulate_conv", "fobq_hessian_finalize", "fobq_quantize_layer",
                 "fobq_quantize_layer_enqueue", "fobq_quantize_layers_batched", "fobq_finish", "fobq_spd_inverse", "fobq_sensitivity",
                 "fobq_sensitivity_static", "fobq_debug_fail_after", "fobq_debug_offset_tables", "fobq_workspace_bytes", "fobq_probe_int8_matrix_rate", "fobq_obq_rows", "fobq_hessian_form",
                 "fobq_profile_enable", "fobq_profile_get", "fobq_profile_reset"):
        getattr(lib, name).restype = i32
    _lib = lib
    return lib


class FobqError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"fobq status {code}: {msg}")
        self.code = code


def _ptr(t: Optional[torch.Tensor], dtype: torch.dtype, what: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{what}: need a contiguous device tensor of {dtype}, got {t.dtype} on {t.device}")
    return t.data_ptr()


# ---- functions with the names of the C entry points -------------------------------------------
def fobq_create(device: int = 0, stream: Optional[int] = None) -> int:
    lib = load_library()
    h = ctypes.c_void_p()
    if stream is None:
        stream = torch.cuda.current_stream(device).cuda_stream
    rc = lib.fobq_create(ctypes.byref(h), device, ctypes.c_void_p(stream))
    if rc != OK:
        raise FobqError(rc, "fobq_create failed")
    return h.value


def fobq_destroy(ctx: int) -> None:
    load_library().fobq_destroy(ctypes.c_void_p(ctx))


def fobq_last_error(ctx: int) -> str:
    return load_library().fobq_last_error(ctypes.c_void_p(ctx)).decode()


def _check(ctx: int, rc: int) -> None:
    if rc != OK:
        raise FobqError(rc, fobq_last_error(ctx))


def fobq_hessian_begin(ctx: int, d_col: int) -> None:
    _check(ctx, load_library().fobq_hessian_begin(ctypes.c_void_p(ctx), d_col))


def fobq_hessian_set_mode(ctx: int, mode: int) -> None:
    _check(ctx, load_library().fobq_hessian_set_mode(ctypes.c_void_p(ctx), mode))


def fobq_hessian_accumulate(ctx: int, X: torch.Tensor) -> None:
    """X: device fp32, d_col x n, unit column stride (row stride = X.stride(0))."""
    if not X.is_cuda or X.dtype != torch.float32 or X.dim() != 2 or (X.shape[1] > 1 and X.stride(1) != 1):
        raise TypeError("X must be a 2-D device fp32 tensor with unit column stride")
    _check(ctx, load_library().fobq_hessian_accumulate(ctypes.c_void_p(ctx), ctypes.c_void_p(X.data_ptr()),
                                                       X.shape[1], X.stride(0)))


def fobq_hessian_accumulate_conv(ctx: int, maps: torch.Tensor, k: int, stride: int = 1, pad: int = 0) -> None:
    """maps: device fp32, images x h x w x channels, contiguous (channels innermost)."""
    if not maps.is_cuda or maps.dtype != torch.float32 or maps.dim() != 4 or not maps.is_contiguous():
        raise TypeError("maps must be a contiguous 4-D device fp32 tensor (images, h, w, channels)")
    n, h, w, c = maps.shape
    _check(ctx, load_library().fobq_hessian_accumulate_conv(ctypes.c_void_p(ctx), ctypes.c_void_p(maps.data_ptr()),
                                                            n, h, w, c, k, stride, pad))


def fobq_hessian_finalize(ctx: int, H_out: Optional[torch.Tensor] = None) -> None:
    _check(ctx, load_library().fobq_hessian_finalize(ctypes.c_void_p(ctx),
                                                     ctypes.c_void_p(_ptr(H_out, torch.float64, "H_out"))))


def _opts(bits, group, damp, damp_abs, order, block, stop_after, perm_in) -> FobqOpts:
    return FobqOpts(bits, group, damp, damp_abs, order, block, stop_after, 0,
                    _ptr(perm_in, torch.int32, "perm_in"))


@dataclass
class LayerOutput:
    codes: torch.Tensor
    scales: torch.Tensor
    zeros: torch.Tensor
    Q: torch.Tensor
    perm: torch.Tensor
    loss: torch.Tensor
    W_work: Optional[torch.Tensor] = None
    Hinv_work: Optional[torch.Tensor] = None


def fobq_quantize_layer(ctx: int, W: torch.Tensor, H: Optional[torch.Tensor] = None, *, bits: int = 4,
                        group: int = 0, damp: float = 0.01, damp_abs: float = 0.0,
                        order: int = ORDER_SENSI_DESC, block: int = 0, stop_after: int = -1,
                        perm_in: Optional[torch.Tensor] = None, debug: bool = False,
                        out: Optional[LayerOutput] = None, wait: bool = True) -> LayerOutput:
    """Allocates the outputs (unless `out` is given) and calls fobq_quantize_layer, or, with
    wait=False, fobq_quantize_layer_enqueue: the outputs are then valid after fobq_finish(ctx), and
    W, H, perm_in must be kept alive until then."""
    if W.dim() != 2:
        raise TypeError("W must be 2-D")
    r, d = W.shape
    dev = W.device
    g = d // group if group > 0 and d % group == 0 else 1
    if out is None:
        out = LayerOutput(
            codes=torch.empty((r, d), dtype=torch.uint8, device=dev),
            scales=torch.empty((r, g), dtype=torch.float32, device=dev),
            zeros=torch.empty((r, g), dtype=torch.float32, device=dev),
            Q=torch.empty((r, d), dtype=torch.float32, device=dev),
            perm=torch.empty((d,), dtype=torch.int32, device=dev),
            loss=torch.empty((1,), dtype=torch.float64, device=dev),
            W_work=torch.empty((r, d), dtype=torch.float64, device=dev) if debug else None,
            Hinv_work=torch.empty((d, d), dtype=torch.float64, device=dev) if debug else None)
    co = FobqOut(_ptr(out.codes, torch.uint8, "codes"), _ptr(out.scales, torch.float32, "scales"),
                 _ptr(out.zeros, torch.float32, "zeros"), _ptr(out.Q, torch.float32, "Q"),
                 _ptr(out.perm, torch.int32, "perm"), _ptr(out.W_work, torch.float64, "W_work"),
                 _ptr(out.Hinv_work, torch.float64, "Hinv_work"), _ptr(out.loss, torch.float64, "loss"))
    op = _opts(bits, group, damp, damp_abs, order, block, stop_after, perm_in)
    lib = load_library()
    fn = lib.fobq_quantize_layer if wait else lib.fobq_quantize_layer_enqueue
    rc = fn(ctypes.c_void_p(ctx), ctypes.c_void_p(_ptr(W, torch.float32, "W")), r, d,
            ctypes.c_void_p(_ptr(H, torch.float64, "H")), ctypes.byref(op), ctypes.byref(co))
    _check(ctx, rc)
    return out


def _alloc_output(W: torch.Tensor, group: int) -> LayerOutput:
    r, d = W.shape
    g = d // group if group > 0 and d % group == 0 else 1
    dev = W.device
    return LayerOutput(codes=torch.empty((r, d), dtype=torch.uint8, device=dev),
                       scales=torch.empty((r, g), dtype=torch.float32, device=dev),
                       zeros=torch.empty((r, g), dtype=torch.float32, device=dev),
                       Q=torch.empty((r, d), dtype=torch.float32, device=dev),
                       perm=torch.empty((d,), dtype=torch.int32, device=dev),
                       loss=torch.empty((1,), dtype=torch.float64, device=dev))


def fobq_quantize_layers_batched(ctx: int, Ws, Hs, *, bits: int = 4, group: int = 0, damp: float = 0.01,
                                 damp_abs: float = 0.0, order: int = ORDER_SENSI_DESC, outs=None):
    """Ws, Hs: lists of device tensors (fp32 d_row x d_col, fp64 d_col x d_col).  Allocates the outputs unless
    `outs` (a list of LayerOutput) is given; returns the list of LayerOutput."""
    n = len(Ws)
    if outs is None:
        outs = [_alloc_output(W, group) for W in Ws]
    arr = (FobqLayer * max(n, 1))()
    for i, (W, H, out) in enumerate(zip(Ws, Hs, outs)):
        if W.dim() != 2:
            raise TypeError("W must be 2-D")
        co = FobqOut(_ptr(out.codes, torch.uint8, "codes"), _ptr(out.scales, torch.float32, "scales"),
                     _ptr(out.zeros, torch.float32, "zeros"), _ptr(out.Q, torch.float32, "Q"),
                     _ptr(out.perm, torch.int32, "perm"), None, None, _ptr(out.loss, torch.float64, "loss"))
        arr[i] = FobqLayer(_ptr(W, torch.float32, "W"), W.shape[0], W.shape[1], _ptr(H, torch.float64, "H"), co)
    op = _opts(bits, group, damp, damp_abs, order, 0, -1, None)
    _check(ctx, load_library().fobq_quantize_layers_batched(ctypes.c_void_p(ctx), n, arr, ctypes.byref(op)))
    return outs


def fobq_finish(ctx: int) -> None:
    _check(ctx, load_library().fobq_finish(ctypes.c_void_p(ctx)))


def fobq_spd_inverse(ctx: int, H: torch.Tensor) -> torch.Tensor:
    d = H.shape[0]
    Hinv = torch.empty((d, d), dtype=torch.float64, device=H.device)
    _check(ctx, load_library().fobq_spd_inverse(ctypes.c_void_p(ctx), ctypes.c_void_p(_ptr(H, torch.float64, "H")),
                                                d, ctypes.c_void_p(Hinv.data_ptr())))
    return Hinv


def _sensitivity(fn, ctx, W, Hinv, bits, group, order, perm_in, S, perm):
    r, d = W.shape
    if S is None:
        S = torch.empty((d,), dtype=torch.float64, device=W.device)
    if perm is None:
        perm = torch.empty((d,), dtype=torch.int32, device=W.device)
    op = _opts(bits, group, 0.0, 0.0, order, 0, -1, perm_in)
    rc = fn(ctypes.c_void_p(ctx), ctypes.c_void_p(_ptr(W, torch.float32, "W")), r, d,
            ctypes.c_void_p(_ptr(Hinv, torch.float64, "Hinv")), ctypes.byref(op),
            ctypes.c_void_p(_ptr(S, torch.float64, "S")), ctypes.c_void_p(_ptr(perm, torch.int32, "perm")))
    _check(ctx, rc)
    return S, perm


def fobq_sensitivity(ctx: int, W: torch.Tensor, Hinv: torch.Tensor, *, bits: int = 4, group: int = 0,
                     order: int = ORDER_SENSI_DESC, perm_in: Optional[torch.Tensor] = None,
                     S: Optional[torch.Tensor] = None, perm: Optional[torch.Tensor] = None):
    return _sensitivity(load_library().fobq_sensitivity, ctx, W, Hinv, bits, group, order, perm_in, S, perm)


def fobq_sensitivity_static(ctx: int, W: torch.Tensor, Hinv: torch.Tensor, *, bits: int = 4, group: int = 0,
                            order: int = ORDER_SENSI_DESC, perm_in: Optional[torch.Tensor] = None,
                            S: Optional[torch.Tensor] = None, perm: Optional[torch.Tensor] = None):
    """The entry point that allocates nothing; pass S and perm to keep torch from allocating either."""
    return _sensitivity(load_library().fobq_sensitivity_static, ctx, W, Hinv, bits, group, order, perm_in, S, perm)


def fobq_obq_rows(ctx: int, W: torch.Tensor, Hinv: torch.Tensor, *, bits: int = 4, group: int = 0,
                  rows: Optional[tuple] = None):
    """The per-row baseline (own inverse and own greedy order per row) on rows[0] .. rows[1] - 1 (default: all).
    Returns codes (uint8), Q (fp32), order (int32), lossrow (fp64); only the processed rows are written."""
    r, d = W.shape
    lo, hi = (0, r) if rows is None else rows
    codes = torch.zeros((r, d), dtype=torch.uint8, device=W.device)
    Q = torch.zeros((r, d), dtype=torch.float32, device=W.device)
    order = torch.zeros((r, d), dtype=torch.int32, device=W.device)
    lossrow = torch.zeros((r,), dtype=torch.float64, device=W.device)
    op = _opts(bits, group, 0.0, 0.0, ORDER_NATURAL, 0, -1, None)
    rc = load_library().fobq_obq_rows(ctypes.c_void_p(ctx), ctypes.c_void_p(_ptr(W, torch.float32, "W")), r, d,
                                      ctypes.c_void_p(_ptr(Hinv, torch.float64, "Hinv")), ctypes.byref(op), lo, hi,
                                      ctypes.c_void_p(_ptr(codes, torch.uint8, "codes")), ctypes.c_void_p(_ptr(Q, torch.float32, "Q")),
                                      ctypes.c_void_p(_ptr(order, torch.int32, "order")),
                                      ctypes.c_void_p(_ptr(lossrow, torch.float64, "lossrow")))
    _check(ctx, rc)
    return codes, Q, order, lossrow


FORM_FP64, FORM_INT8_SLICES, FORM_INT8_TAP_OFFSETS = 0, 1, 2


def fobq_hessian_form(ctx: int) -> int:
    """The arithmetic the running (or last finalized) accumulation took: FORM_FP64 / _INT8_SLICES / _INT8_TAP_OFFSETS."""
    f = ctypes.c_int32(0)
    _check(ctx, load_library().fobq_hessian_form(ctypes.c_void_p(ctx), ctypes.byref(f)))
    return f.value


def fobq_workspace_bytes(ctx: int) -> int:
    b = ctypes.c_int64(0)
    _check(ctx, load_library().fobq_workspace_bytes(ctypes.c_void_p(ctx), ctypes.byref(b)))
    return b.value


PROBE_EQUAL_BYTES, PROBE_RANDOM_BYTES, PROBE_RELU_DIGITS = 0, 1, 2


def fobq_probe_int8_matrix_rate(ctx: int, operand_kind: int) -> float:
    """1e12 int8 operations per second of the X X^T kernel's inner loop with its operands fixed in LDS."""
    r = ctypes.c_double(0.0)
    _check(ctx, load_library().fobq_probe_int8_matrix_rate(ctypes.c_void_p(ctx), operand_kind, ctypes.byref(r)))
    return r.value


def fobq_debug_fail_after(ctx: int, n: int) -> None:
    _check(ctx, load_library().fobq_debug_fail_after(ctypes.c_void_p(ctx), n))


def fobq_debug_offset_tables(k: int, pad: int, h: int, w: int):
    """fobq_debug_offset_tables: (jobs, pairs, terms) as lists of tuples, or None when the geometry does not fit
    the library's tables.  Host code only: no GPU, no context."""
    lib = load_library()
    cap = 3 + 6 * 128 + 4 * 81 + 2 * 384
    buf = (ctypes.c_int32 * cap)()
    used = ctypes.c_int64(0)
    rc = lib.fobq_debug_offset_tables(k, pad, h, w, buf, cap, ctypes.byref(used))
    if rc == ESTATE:
        return None
    if rc != OK:
        raise FobqError(rc, "fobq_debug_offset_tables: bad argument")
    v = list(buf[:used.value])
    nj, npair, nt = v[0], v[1], v[2]
    o = 3
    jobs = [tuple(v[o + 6 * i:o + 6 * i + 6]) for i in range(nj)]
    o += 6 * nj
    pairs = [tuple(v[o + 4 * i:o + 4 * i + 4]) for i in range(npair)]
    o += 4 * npair
    terms = [tuple(v[o + 2 * i:o + 2 * i + 2]) for i in range(nt)]
    return jobs, pairs, terms


def FOBQ_PROFILE_STAGE(stage: int) -> int:
    return 2 << stage


def fobq_profile_enable(ctx: int, on) -> None:
    """on: False / True (every stage), or a sum of FOBQ_PROFILE_STAGE(s)."""
    _check(ctx, load_library().fobq_profile_enable(ctypes.c_void_p(ctx), int(on)))


def fobq_profile_get(ctx: int, stage: int):
    ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
    _check(ctx, load_library().fobq_profile_get(ctypes.c_void_p(ctx), stage, ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value


def fobq_profile_reset(ctx: int) -> None:
    _check(ctx, load_library().fobq_profile_reset(ctypes.c_void_p(ctx)))


class Ctx:
    """Context manager around a fobq context bound to torch's current stream."""

    def __init__(self, device: int = 0, stream: Optional[int] = None):
        self.handle = fobq_create(device, stream)

    def close(self) -> None:
        if self.handle:
            fobq_destroy(self.handle)
            self.handle = 0

    def __enter__(self) -> "Ctx":
        return self

    def __exit__(self, *exc) -> None:
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_hessian_mode(self, mode: int) -> None:
        fobq_hessian_set_mode(self.handle, mode)

    def hessian(self, X: torch.Tensor, chunk: Optional[int] = None, H_out: Optional[torch.Tensor] = None) -> None:
        """begin / accumulate (optionally in column chunks) / finalize."""
        fobq_hessian_begin(self.handle, X.shape[0])
        n = X.shape[1]
        step = n if not chunk else chunk
        for lo in range(0, n, step):
            fobq_hessian_accumulate(self.handle, X[:, lo:lo + step])
        fobq_hessian_finalize(self.handle, H_out)

    def hessian_conv(self, maps: torch.Tensor, k: int, stride: int = 1, pad: int = 0,
                     images_per_call: Optional[int] = None, H_out: Optional[torch.Tensor] = None) -> None:
        """begin / accumulate_conv (optionally a few images per call) / finalize for a k x k convolution."""
        fobq_hessian_begin(self.handle, maps.shape[3] * k * k)
        n = maps.shape[0]
        step = n if not images_per_call else images_per_call
        for lo in range(0, n, step):
            fobq_hessian_accumulate_conv(self.handle, maps[lo:lo + step], k, stride, pad)
        fobq_hessian_finalize(self.handle, H_out)

    def quantize_layer(self, W: torch.Tensor, H: Optional[torch.Tensor] = None, **kw) -> LayerOutput:
        return fobq_quantize_layer(self.handle, W, H, **kw)

    def quantize_layers_batched(self, Ws, Hs, **kw):
        return fobq_quantize_layers_batched(self.handle, Ws, Hs, **kw)

    def finish(self) -> None:
        fobq_finish(self.handle)

    def workspace_bytes(self) -> int:
        return fobq_workspace_bytes(self.handle)

    def hessian_form(self) -> int:
        return fobq_hessian_form(self.handle)

    def obq_rows(self, W, Hinv, **kw):
        return fobq_obq_rows(self.handle, W, Hinv, **kw)

    def probe_int8_matrix_rate(self, operand_kind: int) -> float:
        return fobq_probe_int8_matrix_rate(self.handle, operand_kind)

    def stage_ms(self):
        return {name: fobq_profile_get(self.handle, i) for i, name in enumerate(STAGES)}
