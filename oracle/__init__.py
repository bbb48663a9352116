"""ctypes wrapper around the plain fp64 CPU oracle (oracle/fobq_oracle.c).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; the
tests, the smoke check and the benchmark's cpu_baseline leg do.  The wrapper
only marshals numpy arrays; every step of the method runs in the C file, which
cites the passage of the paper each routine follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fobq_oracle.c")
_LIB = os.path.join(_HERE, "libfobq_oracle.so")

OK, EINVAL, ENOMEM, ENOTPD = 0, -1, -2, -4


# FOBQ_ORACLE_SANITIZE=1 in the environment: the oracle is compiled with AddressSanitizer and
# UndefinedBehaviorSanitizer into a library of its own (the process must then run with the
# sanitizer runtime preloaded; tests/test_oracle_sanitizers.py does that in a subprocess).
_SANITIZE = os.environ.get("FOBQ_ORACLE_SANITIZE", "") == "1"
if _SANITIZE:
    _LIB = os.path.join(_HERE, "libfobq_oracle_san.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        flags = (["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"] if _SANITIZE
                 else ["-O2"])
        subprocess.check_call([
            "gcc", *flags, "-fopenmp", "-fPIC", "-shared", "-std=c99", "-ffp-contract=off",
            "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _get():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float32, a.dtype
    return a


def _chk(rc: int, what: str) -> None:
    if rc != OK:
        raise OracleError(rc, what)


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: status {code}")
        self.code = code


def num_threads() -> int:
    """Threads the oracle's OpenMP loops use."""
    return int(_get().oracle_num_threads())


def hessian(X: np.ndarray) -> np.ndarray:
    """H = (2/N) X X^T in fp64 from fp32 X (d_col x N)."""
    X = _f32(X)
    d, n = X.shape
    H = np.empty((d, d), dtype=np.float64)
    _chk(_get().oracle_hessian(_p(X), ctypes.c_int64(d), ctypes.c_int64(n), ctypes.c_int64(n), _p(H)),
         "oracle_hessian")
    return H


def damp(H: np.ndarray, damp: float, damp_abs: float = 0.0):
    """Returns (H + lambda I, lambda), lambda = damp * mean(diag H) + damp_abs."""
    Hd = np.array(H, dtype=np.float64, order="C", copy=True)
    lam = ctypes.c_double(0.0)
    _chk(_get().oracle_damp(_p(Hd), ctypes.c_int64(Hd.shape[0]), ctypes.c_double(damp),
                            ctypes.c_double(damp_abs), ctypes.byref(lam)), "oracle_damp")
    return Hd, lam.value


def spd_inverse(H: np.ndarray) -> np.ndarray:
    H = np.ascontiguousarray(H, dtype=np.float64)
    d = H.shape[0]
    Hinv = np.empty((d, d), dtype=np.float64)
    _chk(_get().oracle_spd_inverse(_p(H), ctypes.c_int64(d), _p(Hinv)), "oracle_spd_inverse")
    return Hinv


def grid(W: np.ndarray, bits: int, group: int = 0):
    W = _f32(W)
    r, d = W.shape
    g = d // group if group > 0 else 1
    scale = np.empty((r, g), dtype=np.float64)
    zero = np.empty((r, g), dtype=np.float64)
    _chk(_get().oracle_grid(_p(W), ctypes.c_int64(r), ctypes.c_int64(d), ctypes.c_int(bits),
                            ctypes.c_int64(group), _p(scale), _p(zero)), "oracle_grid")
    return scale, zero


def sensitivity(W: np.ndarray, Hinv_diag: np.ndarray, bits: int, group: int,
                scale: np.ndarray, zero: np.ndarray) -> np.ndarray:
    W = _f32(W)
    r, d = W.shape
    hd = np.ascontiguousarray(Hinv_diag, dtype=np.float64)
    S = np.empty(d, dtype=np.float64)
    _chk(_get().oracle_sensitivity(_p(W), ctypes.c_int64(r), ctypes.c_int64(d), _p(hd), ctypes.c_int(bits),
                                   ctypes.c_int64(group), _p(scale), _p(zero), _p(S)), "oracle_sensitivity")
    return S


def order(S: np.ndarray, ascending: bool = False) -> np.ndarray:
    S = np.ascontiguousarray(S, dtype=np.float64)
    perm = np.empty(S.shape[0], dtype=np.int32)
    _chk(_get().oracle_order_dir(_p(S), ctypes.c_int64(S.shape[0]), ctypes.c_int(int(ascending)), _p(perm)),
         "oracle_order_dir")
    return perm


KEY_SENSI, KEY_ERR, KEY_W = 0, 1, 2


def column_key(W: np.ndarray, Hinv_diag: np.ndarray, bits: int, group: int, scale: np.ndarray,
               zero: np.ndarray, kind: int) -> np.ndarray:
    """Sort key per column: KEY_SENSI = S_j, KEY_ERR = summed squared quantization error,
    KEY_W = summed squared weight."""
    W = _f32(W)
    r, d = W.shape
    hd = np.ascontiguousarray(Hinv_diag, dtype=np.float64)
    key = np.empty(d, dtype=np.float64)
    _chk(_get().oracle_column_key(_p(W), ctypes.c_int64(r), ctypes.c_int64(d), _p(hd), ctypes.c_int(bits),
                                  ctypes.c_int64(group), _p(scale), _p(zero), ctypes.c_int(kind), _p(key)),
         "oracle_column_key")
    return key


@dataclass
class LoopResult:
    codes: np.ndarray      # int64 d_row x d_col, original column order
    Q: np.ndarray          # fp64
    W_work: np.ndarray     # fp64 running weights (original column order)
    Hinv_work: np.ndarray  # fp64 running shared inverse (processed rows/cols = 0)
    loss: float


def column_loop(W: np.ndarray, Hinv: np.ndarray, perm: np.ndarray, bits: int, group: int,
                scale: np.ndarray, zero: np.ndarray, steps: Optional[int] = None) -> LoopResult:
    W = _f32(W)
    r, d = W.shape
    Hw = np.array(Hinv, dtype=np.float64, order="C", copy=True)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    steps = d if steps is None else steps
    codes = np.empty((r, d), dtype=np.int64)
    Q = np.empty((r, d), dtype=np.float64)
    Ww = np.empty((r, d), dtype=np.float64)
    loss = ctypes.c_double(0.0)
    _chk(_get().oracle_column_loop(_p(W), ctypes.c_int64(r), ctypes.c_int64(d), _p(Hw), _p(perm),
                                   ctypes.c_int(bits), ctypes.c_int64(group), _p(scale), _p(zero),
                                   ctypes.c_int64(steps), _p(codes), _p(Q), _p(Ww), ctypes.byref(loss)),
         "oracle_column_loop")
    return LoopResult(codes, Q, Ww, Hw, loss.value)


def column_loop_dynamic(W: np.ndarray, Hinv: np.ndarray, bits: int, group: int, scale: np.ndarray,
                        zero: np.ndarray, steps: Optional[int] = None):
    """Column loop with the order chosen step by step (largest current score first).
    Returns (LoopResult, perm)."""
    W = _f32(W)
    r, d = W.shape
    Hw = np.array(Hinv, dtype=np.float64, order="C", copy=True)
    perm = np.empty(d, dtype=np.int32)
    steps = d if steps is None else steps
    codes = np.empty((r, d), dtype=np.int64)
    Q = np.empty((r, d), dtype=np.float64)
    Ww = np.empty((r, d), dtype=np.float64)
    loss = ctypes.c_double(0.0)
    _chk(_get().oracle_column_loop_dynamic(_p(W), ctypes.c_int64(r), ctypes.c_int64(d), _p(Hw), _p(perm),
                                           ctypes.c_int(bits), ctypes.c_int64(group), _p(scale), _p(zero),
                                           ctypes.c_int64(steps), _p(codes), _p(Q), _p(Ww), ctypes.byref(loss)),
         "oracle_column_loop_dynamic")
    return LoopResult(codes, Q, Ww, Hw, loss.value), perm


@dataclass
class ObqResult:
    codes: np.ndarray      # int64 d_row x d_col (only rows[0]:rows[1] are meaningful)
    Q: np.ndarray
    order: np.ndarray      # int32 d_row x d_col: per row, the index processed at each step
    lossrow: np.ndarray    # fp64 d_row
    rows: tuple


def obq_rows(W: np.ndarray, Hinv: np.ndarray, bits: int, group: int, scale: np.ndarray, zero: np.ndarray,
             rows: Optional[tuple] = None) -> ObqResult:
    """The per-row baseline (own inverse Hessian and own order per row, smallest loss term first)."""
    W = _f32(W)
    r, d = W.shape
    lo, hi = (0, r) if rows is None else rows
    Hinv = np.ascontiguousarray(Hinv, dtype=np.float64)
    codes = np.zeros((r, d), dtype=np.int64)
    Q = np.zeros((r, d), dtype=np.float64)
    order_ = np.zeros((r, d), dtype=np.int32)
    lossrow = np.zeros(r, dtype=np.float64)
    _chk(_get().oracle_obq_rows(_p(W), ctypes.c_int64(r), ctypes.c_int64(d), _p(Hinv), ctypes.c_int(bits),
                                ctypes.c_int64(group), _p(scale), _p(zero), ctypes.c_int64(lo), ctypes.c_int64(hi),
                                _p(codes), _p(Q), _p(order_), _p(lossrow)), "oracle_obq_rows")
    return ObqResult(codes, Q, order_, lossrow, (lo, hi))


def loss_eval(W: np.ndarray, Q: np.ndarray, H: np.ndarray) -> float:
    """1/2 tr((W - Q) H (W - Q)^T)."""
    W = _f32(W)
    r, d = W.shape
    Q = np.ascontiguousarray(Q, dtype=np.float64)
    H = np.ascontiguousarray(H, dtype=np.float64)
    out = ctypes.c_double(0.0)
    _chk(_get().oracle_loss_eval(_p(W), _p(Q), _p(H), ctypes.c_int64(r), ctypes.c_int64(d), ctypes.byref(out)),
         "oracle_loss_eval")
    return out.value


def output_error(W: np.ndarray, Q: np.ndarray, X: np.ndarray) -> float:
    """(1/N) |(W - Q) X|_F^2 straight from X."""
    W = _f32(W)
    X = _f32(X)
    r, d = W.shape
    Q = np.ascontiguousarray(Q, dtype=np.float64)
    out = ctypes.c_double(0.0)
    _chk(_get().oracle_output_error(_p(W), _p(Q), _p(X), ctypes.c_int64(r), ctypes.c_int64(d),
                                    ctypes.c_int64(X.shape[1]), ctypes.c_int64(X.shape[1]), ctypes.byref(out)),
         "oracle_output_error")
    return out.value


ORDER_NATURAL, ORDER_SENSI_DESC, ORDER_CUSTOM = 0, 1, 2
ORDER_ERR_DESC, ORDER_W_DESC, ORDER_SENSI_ASC, ORDER_ERR_ASC, ORDER_W_ASC = 3, 4, 5, 6, 7
ORDER_SENSI_DYNAMIC = 8
_ORDER_KEYS = {ORDER_SENSI_DESC: (KEY_SENSI, False), ORDER_ERR_DESC: (KEY_ERR, False), ORDER_W_DESC: (KEY_W, False),
               ORDER_SENSI_ASC: (KEY_SENSI, True), ORDER_ERR_ASC: (KEY_ERR, True), ORDER_W_ASC: (KEY_W, True)}


@dataclass
class LayerResult:
    codes: np.ndarray
    scales: np.ndarray
    zeros: np.ndarray
    Q: np.ndarray
    perm: np.ndarray
    loss: float
    H: np.ndarray          # undamped (2/N) X X^T, or the H passed in
    H_damped: np.ndarray
    Hinv: np.ndarray       # initial inverse
    S: np.ndarray
    W_work: np.ndarray
    Hinv_work: np.ndarray
    lam: float


def quantize_layer(W: np.ndarray, X: Optional[np.ndarray] = None, H: Optional[np.ndarray] = None,
                   bits: int = 4, group: int = 0, damp_rel: float = 0.01, damp_abs: float = 0.0,
                   order_mode: int = ORDER_SENSI_DESC, perm: Optional[np.ndarray] = None,
                   steps: Optional[int] = None) -> LayerResult:
    """The whole path, each stage by the C routine that implements it."""
    W = _f32(W)
    if H is None:
        H = hessian(X)
    H = np.ascontiguousarray(H, dtype=np.float64)
    Hd, lam = damp(H, damp_rel, damp_abs)
    Hinv = spd_inverse(Hd)
    scale, zero = grid(W, bits, group)
    S = sensitivity(W, np.ascontiguousarray(np.diag(Hinv)), bits, group, scale, zero)
    if order_mode == ORDER_NATURAL:
        p = np.arange(W.shape[1], dtype=np.int32)
    elif order_mode == ORDER_SENSI_DESC:
        p = order(S)
    elif order_mode in _ORDER_KEYS:
        kind, asc = _ORDER_KEYS[order_mode]
        S = column_key(W, np.ascontiguousarray(np.diag(Hinv)), bits, group, scale, zero, kind)
        p = order(S, asc)
    elif order_mode == ORDER_SENSI_DYNAMIC:
        res, p = column_loop_dynamic(W, Hinv, bits, group, scale, zero, steps)
        return LayerResult(res.codes, scale, zero, res.Q, p, res.loss, H, Hd, Hinv, S,
                           res.W_work, res.Hinv_work, lam)
    else:
        p = np.ascontiguousarray(perm, dtype=np.int32)
    res = column_loop(W, Hinv, p, bits, group, scale, zero, steps)
    return LayerResult(res.codes, scale, zero, res.Q, p, res.loss, H, Hd, Hinv, S,
                       res.W_work, res.Hinv_work, lam)
