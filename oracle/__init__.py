"""CPU oracle of the integer-only encoder layer -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to `qasr_oracle.cpp` (plain C++, built with g++), plus the encoder as
"the op list applied in order".  Nothing in the product package may import this module;
only tests, the smoke check and the benchmark's cpu_baseline leg do.  It imports nothing
from the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qasr_oracle.cpp")
_LIB = os.path.join(_HERE, "libqasr_oracle.so")
_lib = None


SANITIZE_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]


def build(force: bool = True, out: str | None = None, sanitize: bool = False) -> str:
    """Compile the oracle with g++ (generic x86-64 code: the .so is also run on another box).
    `sanitize` builds an instrumented copy (-O1, AddressSanitizer and UndefinedBehaviorSanitizer,
    first report aborts) at `out`; the tests run the pins against it in a child process."""
    out = out or _LIB
    if force or not os.path.exists(out):
        opt = ["-O1"] + SANITIZE_FLAGS if sanitize else ["-O3"]
        cmd = ["g++", "-std=c++17", *opt, "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", _SRC, "-o", out]
        subprocess.check_call(cmd)
    return out


def lib():
    global _lib
    if _lib is None:
        # QASR_ORACLE_SO: load this build instead (the sanitizer tier of the tests sets it)
        path = os.environ.get("QASR_ORACLE_SO") or build(force=False)
        L = ctypes.CDLL(path)
        i32, i64, u32, p = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_void_p
        L.qasr_oracle_num_threads.restype = i32
        L.qasr_oracle_num_threads.argtypes = []
        L.qasr_oracle_out_len.restype = i64
        L.qasr_oracle_out_len.argtypes = [i64, i32, i32, i32, i32, i32]
        L.qasr_oracle_conv1d_acc.restype = None
        L.qasr_oracle_conv1d_acc.argtypes = [i32, i32, i32, i64, i32, i32, i32, i32, i32, i32, i64, p, p, p, p]
        L.qasr_oracle_conv1d_int8.restype = i64
        L.qasr_oracle_conv1d_int8.argtypes = [i32, i32, i32, i64, i32, i32, i32, i32, i32, i32, i64, i64, u32,
                                              p, p, p, p, p, p, p]
        L.qasr_oracle_conv1d_int8_multi.restype = i64
        L.qasr_oracle_conv1d_int8_multi.argtypes = [i32, i32, i32, i64, i32, i32, i32, i32, i32, i32, i64, i64, u32,
                                                    p, p, p, p, p, p, i32, p]
        L.qasr_oracle_requant.restype = None
        L.qasr_oracle_requant.argtypes = [p, i32, i32, i64, p, p, p, p, u32, p]
        L.qasr_oracle_requant_scalar.restype = i64
        L.qasr_oracle_requant_scalar.argtypes = [i64, i32, i32]
        L.qasr_oracle_quantize.restype = None
        L.qasr_oracle_quantize.argtypes = [p, i64, ctypes.c_float, p]
        L.qasr_oracle_dequantize.restype = None
        L.qasr_oracle_dequantize.argtypes = [p, i64, ctypes.c_float, p]
        L.qasr_oracle_iexp_constants.restype = i32
        L.qasr_oracle_iexp_constants.argtypes = [ctypes.c_double, i32, p]
        L.qasr_oracle_iexp.restype = i64
        L.qasr_oracle_iexp.argtypes = [i64, i32, i64, i64, i64]
        L.qasr_oracle_sigmoid_code.restype = i64
        L.qasr_oracle_sigmoid_code.argtypes = [i32, i32, i64, i64, i64]
        L.qasr_oracle_act.restype = None
        L.qasr_oracle_act.argtypes = [i32, p, i32, i32, i64, i64, i64, i32, i64, i64, i64, i32, i32, p]
        L.qasr_oracle_softmax.restype = None
        L.qasr_oracle_softmax.argtypes = [p, i64, i64, i32, i64, i64, i64, p]
        L.qasr_oracle_minmax.restype = None
        L.qasr_oracle_minmax.argtypes = [p, i64, p]
        L.qasr_oracle_dyadic.restype = i32
        L.qasr_oracle_dyadic.argtypes = [ctypes.c_double, p, p]
        L.qasr_oracle_fold_quantize.restype = i32
        L.qasr_oracle_fold_quantize.argtypes = [p, p, p, p, p, p, ctypes.c_float, i32, i64, ctypes.c_float,
                                                ctypes.c_float, p, p, p, p, p]
        _lib = L
    return _lib


def _ptr(a, dtype):
    if a is None:
        return None
    assert a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(lib().qasr_oracle_num_threads())


def out_len(Tin, k, stride=1, dilation=1, pad_left=0, pad_right=0) -> int:
    return int(lib().qasr_oracle_out_len(Tin, k, stride, dilation, pad_left, pad_right))


def conv1d_acc(x, w, bias=None, *, stride=1, dilation=1, pad_left=0, pad_right=0, groups=1,
               Cin=None, x_batch_stride=0) -> np.ndarray:
    """int64 accumulators [B,Cout,Tout] (bias included if given)."""
    B = x.shape[0]
    Cin = x.shape[1] if Cin is None else Cin
    Tin = x.shape[2]
    Cout, _, k = w.shape
    Tout = out_len(Tin, k, stride, dilation, pad_left, pad_right)
    acc = np.empty((B, Cout, Tout), dtype=np.int64)
    lib().qasr_oracle_conv1d_acc(B, Cin, Cout, Tin, k, stride, dilation, pad_left, pad_right, groups,
                                 x_batch_stride, _ptr(x, np.int8), _ptr(w, np.int8), _ptr(bias, np.int32),
                                 _ptr(acc, np.int64))
    return acc


def conv1d_int8(x, w, bias, m, s, residual=None, *, stride=1, dilation=1, pad_left=0, pad_right=0,
                groups=1, relu=False, Cin=None, x_batch_stride=0, y_batch_stride=0, y_fill=0,
                check_overflow=True) -> np.ndarray:
    """One integer layer on host arrays. x int8 [B,Cx,Tin] (Cx >= Cin when a channel-prefix
    view is read through x_batch_stride), w int8 [Cout,Cin/groups,k], returns int8 [B,Cout,Tout].

    With y_batch_stride (elements, >= Cout*Tout) the output, and the residual operand(s), which share
    its layout, are [B, y_batch_stride] arrays: item b's [Cout,Tout] block starts at b*y_batch_stride;
    the bytes between blocks are never read or written (the returned array holds `y_fill` there)."""
    B = x.shape[0]
    Cin = x.shape[1] if Cin is None else Cin
    Tin = x.shape[2]
    Cout, _, k = w.shape
    Tout = out_len(Tin, k, stride, dilation, pad_left, pad_right)
    if y_batch_stride:
        assert y_batch_stride >= Cout * Tout
        yshape = (B, y_batch_stride)
    else:
        yshape = (B, Cout, Tout)
    y = np.full(yshape, y_fill, dtype=np.int8)
    if isinstance(residual, (list, tuple)):          # several residual operands: summed, one clamp
        rs = [np.ascontiguousarray(r, dtype=np.int8) for r in residual]
        assert all(r.shape == y.shape for r in rs)
        arr = (ctypes.c_void_p * len(rs))(*[r.ctypes.data for r in rs])
        ovf = lib().qasr_oracle_conv1d_int8_multi(B, Cin, Cout, Tin, k, stride, dilation, pad_left, pad_right,
                                                  groups, x_batch_stride, y_batch_stride, 1 if relu else 0,
                                                  _ptr(x, np.int8), _ptr(w, np.int8), _ptr(bias, np.int32),
                                                  _ptr(m, np.int32), _ptr(s, np.int32), arr, len(rs),
                                                  _ptr(y, np.int8))
        if check_overflow and ovf:
            raise OverflowError(f"{ovf} accumulators left the int32 range")
        return y
    if residual is not None:
        assert residual.shape == y.shape
    ovf = lib().qasr_oracle_conv1d_int8(B, Cin, Cout, Tin, k, stride, dilation, pad_left, pad_right, groups,
                                        x_batch_stride, y_batch_stride, 1 if relu else 0,
                                        _ptr(x, np.int8), _ptr(w, np.int8), _ptr(bias, np.int32),
                                        _ptr(m, np.int32), _ptr(s, np.int32), _ptr(residual, np.int8),
                                        _ptr(y, np.int8))
    if check_overflow and ovf:
        raise OverflowError(f"{ovf} accumulators left the int32 range")
    return y


def requant(acc, bias, m, s, residual=None, relu=False) -> np.ndarray:
    B, C, T = acc.shape
    y = np.empty((B, C, T), dtype=np.int8)
    lib().qasr_oracle_requant(_ptr(acc, np.int32), B, C, T, _ptr(bias, np.int32), _ptr(m, np.int32),
                              _ptr(s, np.int32), _ptr(residual, np.int8), 1 if relu else 0, _ptr(y, np.int8))
    return y


def requant_scalar(A: int, m: int, s: int) -> int:
    return int(lib().qasr_oracle_requant_scalar(A, m, s))


def quantize(x, alpha: float) -> np.ndarray:
    """Eq. 1 with b = 8: float32 features -> int8 codes in [-127, 127] (same shape)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.shape, dtype=np.int8)
    lib().qasr_oracle_quantize(_ptr(x, np.float32), x.size, alpha, _ptr(q, np.int8))
    return q


def dequantize(q, S: float) -> np.ndarray:
    """DQ(q, S) = S q in float32 (same shape)."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    x = np.empty(q.shape, dtype=np.float32)
    lib().qasr_oracle_dequantize(_ptr(q, np.int8), q.size, S, _ptr(x, np.float32))
    return x


def minmax(x, start=(np.inf, -np.inf)) -> np.ndarray:
    """Running (min, max) of float32 values, NaNs skipped."""
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    mm = np.array(start, dtype=np.float32)
    lib().qasr_oracle_minmax(_ptr(x, np.float32), x.size, _ptr(mm, np.float32))
    return mm


def dyadic(M: float):
    """(m, s) with 2^30 <= m < 2^31 and m 2^-s nearest to M."""
    m, s = ctypes.c_int32(), ctypes.c_int32()
    if lib().qasr_oracle_dyadic(float(M), ctypes.byref(m), ctypes.byref(s)) != 0:
        raise ValueError("multiplier has no dyadic form in range")
    return m.value, s.value


def fold_quantize(w, b, gamma, beta, mu, var, eps, S_x, S_y):
    """BatchNorm folding + per-channel weight quantisation + bias / (m, s) derivation.
    w float32 [Cout, Cin/groups, k]; returns (q_w int8, bias int32, m, s, S_w float32, n_bad)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    Cout = w.shape[0]
    per = w.size // Cout
    f32 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.float32)
    b, gamma, beta, mu, var = f32(b), f32(gamma), f32(beta), f32(mu), f32(var)
    qw = np.empty(w.shape, dtype=np.int8)
    bq, m, s = (np.empty(Cout, dtype=np.int32) for _ in range(3))
    Sw = np.empty(Cout, dtype=np.float32)
    bad = lib().qasr_oracle_fold_quantize(_ptr(w, np.float32), _ptr(b, np.float32), _ptr(gamma, np.float32),
                                          _ptr(beta, np.float32), _ptr(mu, np.float32), _ptr(var, np.float32),
                                          eps, Cout, per, S_x, S_y, _ptr(qw, np.int8), _ptr(bq, np.int32),
                                          _ptr(m, np.int32), _ptr(s, np.int32), _ptr(Sw, np.float32))
    return qw, bq, m, s, Sw, int(bad)


ACT_SIGMOID, ACT_SWISH, ACT_GLU = 1, 2, 3


def iexp_constants(S: float, u: int) -> dict:
    """Integer constants of the exponential at scale S / 2^u (Sec. 2.2: polynomial activations)."""
    out = (ctypes.c_int64 * 3)()
    if lib().qasr_oracle_iexp_constants(float(S), int(u), out) != 0:
        raise ValueError("unusable scale")
    return {"u": int(u), "q_ln2": int(out[0]), "q_b": int(out[1]), "q_c": int(out[2])}


def iexp(r: int, c: dict) -> int:
    assert r <= 0
    return int(lib().qasr_oracle_iexp(int(r), c["u"], c["q_ln2"], c["q_b"], c["q_c"]))


def sigmoid_code(q: int, c: dict) -> int:
    return int(lib().qasr_oracle_sigmoid_code(int(q), c["u"], c["q_ln2"], c["q_b"], c["q_c"]))


def act(kind: int, x, c: dict, m: int, s: int) -> np.ndarray:
    """x int8 [B, C, T] ([B, 2C, T] for GLU) -> int8 [B, C, T]."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    B, Cx, T = x.shape
    C = Cx // 2 if kind == ACT_GLU else Cx
    y = np.empty((B, C, T), dtype=np.int8)
    lib().qasr_oracle_act(kind, _ptr(x, np.int8), B, C, T, Cx * T, C * T, c["u"], c["q_ln2"], c["q_b"],
                          c["q_c"], int(m), int(s), _ptr(y, np.int8))
    return y


def softmax(x, c: dict) -> np.ndarray:
    """x int32 [rows, L] -> int8 probabilities at scale 2^-7."""
    x = np.ascontiguousarray(x, dtype=np.int32)
    rows, L = x.shape
    y = np.empty((rows, L), dtype=np.int8)
    lib().qasr_oracle_softmax(_ptr(x, np.int32), rows, L, c["u"], c["q_ln2"], c["q_b"], c["q_c"],
                              _ptr(y, np.int8))
    return y


def run_op(op, p, x, residual=None) -> np.ndarray:
    """Apply one op of a network spec (fields: Cin, k, stride, ... as in the workload tables)."""
    return conv1d_int8(x, p["w"], p["bias"], p["m"], p["s"], residual, stride=op.stride,
                       dilation=op.dilation, pad_left=op.pad_left, pad_right=op.pad_right,
                       groups=op.groups, relu=bool(op.flags & 1), Cin=op.Cin,
                       x_batch_stride=op.x_batch_stride)


def apply_act(a: dict, y: np.ndarray) -> np.ndarray:
    """The activation of an op on its output, as the encoder applies it: in place; GLU leaves its
    C/2 channels in the first half of the tensor and the gate half as it was."""
    c = iexp_constants(a["S"], a["u"])
    r = act(a["kind"], y, c, a["m"], a["s"])
    if a["kind"] != ACT_GLU:
        return r
    out = y.copy()
    out[:, : y.shape[1] // 2] = r
    return out


def encoder_forward(net, params, x, keep=False):
    """The op list applied in order over activation slots; returns the last op's output
    (and every op's output when keep=True)."""
    slots = {0: x}
    outs = []
    for op, p in zip(net.ops, params):
        xin = slots[op.in_slot]
        res = slots[op.res_slot] if op.res_slot >= 0 else None
        if getattr(op, "more_res", None):
            res = [res] + [slots[r] for r in op.more_res]
        y = run_op(op, p, xin, res)
        if getattr(op, "act", 0):
            y = apply_act(p["act"], y)
        slots[op.out_slot] = y
        if keep:
            outs.append(y)
    return (y, outs) if keep else y
