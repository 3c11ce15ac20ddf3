"""ctypes binding of libqasr.so: same names as the C ABI, marshalling only.

Tensors are torch tensors on the GPU (PyTorch is used for device memory and streams only);
the binding passes `data_ptr()` and the current stream to the library.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqasr.so")

FLAG_RELU = 1
FLAG_W_PACKED = 2

_i32, _i64, _u32, _vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_void_p


class ConvDesc(ctypes.Structure):
    """Mirror of qasr_conv1d_desc."""
    _fields_ = [("B", _i32), ("Cin", _i32), ("Cout", _i32), ("Tin", _i32),
                ("k", _i32), ("stride", _i32), ("dilation", _i32),
                ("pad_left", _i32), ("pad_right", _i32), ("groups", _i32),
                ("x_batch_stride", _i64), ("y_batch_stride", _i64), ("flags", _u32)]


ACT_SIGMOID, ACT_SWISH, ACT_GLU = 1, 2, 3
MAX_RESIDUALS = 12


class IExp(ctypes.Structure):
    """Mirror of qasr_iexp."""
    _fields_ = [("u", _i32), ("reserved", _i32), ("q_ln2", _i64), ("q_b", _i64), ("q_c", _i64)]


class Act(ctypes.Structure):
    """Mirror of qasr_act."""
    _fields_ = [("kind", _i32), ("m", _i32), ("s", _i32), ("reserved", _i32), ("e", IExp)]


class _Op(ctypes.Structure):
    """Mirror of qasr_op."""
    _fields_ = [("d", ConvDesc), ("w", _vp), ("bias", _vp), ("m", _vp), ("s", _vp),
                ("in_slot", _i32), ("res_slot", _i32), ("out_slot", _i32), ("act", ctypes.POINTER(Act)),
                ("n_more_res", _i32), ("more_res_slots", _i32 * (MAX_RESIDUALS - 1))]


class QasrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = f" [{lib().qasr_last_hip_error().decode()}]" if status == -7 else ""
        super().__init__(f"{where}: {status_string(status)} ({status}){detail}")


_lib = None


def lib():
    """Loads the built library; raises if it is missing (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        # PyTorch ships its own HIP runtime; it has to be in the process before this library is
        # loaded so that both resolve to the same runtime instance (two instances cannot share
        # the device, streams or allocations).
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        dp = ctypes.POINTER(ConvDesc)
        L.qasr_conv1d_out_len.restype = _i32
        L.qasr_conv1d_out_len.argtypes = [dp]
        L.qasr_conv1d_int8.restype = _i32
        L.qasr_conv1d_int8.argtypes = [dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
        L.qasr_packed_weight_bytes.restype = ctypes.c_size_t
        L.qasr_packed_weight_bytes.argtypes = [dp]
        L.qasr_pack_weights.restype = _i32
        L.qasr_pack_weights.argtypes = [dp, _vp, _vp, _vp]
        L.qasr_requant.restype = _i32
        L.qasr_requant.argtypes = [_vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _u32, _vp, _vp]
        L.qasr_quantize.restype = _i32
        L.qasr_quantize.argtypes = [_vp, ctypes.c_size_t, ctypes.c_float, _vp, _vp]
        L.qasr_dequantize.restype = _i32
        L.qasr_dequantize.argtypes = [_vp, ctypes.c_size_t, ctypes.c_float, _vp, _vp]
        L.qasr_plan_slot_buffers.restype = _i32
        L.qasr_plan_slot_buffers.argtypes = [_vp, _vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, ctypes.POINTER(_i32)]
        L.qasr_probe_copy.restype = _i32
        L.qasr_probe_copy.argtypes = [_vp, _vp, ctypes.c_size_t, _vp]
        L.qasr_probe_mfma_i8_outputs.restype = _i32
        L.qasr_probe_mfma_i8_outputs.argtypes = []
        L.qasr_probe_mfma_i8.restype = _i32
        L.qasr_probe_mfma_i8.argtypes = [_i32, _vp, ctypes.POINTER(ctypes.c_double), _vp]
        L.qasr_encoder_create.restype = _i32
        L.qasr_encoder_create.argtypes = [ctypes.POINTER(_Op), _i32, _i32, ctypes.POINTER(_vp)]
        L.qasr_encoder_workspace_bytes.restype = ctypes.c_size_t
        L.qasr_encoder_workspace_bytes.argtypes = [_vp]
        L.qasr_encoder_forward.restype = _i32
        L.qasr_encoder_forward.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.qasr_encoder_forward_static.restype = _i32
        L.qasr_encoder_forward_static.argtypes = [_vp, _vp, _vp, _vp]
        L.qasr_static_workspace_bytes.restype = ctypes.c_size_t
        L.qasr_static_workspace_bytes.argtypes = []
        L.qasr_encoder_forward_layerwise.restype = _i32
        L.qasr_encoder_forward_layerwise.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.qasr_encoder_op_in_team.restype = _i32
        L.qasr_encoder_op_in_team.argtypes = [_vp, _i32]
        L.qasr_encoder_team_check.restype = _i32
        L.qasr_encoder_team_check.argtypes = [_vp, ctypes.POINTER(_i32)]
        L.qasr_encoder_forward_team_stamps.restype = _i32
        L.qasr_encoder_forward_team_stamps.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_size_t, _vp, ctypes.POINTER(ctypes.c_float)]
        L.qasr_encoder_forward_timed.restype = _i32
        L.qasr_encoder_forward_timed.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_size_t, _vp, ctypes.POINTER(ctypes.c_float)]
        L.qasr_encoder_graph_create.restype = _i32
        L.qasr_encoder_graph_create.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_size_t, ctypes.POINTER(_vp)]
        L.qasr_encoder_graph_launch.restype = _i32
        L.qasr_encoder_graph_launch.argtypes = [_vp, _vp]
        L.qasr_encoder_graph_destroy.restype = None
        L.qasr_encoder_graph_destroy.argtypes = [_vp]
        L.qasr_encoder_num_ops.restype = _i32
        L.qasr_encoder_num_ops.argtypes = [_vp]
        L.qasr_encoder_op_kernel.restype = ctypes.c_char_p
        L.qasr_encoder_op_kernel.argtypes = [_vp, _i32]
        L.qasr_encoder_op_act_fused.restype = _i32
        L.qasr_encoder_op_act_fused.argtypes = [_vp, _i32]
        L.qasr_encoder_destroy.restype = None
        L.qasr_encoder_destroy.argtypes = [_vp]
        L.qasr_conv1d_kernel_name.restype = ctypes.c_char_p
        L.qasr_conv1d_kernel_name.argtypes = [dp]
        L.qasr_conv1d_int8_multi.restype = _i32
        L.qasr_conv1d_int8_multi.argtypes = [dp, _vp, _vp, _vp, _vp, _vp, ctypes.POINTER(_vp), _i32, _vp, _vp]
        L.qasr_observe_minmax.restype = _i32
        L.qasr_observe_minmax.argtypes = [_vp, ctypes.c_size_t, _vp, _vp]
        L.qasr_dyadic_from_scale.restype = _i32
        L.qasr_dyadic_from_scale.argtypes = [ctypes.c_double, ctypes.POINTER(_i32), ctypes.POINTER(_i32)]
        L.qasr_fold_bn_quantize.restype = _i32
        L.qasr_fold_bn_quantize.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_float, _i32, _i64, ctypes.c_float,
                                            ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
        L.qasr_encoder_workspace_bytes_f32.restype = ctypes.c_size_t
        L.qasr_encoder_workspace_bytes_f32.argtypes = [_vp]
        L.qasr_encoder_forward_f32.restype = _i32
        L.qasr_encoder_forward_f32.argtypes = [_vp, _vp, ctypes.c_float, ctypes.c_float, _vp, _vp, ctypes.c_size_t, _vp]
        L.qasr_iexp_init.restype = _i32
        L.qasr_iexp_init.argtypes = [ctypes.c_double, _i32, ctypes.POINTER(IExp)]
        L.qasr_act_int8.restype = _i32
        L.qasr_act_int8.argtypes = [ctypes.POINTER(Act), _vp, _i32, _i32, _i32, _i64, _i64, _vp, _vp]
        L.qasr_softmax_int32.restype = _i32
        L.qasr_softmax_int32.argtypes = [ctypes.POINTER(IExp), _vp, _i64, _i32, _vp, _vp]
        L.qasr_last_hip_error.restype = ctypes.c_char_p
        L.qasr_last_hip_error.argtypes = []
        L.qasr_status_string.restype = ctypes.c_char_p
        L.qasr_status_string.argtypes = [_i32]
        L.qasr_tuning_reload.restype = None
        L.qasr_tuning_reload.argtypes = []
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().qasr_status_string(status).decode()


def _check(status: int, where: str):
    if status != 0:
        raise QasrError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_desc(B, Cin, Cout, Tin, k=1, stride=1, dilation=1, pad_left=0, pad_right=0, groups=1,
              x_batch_stride=0, y_batch_stride=0, flags=0) -> ConvDesc:
    return ConvDesc(B, Cin, Cout, Tin, k, stride, dilation, pad_left, pad_right, groups,
                    x_batch_stride, y_batch_stride, flags)


def static_workspace_bytes() -> int:
    return int(lib().qasr_static_workspace_bytes())


def tuning_reload() -> None:
    """qasr_tuning_reload: read the QASR_* tuning environment variables again."""
    lib().qasr_tuning_reload()


def conv1d_out_len(d: ConvDesc) -> int:
    return int(lib().qasr_conv1d_out_len(ctypes.byref(d)))


def conv1d_kernel_name(d: ConvDesc) -> Optional[str]:
    r = lib().qasr_conv1d_kernel_name(ctypes.byref(d))
    return r.decode() if r else None


def conv1d_int8(d: ConvDesc, x, w, bias, m, s, residual, y):
    """qasr_conv1d_int8 on torch CUDA tensors; y is written in place (asynchronously)."""
    _check(lib().qasr_conv1d_int8(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(m), _ptr(s),
                                  _ptr(residual), _ptr(y), _stream()), "qasr_conv1d_int8")
    return y


def conv1d_int8_multi(d: ConvDesc, x, w, bias, m, s, residuals, y):
    """qasr_conv1d_int8_multi: the layer with a list of residual operands (all added, one clamp)."""
    arr = (_vp * max(1, len(residuals)))(*[r.data_ptr() for r in residuals])
    _check(lib().qasr_conv1d_int8_multi(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(m), _ptr(s), arr,
                                        len(residuals), _ptr(y), _stream()), "qasr_conv1d_int8_multi")
    return y


def packed_weight_bytes(d: ConvDesc) -> int:
    return int(lib().qasr_packed_weight_bytes(ctypes.byref(d)))


def pack_weights(d: ConvDesc, w, w_packed):
    _check(lib().qasr_pack_weights(ctypes.byref(d), _ptr(w), _ptr(w_packed), _stream()), "qasr_pack_weights")
    return w_packed


def requant(acc, bias, m, s, residual, flags, y):
    B, C, T = acc.shape
    _check(lib().qasr_requant(_ptr(acc), B, C, T, _ptr(bias), _ptr(m), _ptr(s), _ptr(residual), flags,
                              _ptr(y), _stream()), "qasr_requant")
    return y


def quantize(x, alpha: float, q):
    """qasr_quantize: float32 tensor x -> int8 tensor q of the same number of elements."""
    _check(lib().qasr_quantize(_ptr(x), x.numel(), alpha, _ptr(q), _stream()), "qasr_quantize")
    return q


def dequantize(q, S: float, x):
    """qasr_dequantize: int8 tensor q -> float32 tensor x of the same number of elements."""
    _check(lib().qasr_dequantize(_ptr(q), q.numel(), S, _ptr(x), _stream()), "qasr_dequantize")
    return x


def plan_slot_buffers(in_slot, res_slot, out_slot, n_slots: int, depth: int):
    """qasr_plan_slot_buffers (host only): (in_buf, res_buf, out_buf, n_buffers) for bare slot wiring."""
    n = len(in_slot)
    A = _i32 * n
    ib, rb, ob, nb = A(), A(), A(), _i32(0)
    _check(lib().qasr_plan_slot_buffers(A(*in_slot), A(*res_slot), A(*out_slot), n, n_slots, depth, ib, rb, ob,
                                        ctypes.byref(nb)), "qasr_plan_slot_buffers")
    return list(ib), list(rb), list(ob), int(nb.value)


def probe_copy(src, dst):
    """qasr_probe_copy: streaming copy of the bytes of tensor src into dst (same size, a multiple of 16 bytes)."""
    n = src.numel() * src.element_size()
    assert n == dst.numel() * dst.element_size()
    _check(lib().qasr_probe_copy(_ptr(src), _ptr(dst), n, _stream()), "qasr_probe_copy")
    return dst


def probe_mfma_outputs() -> int:
    return int(lib().qasr_probe_mfma_i8_outputs())


def probe_mfma_i8(iters: int, out) -> float:
    """qasr_probe_mfma_i8: register-resident int8 matrix-core loop; returns the integer operations of the launch."""
    assert out.numel() >= probe_mfma_outputs() and out.element_size() == 4
    ops = ctypes.c_double(0.0)
    _check(lib().qasr_probe_mfma_i8(iters, _ptr(out), ctypes.byref(ops), _stream()), "qasr_probe_mfma_i8")
    return float(ops.value)


def observe_minmax(x, minmax):
    """qasr_observe_minmax: widen the running (min, max) in the 2-float tensor `minmax` by float32 tensor x."""
    _check(lib().qasr_observe_minmax(_ptr(x), x.numel(), _ptr(minmax), _stream()), "qasr_observe_minmax")
    return minmax


def dyadic_from_scale(M: float):
    """qasr_dyadic_from_scale: (m, s) with 2^30 <= m < 2^31 and m 2^-s nearest to M."""
    m, s = _i32(), _i32()
    _check(lib().qasr_dyadic_from_scale(M, ctypes.byref(m), ctypes.byref(s)), "qasr_dyadic_from_scale")
    return m.value, s.value


def fold_bn_quantize(w, conv_bias, gamma, beta, mean, var, eps, S_x, S_y, q_w, bias_q, m, s, S_w=None, bad_count=None):
    """qasr_fold_bn_quantize on torch CUDA tensors (w float32 [Cout, ...], outputs preallocated)."""
    Cout = w.shape[0]
    _check(lib().qasr_fold_bn_quantize(_ptr(w), _ptr(conv_bias), _ptr(gamma), _ptr(beta), _ptr(mean), _ptr(var), eps,
                                       Cout, w.numel() // Cout, S_x, S_y, _ptr(q_w), _ptr(bias_q), _ptr(m), _ptr(s),
                                       _ptr(S_w), _ptr(bad_count), _stream()), "qasr_fold_bn_quantize")


def iexp_init(S: float, u: int) -> IExp:
    """qasr_iexp_init: integer constants of the exponential at scale S / 2^u."""
    c = IExp()
    _check(lib().qasr_iexp_init(S, u, ctypes.byref(c)), "qasr_iexp_init")
    return c


def make_act(kind: int, e: IExp, m: int, s: int) -> Act:
    return Act(kind, m, s, 0, e)


def act_int8(a: Act, x, B: int, C: int, T: int, y, x_batch_stride: int = 0, y_batch_stride: int = 0):
    """qasr_act_int8: x int8 [B, C, T] ([B, 2C, T] for GLU) -> y int8 [B, C, T]; y may be x."""
    _check(lib().qasr_act_int8(ctypes.byref(a), _ptr(x), B, C, T, x_batch_stride, y_batch_stride, _ptr(y),
                               _stream()), "qasr_act_int8")
    return y


def softmax_int32(e: IExp, x, y):
    """qasr_softmax_int32: x int32 [rows, L] -> y int8 [rows, L] (probabilities at scale 2^-7)."""
    rows, L = x.shape
    _check(lib().qasr_softmax_int32(ctypes.byref(e), _ptr(x), rows, L, _ptr(y), _stream()), "qasr_softmax_int32")
    return y


class Encoder:
    """qasr_encoder_* handle.  `ops` is a sequence of (ConvDesc, w, bias, m, s, in_slot, res_slot,
    out_slot[, Act or None[, list of further residual slots]]) with torch CUDA tensors, which the
    handle keeps alive."""

    def __init__(self, ops: Sequence[tuple], n_slots: int):
        self._keep = [o[1:5] for o in ops]
        arr = (_Op * len(ops))()
        acts = []
        for i, o in enumerate(ops):
            d, w, bias, m, s, i_s, r_s, o_s = o[:8]
            a = o[8] if len(o) > 8 else None
            more = list(o[9]) if len(o) > 9 and o[9] else []
            if a is not None:
                acts.append(a)
            if len(more) > MAX_RESIDUALS - 1:
                raise ValueError("too many residual operands")
            arr[i] = _Op(d, w.data_ptr(), bias.data_ptr() if bias is not None else None, m.data_ptr(),
                         s.data_ptr(), i_s, r_s, o_s, ctypes.pointer(a) if a is not None else None,
                         len(more), (_i32 * (MAX_RESIDUALS - 1))(*more))
        h = _vp()
        _check(lib().qasr_encoder_create(arr, len(ops), n_slots, ctypes.byref(h)), "qasr_encoder_create")
        self._h = h
        self.n_ops = int(lib().qasr_encoder_num_ops(h))
        self.workspace_bytes = int(lib().qasr_encoder_workspace_bytes(h))

    def op_kernel(self, i: int) -> str:
        return lib().qasr_encoder_op_kernel(self._h, i).decode()

    def op_act_fused(self, i: int) -> bool:
        return lib().qasr_encoder_op_act_fused(self._h, i) == 1

    def forward(self, x, y, workspace):
        _check(lib().qasr_encoder_forward(self._h, _ptr(x), _ptr(y), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream()),
               "qasr_encoder_forward")
        return y

    def forward_layerwise(self, x, y, workspace):
        """qasr_encoder_forward_layerwise: every layer as a launch of its own."""
        _check(lib().qasr_encoder_forward_layerwise(self._h, _ptr(x), _ptr(y), _ptr(workspace),
                                                    workspace.numel() * workspace.element_size(), _stream()),
               "qasr_encoder_forward_layerwise")
        return y

    def op_in_team(self, i: int) -> bool:
        return lib().qasr_encoder_op_in_team(self._h, i) == 1

    def team_aborted(self) -> bool:
        """qasr_encoder_team_check (synchronise first): a bounded wait of a persistent kernel gave up."""
        a = _i32(0)
        _check(lib().qasr_encoder_team_check(self._h, ctypes.byref(a)), "qasr_encoder_team_check")
        return bool(a.value)

    def forward_team_stamps(self, x, y, workspace):
        """qasr_encoder_forward_team_stamps: per-op microseconds inside the persistent kernels (0 elsewhere)."""
        us = (ctypes.c_float * self.n_ops)()
        _check(lib().qasr_encoder_forward_team_stamps(self._h, _ptr(x), _ptr(y), _ptr(workspace),
                                                      workspace.numel() * workspace.element_size(), _stream(), us),
               "qasr_encoder_forward_team_stamps")
        return list(us)

    def forward_static(self, x, y):
        """qasr_encoder_forward_static: the slots live in the library's static device array."""
        _check(lib().qasr_encoder_forward_static(self._h, _ptr(x), _ptr(y), _stream()), "qasr_encoder_forward_static")
        return y

    @property
    def workspace_bytes_f32(self) -> int:
        return int(lib().qasr_encoder_workspace_bytes_f32(self._h))

    def forward_f32(self, x, alpha: float, S_out: float, y, workspace):
        """qasr_encoder_forward_f32: float32 features in, float32 outputs out."""
        _check(lib().qasr_encoder_forward_f32(self._h, _ptr(x), alpha, S_out, _ptr(y), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream()),
               "qasr_encoder_forward_f32")
        return y

    def forward_timed(self, x, y, workspace):
        ms = (ctypes.c_float * self.n_ops)()
        _check(lib().qasr_encoder_forward_timed(self._h, _ptr(x), _ptr(y), _ptr(workspace),
                                                workspace.numel() * workspace.element_size(), _stream(), ms),
               "qasr_encoder_forward_timed")
        return list(ms)

    def graph(self, x, y, workspace) -> "EncoderGraph":
        """qasr_encoder_graph_create for these buffers (which the returned handle keeps alive)."""
        return EncoderGraph(self, x, y, workspace)

    def close(self):
        if getattr(self, "_h", None):
            lib().qasr_encoder_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class EncoderGraph:
    """qasr_encoder_graph_* handle: one launch() replays the encoder's forward on (x, y, workspace)."""

    def __init__(self, enc: Encoder, x, y, workspace):
        self._keep = (enc, x, y, workspace)
        h = _vp()
        _check(lib().qasr_encoder_graph_create(enc._h, _ptr(x), _ptr(y), _ptr(workspace),
                                               workspace.numel() * workspace.element_size(), ctypes.byref(h)),
               "qasr_encoder_graph_create")
        self._h = h

    def launch(self):
        _check(lib().qasr_encoder_graph_launch(self._h, _stream()), "qasr_encoder_graph_launch")
        return self._keep[2]

    def close(self):
        if getattr(self, "_h", None):
            lib().qasr_encoder_graph_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
