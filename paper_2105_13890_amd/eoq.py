"""Thin ctypes binding over libeoq's C ABI (include/eoq.h): same names, argument
marshalling only.  PyTorch supplies device memory and the stream; every step of the
path runs in the library's kernels.  Fails loudly if the library is not built.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("EOQ_LIB_PATH") or os.path.join(_HERE, "libeoq.so")

OK, ERR_ARG, ERR_SHAPE, ERR_WORKSPACE, ERR_RANGE, ERR_HIP = range(6)
FLAG_ACC_OVERFLOW, FLAG_EXP_GAP, FLAG_NONFINITE, FLAG_SHIFT_RANGE = 1, 2, 4, 8
Q, CQ, SQ = 0, 1, 2
OP_CONV_FWD, OP_CONV_BWD_DATA, OP_CONV_BWD_WEIGHT = 0, 1, 2
RQ_FWD, RQ_SQ_ACC, RQ_SQ_GAMMA, RQ_SQ_MERGE = 0, 1, 2, 3

EXPORTS = [
    "eoq_create", "eoq_destroy", "eoq_strerror", "eoq_status", "eoq_spec_counters", "eoq_workspace_bytes", "eoq_fill_zero",
    "eoq_reduce_sum_i64",
    "eoq_quantize", "eoq_pre_bias", "eoq_conv_fwd", "eoq_conv_bwd_data", "eoq_conv_bwd_data_sq", "eoq_transpose_filters", "eoq_conv_bwd_weight", "eoq_conv_bwd_weight_static",
    "eoq_relu_bwd", "eoq_relu_bwd_recompute", "eoq_merge_absmax", "eoq_requant_epilogue", "eoq_update_int8", "eoq_grad_update", "eoq_update_scalars",
    "eoq_update_int8_sr", "eoq_grad_update_sr", "eoq_update_scalars_sr", "eoq_sr_next_step",
    "eoq_maxpool_fwd", "eoq_maxpool_bwd", "eoq_maxpool_bwd_sq", "eoq_gap_sum", "eoq_broadcast_hw", "eoq_head_workspace_bytes",
    "eoq_head_fwd_bwd", "eoq_head_update",
]


class BwdFuse(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("mask_bits", "e1", "sum_e1", "absmax_e1", "merge_other", "merge_exp_other",
                                          "merge_absmax", "w_transposed", "merge_mask_bits", "merge_absmax_masked", "spec_state")]


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "H", "W", "C", "K", "R", "S", "stride", "pad")]

    @property
    def P(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1


class Epilogue(C.Structure):
    _fields_ = [("gamma", C.c_void_p), ("b_post", C.c_void_p), ("skip", C.c_void_p), ("skip_is_wide", C.c_int32),
                ("relu", C.c_int32), ("b_next_pre", C.c_void_p), ("y", C.c_void_p), ("u_next", C.c_void_p),
                ("relu_mask_bits", C.c_void_p), ("t_wide", C.c_void_p), ("t_wide_is_16", C.c_int32)]


class RequantArgs(C.Structure):
    _fields_ = [("mode", C.c_int32), ("K", C.c_int32), ("n", C.c_size_t), ("acc", C.c_void_p), ("ep", C.c_void_p),
                ("src_a", C.c_void_p), ("src_b", C.c_void_p), ("exp_b", C.c_void_p), ("gamma", C.c_void_p),
                ("absmax", C.c_void_p), ("exp_in", C.c_void_p), ("exp_in_off", C.c_int32), ("out", C.c_void_p),
                ("exp_out", C.c_void_p), ("sum_out", C.c_void_p), ("max_code_out", C.c_void_p),
                ("mask_bits", C.c_void_p), ("absmax_out", C.c_void_p), ("out_b", C.c_void_p),
                ("exp_out_b", C.c_void_p), ("absmax_masked", C.c_void_p)]


class ScalarGrad(C.Structure):
    _fields_ = [("param", C.c_int32), ("n_terms", C.c_int32), ("sum_idx", C.c_int32 * 2),
                ("exp_idx", C.c_int32 * 2), ("exp_off", C.c_int32 * 2)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2105_13890_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    lib.eoq_strerror.restype = C.c_char_p
    lib.eoq_workspace_bytes.restype = C.c_size_t
    lib.eoq_head_workspace_bytes.restype = C.c_size_t
    vp, sz, i32 = C.c_void_p, C.c_size_t, C.c_int32
    lib.eoq_create.argtypes = [C.POINTER(vp), vp]
    lib.eoq_destroy.argtypes = [vp]
    lib.eoq_status.argtypes = [vp, C.POINTER(C.c_uint32)]
    lib.eoq_spec_counters.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.eoq_reduce_sum_i64.argtypes = [vp, vp, vp, sz, vp]
    lib.eoq_workspace_bytes.argtypes = [C.POINTER(ConvDesc), i32]
    lib.eoq_fill_zero.argtypes = [vp, vp, sz]
    lib.eoq_quantize.argtypes = [vp, vp, sz, i32, i32, vp, vp]
    lib.eoq_pre_bias.argtypes = [vp, vp, sz, vp, vp]
    lib.eoq_conv_fwd.argtypes = [vp, C.POINTER(ConvDesc), vp, vp, vp, C.POINTER(Epilogue), vp, sz]
    lib.eoq_conv_bwd_data.argtypes = [vp, C.POINTER(ConvDesc), vp, vp, vp, vp, vp, sz]
    lib.eoq_transpose_filters.argtypes = [vp, C.POINTER(ConvDesc), vp, vp]
    lib.eoq_conv_bwd_data_sq.argtypes = [vp, C.POINTER(ConvDesc), vp, vp, vp, vp, vp, i32, vp, vp, C.POINTER(BwdFuse), vp, sz]
    lib.eoq_conv_bwd_weight.argtypes = [vp, C.POINTER(ConvDesc), vp, vp, vp, vp, vp, sz]
    lib.eoq_conv_bwd_weight_static.argtypes = [vp, C.POINTER(ConvDesc), vp, vp, vp, vp]
    lib.eoq_relu_bwd.argtypes = [vp, vp, vp, vp, sz, vp, vp, vp, vp]
    lib.eoq_relu_bwd_recompute.argtypes = [vp, C.POINTER(ConvDesc), vp, vp, vp, vp, vp, vp, vp, vp]
    lib.eoq_merge_absmax.argtypes = [vp, vp, vp, vp, vp, sz, vp]
    lib.eoq_requant_epilogue.argtypes = [vp, C.POINTER(RequantArgs)]
    lib.eoq_update_int8.argtypes = [vp, vp, sz, vp, vp, vp, vp]
    lib.eoq_grad_update.argtypes = [vp, C.POINTER(ConvDesc), vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.eoq_update_scalars.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp]
    u32 = C.c_uint32
    lib.eoq_update_int8_sr.argtypes = [vp, vp, sz, vp, vp, vp, vp, vp, u32]
    lib.eoq_grad_update_sr.argtypes = [vp, C.POINTER(ConvDesc), vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, u32]
    lib.eoq_update_scalars_sr.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.eoq_sr_next_step.argtypes = [vp, vp]
    lib.eoq_maxpool_fwd.argtypes = [vp, vp] + [i32] * 8 + [vp, vp, vp, vp]
    lib.eoq_maxpool_bwd.argtypes = [vp, vp, vp] + [i32] * 8 + [vp, vp]
    lib.eoq_maxpool_bwd_sq.argtypes = [vp, vp, vp] + [i32] * 8 + [vp, vp, vp, vp, vp, vp, vp]
    lib.eoq_gap_sum.argtypes = [vp, vp, i32, i32, i32, vp]
    lib.eoq_broadcast_hw.argtypes = [vp, vp, i32, i32, i32, vp]
    lib.eoq_head_workspace_bytes.argtypes = [i32, i32, i32]
    lib.eoq_head_fwd_bwd.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz]
    lib.eoq_head_update.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, sz]
    return lib


_lib = _load()


class EoqError(RuntimeError):
    pass


def _check(rc: int, what: str):
    if rc != OK:
        raise EoqError(f"{what}: {_lib.eoq_strerror(rc).decode()} (code {rc})")


def _ptr(t):
    """Device pointer of a tensor (or None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    return t.data_ptr()


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


class Context:
    """eoq_create / eoq_destroy; methods mirror the C entry points one to one."""

    def __init__(self, stream: torch.cuda.Stream | None = None):
        self._h = C.c_void_p()
        s = stream.cuda_stream if stream is not None else torch.cuda.current_stream().cuda_stream
        _check(_lib.eoq_create(C.byref(self._h), s), "eoq_create")

    def close(self):
        if self._h:
            _lib.eoq_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def status(self) -> int:
        f = C.c_uint32(0)
        _lib.eoq_status(self._h, C.byref(f))
        return f.value

    def spec_counters(self) -> tuple[int, int]:
        h, m = C.c_int64(0), C.c_int64(0)
        _check(_lib.eoq_spec_counters(self._h, C.byref(h), C.byref(m)), "eoq_spec_counters")
        return h.value, m.value

    def reduce_sum_i64(self, e, t, sum_slot):
        _check(_lib.eoq_reduce_sum_i64(self._h, _ptr(e), _ptr(t), e.numel(), _ptr(sum_slot)), "eoq_reduce_sum_i64")

    @staticmethod
    def workspace_bytes(desc: ConvDesc, op: int) -> int:
        return _lib.eoq_workspace_bytes(C.byref(desc), op)

    def fill_zero(self, t):
        _check(_lib.eoq_fill_zero(self._h, _ptr(t), _nbytes(t)), "eoq_fill_zero")

    def quantize(self, x, mode, pre_shift, q, exp_slot=None):
        _check(_lib.eoq_quantize(self._h, _ptr(x), x.numel(), mode, pre_shift, _ptr(q), _ptr(exp_slot)), "eoq_quantize")

    def pre_bias(self, a, b_pre, u):
        _check(_lib.eoq_pre_bias(self._h, _ptr(a), a.numel(), _ptr(b_pre), _ptr(u)), "eoq_pre_bias")

    @staticmethod
    def epilogue(gamma=None, b_post=None, skip=None, relu=1, b_next_pre=None, y=None, u_next=None, mask=None,
                 t_wide=None) -> Epilogue:
        wide = 0
        if skip is not None and not isinstance(skip, int):
            wide = {torch.int32: 1, torch.int16: 2}.get(skip.dtype, 0)
        t16 = 1 if (t_wide is not None and not isinstance(t_wide, int) and t_wide.dtype == torch.int16) else 0
        return Epilogue(_ptr(gamma), _ptr(b_post), _ptr(skip), wide, relu, _ptr(b_next_pre), _ptr(y), _ptr(u_next),
                        _ptr(mask), _ptr(t_wide), t16)

    def conv_fwd(self, desc, u, w, acc=None, ep: Epilogue | None = None, ws=None):
        _check(_lib.eoq_conv_fwd(self._h, C.byref(desc), _ptr(u), _ptr(w), _ptr(acc),
                                 C.byref(ep) if ep is not None else None, _ptr(ws), _nbytes(ws)), "eoq_conv_fwd")

    def conv_bwd_data(self, desc, e, w, d_acc, absmax_slot, ws):
        _check(_lib.eoq_conv_bwd_data(self._h, C.byref(desc), _ptr(e), _ptr(w), _ptr(d_acc), _ptr(absmax_slot),
                                      _ptr(ws), _nbytes(ws)), "eoq_conv_bwd_data")

    def transpose_filters(self, desc, w, wt):
        _check(_lib.eoq_transpose_filters(self._h, C.byref(desc), _ptr(w), _ptr(wt)), "eoq_transpose_filters")

    def conv_bwd_data_sq(self, desc, e, w, e4, absmax_slot, exp_in, exp_in_off, exp_out, sum_out, ws,
                         mask=None, e1=None, sum_e1=None, absmax_e1=None, merge_other=None, merge_exp_other=None,
                         merge_absmax=None, w_transposed=None, merge_mask=None, merge_absmax_masked=None, spec_state=None):
        fuse = None
        if e1 is not None or merge_other is not None or w_transposed is not None or spec_state is not None:
            fuse = BwdFuse(_ptr(mask), _ptr(e1), _ptr(sum_e1), _ptr(absmax_e1), _ptr(merge_other),
                           _ptr(merge_exp_other), _ptr(merge_absmax), _ptr(w_transposed), _ptr(merge_mask),
                           _ptr(merge_absmax_masked), _ptr(spec_state))
        _check(_lib.eoq_conv_bwd_data_sq(self._h, C.byref(desc), _ptr(e), _ptr(w), _ptr(e4), _ptr(absmax_slot),
                                         _ptr(exp_in), exp_in_off, _ptr(exp_out), _ptr(sum_out),
                                         C.byref(fuse) if fuse is not None else None, _ptr(ws), _nbytes(ws)),
               "eoq_conv_bwd_data_sq")

    def conv_bwd_weight(self, desc, e, u, g_acc, absmax_slot, ws):
        _check(_lib.eoq_conv_bwd_weight(self._h, C.byref(desc), _ptr(e), _ptr(u), _ptr(g_acc), _ptr(absmax_slot),
                                        _ptr(ws), _nbytes(ws)), "eoq_conv_bwd_weight")

    def conv_bwd_weight_static(self, desc, e, u, g_acc, absmax_slot):
        _check(_lib.eoq_conv_bwd_weight_static(self._h, C.byref(desc), _ptr(e), _ptr(u), _ptr(g_acc),
                                               _ptr(absmax_slot)), "eoq_conv_bwd_weight_static")

    def relu_bwd(self, e0, mask, t_wide, e1, sum_e1=None, sum_e1t=None, absmax_e1=None):
        _check(_lib.eoq_relu_bwd(self._h, _ptr(e0), _ptr(mask), _ptr(t_wide), e0.numel(), _ptr(e1), _ptr(sum_e1),
                                 _ptr(sum_e1t), _ptr(absmax_e1)), "eoq_relu_bwd")

    def relu_bwd_recompute(self, desc, u, w, e0, mask, e1, sum_e1=None, sum_e1t=None, absmax_e1=None):
        _check(_lib.eoq_relu_bwd_recompute(self._h, C.byref(desc), _ptr(u), _ptr(w), _ptr(e0), _ptr(mask), _ptr(e1),
                                           _ptr(sum_e1), _ptr(sum_e1t), _ptr(absmax_e1)), "eoq_relu_bwd_recompute")

    def merge_absmax(self, a, exp_a, b, exp_b, absmax_slot):
        _check(_lib.eoq_merge_absmax(self._h, _ptr(a), _ptr(exp_a), _ptr(b), _ptr(exp_b), a.numel(),
                                     _ptr(absmax_slot)), "eoq_merge_absmax")

    def requant_epilogue(self, mode, n, *, K=0, acc=None, ep=None, src_a=None, src_b=None, exp_b=None, gamma=None,
                         absmax=None, exp_in=None, exp_in_off=0, out=None, exp_out=None, sum_out=None,
                         max_code_out=None, mask=None, absmax_out=None, out_b=None, exp_out_b=None,
                         absmax_masked=None):
        a = RequantArgs(mode, K, n, _ptr(acc), C.addressof(ep) if ep is not None else None, _ptr(src_a), _ptr(src_b),
                        _ptr(exp_b), _ptr(gamma), _ptr(absmax), _ptr(exp_in), exp_in_off, _ptr(out), _ptr(exp_out),
                        _ptr(sum_out), _ptr(max_code_out), _ptr(mask), _ptr(absmax_out), _ptr(out_b), _ptr(exp_out_b),
                        _ptr(absmax_masked))
        _check(_lib.eoq_requant_epilogue(self._h, C.byref(a)), "eoq_requant_epilogue")

    def update_int8(self, w, g, g_exp_slot, g_max_code, lr_slot, sr_slot=None, tensor_id=0):
        if sr_slot is not None:
            _check(_lib.eoq_update_int8_sr(self._h, _ptr(w), w.numel(), _ptr(g), _ptr(g_exp_slot), _ptr(g_max_code),
                                           _ptr(lr_slot), _ptr(sr_slot), tensor_id), "eoq_update_int8_sr")
            return
        _check(_lib.eoq_update_int8(self._h, _ptr(w), w.numel(), _ptr(g), _ptr(g_exp_slot), _ptr(g_max_code),
                                    _ptr(lr_slot)), "eoq_update_int8")

    def sr_next_step(self, sr_slot):
        _check(_lib.eoq_sr_next_step(self._h, _ptr(sr_slot)), "eoq_sr_next_step")

    def grad_update(self, desc, acc, absmax_slot, exp_in, exp_in_off, lr_slot, w, wt=None, g_out=None, exp_out=None,
                    max_code_out=None, sr_slot=None, tensor_id=0):
        if sr_slot is not None:
            _check(_lib.eoq_grad_update_sr(self._h, C.byref(desc), _ptr(acc), _ptr(absmax_slot), _ptr(exp_in), exp_in_off,
                                           _ptr(lr_slot), _ptr(w), _ptr(wt), _ptr(g_out), _ptr(exp_out),
                                           _ptr(max_code_out), _ptr(sr_slot), tensor_id), "eoq_grad_update_sr")
            return
        _check(_lib.eoq_grad_update(self._h, C.byref(desc), _ptr(acc), _ptr(absmax_slot), _ptr(exp_in), exp_in_off,
                                    _ptr(lr_slot), _ptr(w), _ptr(wt), _ptr(g_out), _ptr(exp_out), _ptr(max_code_out)),
               "eoq_grad_update")

    def update_scalars(self, scalars, descs, count, sums, exps, lr_slot, g_code_out=None, g_exp_out=None,
                       sr_slot=None, tensor_ids=None):
        if sr_slot is not None:
            _check(_lib.eoq_update_scalars_sr(self._h, _ptr(scalars), _ptr(descs), count, _ptr(sums), _ptr(exps),
                                              _ptr(lr_slot), _ptr(g_code_out), _ptr(g_exp_out), _ptr(sr_slot),
                                              _ptr(tensor_ids)), "eoq_update_scalars_sr")
            return
        _check(_lib.eoq_update_scalars(self._h, _ptr(scalars), _ptr(descs), count, _ptr(sums), _ptr(exps),
                                       _ptr(lr_slot), _ptr(g_code_out), _ptr(g_exp_out)), "eoq_update_scalars")

    def maxpool_fwd(self, a, N, H, W, Cc, R, S, stride, pad, y, b_next_pre=None, u_next=None, arg=None):
        _check(_lib.eoq_maxpool_fwd(self._h, _ptr(a), N, H, W, Cc, R, S, stride, pad, _ptr(y), _ptr(b_next_pre),
                                    _ptr(u_next), _ptr(arg)), "eoq_maxpool_fwd")

    def maxpool_bwd(self, arg, e, N, H, W, Cc, R, S, stride, pad, d, absmax_slot):
        _check(_lib.eoq_maxpool_bwd(self._h, _ptr(arg), _ptr(e), N, H, W, Cc, R, S, stride, pad, _ptr(d),
                                    _ptr(absmax_slot)), "eoq_maxpool_bwd")

    def maxpool_bwd_sq(self, arg, e, N, H, W, Cc, R, S, stride, pad, e_out, absmax_slot, exp_in, exp_out, mask=None,
                       sum_out=None, spec_state=None):
        _check(_lib.eoq_maxpool_bwd_sq(self._h, _ptr(arg), _ptr(e), N, H, W, Cc, R, S, stride, pad, _ptr(e_out),
                                       _ptr(absmax_slot), _ptr(exp_in), _ptr(exp_out), _ptr(mask), _ptr(sum_out),
                                       _ptr(spec_state)), "eoq_maxpool_bwd_sq")

    def gap_sum(self, y, N, HW, Cc, out):
        _check(_lib.eoq_gap_sum(self._h, _ptr(y), N, HW, Cc, _ptr(out)), "eoq_gap_sum")

    def broadcast_hw(self, codes, N, HW, Cc, e):
        _check(_lib.eoq_broadcast_hw(self._h, _ptr(codes), N, HW, Cc, _ptr(e)), "eoq_broadcast_hw")

    @staticmethod
    def head_workspace_bytes(N, F, J) -> int:
        return _lib.eoq_head_workspace_bytes(N, F, J)

    def head_fwd_bwd(self, N, F, J, HW, gap_sum, Wfc, bfc, labels, lr_slot, loss, d, logits, ws):
        _check(_lib.eoq_head_fwd_bwd(self._h, N, F, J, HW, _ptr(gap_sum), _ptr(Wfc), _ptr(bfc), _ptr(labels),
                                     _ptr(lr_slot), _ptr(loss), _ptr(d), _ptr(logits), _ptr(ws), _nbytes(ws)),
               "eoq_head_fwd_bwd")

    def head_update(self, N, F, J, Wfc, bfc, lr_slot, ws):
        _check(_lib.eoq_head_update(self._h, N, F, J, _ptr(Wfc), _ptr(bfc), _ptr(lr_slot), _ptr(ws), _nbytes(ws)),
               "eoq_head_update")


def scalar_grad_table(entries, device) -> torch.Tensor:
    """Pack [(param, [(sum_idx, exp_idx, exp_off), ...]), ...] into a device array of eoq_scalar_grad."""
    import numpy as np
    arr = np.zeros((len(entries), 8), dtype=np.int32)
    for i, (param, terms) in enumerate(entries):
        assert 1 <= len(terms) <= 2
        arr[i, 0], arr[i, 1] = param, len(terms)
        for t, (si, ei, eo) in enumerate(terms):
            arr[i, 2 + t], arr[i, 4 + t], arr[i, 6 + t] = si, ei, eo
    assert C.sizeof(ScalarGrad) == 32
    return torch.from_numpy(arr).to(device)
