"""Thin ctypes binding of libquaff.so: the same entry points as include/quaff.h, taking torch device tensors.

Argument marshalling only - every step of the path runs in the HIP kernels behind the C ABI.  PyTorch is used
for device memory (`tensor.data_ptr()`) and the current HIP stream.  The library must have been built
(`python -m paper_2505_14742_amd.build`); loading fails loudly otherwise - there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libquaff.so")

OK, ERR_NULL, ERR_SHAPE, ERR_WORKSPACE, ERR_ALIGN, ERR_HIP = 0, -1, -2, -3, -4, -5

_vp, _i64, _i32, _f32, _sz = C.c_void_p, C.c_int64, C.c_int32, C.c_float, C.c_size_t

SIGNATURES = {
    "quaff_status_string": (C.c_char_p, [C.c_int]),
    "quaff_last_hip_error": (C.c_int, []),
    "quaff_padded_outliers": (_i32, [_i32]),
    "quaff_packed_weight_bytes": (_sz, [_i64, _i64]),
    "quaff_packed_weight_offset": (_i64, [_i64, _i64, _i64, _i64]),
    "quaff_prepare_workspace_bytes": (_sz, [_i64, _i64]),
    "quaff_workspace_bytes": (_sz, [_i64, _i64, _i64, _i32, _i32]),
    "quaff_prepare_weight": (C.c_int, [_vp, _i64, _i64, _i64, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "quaff_scale_update": (C.c_int, [_vp, _i64, _i64, _i64, _vp, _i32, _vp, _vp, _i64, _f32, _vp, _vp, _vp, _vp, _vp,
                                     _vp, _sz, _vp]),
    "quaff_check_outliers": (C.c_int, [_vp, _i32, _i64, _vp, _vp]),
    "quaff_scale_update_static_max_outliers": (_i32, []),
    "quaff_scale_update_static": (C.c_int, [_vp, _i64, _i64, _i64, _vp, _i32, _vp, _vp, _i64, _f32, _vp, _vp, _vp, _vp,
                                            _vp, _vp]),
    "quaff_quant_act": (C.c_int, [_vp, _i64, _i64, _i64, _vp, _vp, _i32, _vp, _vp, _vp, _vp]),
    "quaff_linear_fwd": (C.c_int, [_vp, _vp, _vp, _i64, _vp, _vp, _i64, _i64, _vp, _vp, _i32, _vp, _i64, _vp, _vp,
                                   _i32, _f32, _vp, _i64, _vp, _sz, _vp]),
    "quaff_linear_fwd_bf16": (C.c_int, [_vp, _vp, _vp, _i64, _vp, _vp, _i64, _i64, _vp, _vp, _i32, _vp, _i64, _vp, _vp,
                                   _i32, _f32, _vp, _i64, _vp, _sz, _vp]),
    "quaff_linear_fwd_acc": (C.c_int, [_vp, _vp, _i64, _vp, _i64, _i64, _vp, _i32, _vp, _vp, _vp]),
    "quaff_linear_bwd_dx": (C.c_int, [_vp, _i64, _i64, _vp, _vp, _i64, _i64, _vp, _vp, _i32, _f32, _vp, _i64, _vp,
                                      _sz, _vp]),
    "quaff_linear_bwd_dx_bf16": (C.c_int, [_vp, _i64, _i64, _vp, _vp, _i64, _i64, _vp, _vp, _i32, _f32, _vp, _i64, _vp,
                                      _sz, _vp]),
    "quaff_linear_bwd_dx_acc": (C.c_int, [_vp, _i64, _i64, _vp, _vp, _i64, _i64, _vp, _vp, _vp, _vp]),
    "quaff_lora_bwd_workspace_bytes": (_sz, [_i64, _i64, _i64, _i32]),
    "quaff_bwd_step_workspace_bytes": (_sz, [_i64, _i64, _i64, _i32]),
    "quaff_linear_bwd_step": (C.c_int, [_vp, _i64, _i64, _vp, _i64, _vp, _vp, _i64, _i64, _vp, _vp, _i32, _f32, _vp,
                                        _i64, _vp, _vp, _vp, _sz, _vp, _vp, _vp, _vp]),
    "quaff_lora_bwd_weights": (C.c_int, [_vp, _i64, _vp, _i64, _i64, _i64, _i64, _vp, _vp, _i32, _f32, _vp, _vp, _vp,
                                         _sz, _vp]),
    "quaff_bwd_dx_outlier_workspace_bytes": (_sz, [_i64, _i64]),
    "quaff_bwd_dx_outlier_exact": (C.c_int, [_vp, _i64, _i64, _i64, _i64, _vp, _i32, _vp, _vp, _vp, _i32, _f32, _vp,
                                             _i64, _vp, _sz, _vp]),
    "quaff_calibrate_workspace_bytes": (_sz, [_i64, _i32]),
    "quaff_calibrate_outliers": (C.c_int, [_vp, _i64, _i64, _i64, _vp, _i32, C.c_double, _i32, _vp, _vp, _vp, _vp, _sz,
                                           _vp]),
    "quaff_fwd_step_workspace_bytes": (_sz, [_i64, _i64, _i64, _i32, _i32]),
    "quaff_linear_fwd_step": (C.c_int, [_vp, _i64, _i64, _i64, _vp, _i32, _vp, _vp, _i64, _f32, _vp, _vp, _vp, _vp, _vp,
                                        _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _f32, _vp, _i64, _vp, _sz, _vp]),
    "quaff_debug_grid_wait_ticks": (C.c_longlong, [C.c_longlong]),
    "quaff_profile_enable": (C.c_int, [C.c_int]),
    "quaff_profile_collect": (_i64, []),
    "quaff_profile_launch": (C.c_int, [_i64, C.POINTER(C.c_int), C.POINTER(C.c_float)]),
    "quaff_profile_kind_name": (C.c_char_p, [C.c_int]),
    "quaff_microbench_mfma_i8": (C.c_int, [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "quaff_microbench_copy": (C.c_int, [_sz, C.POINTER(C.c_double)]),
}

_lib = None


class QuaffError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        msg = lib().quaff_status_string(status).decode()
        if status == ERR_HIP:
            msg += " (hipError %d)" % lib().quaff_last_hip_error()
        super().__init__(msg)


def lib():
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libquaff.so is not built: run `python -m paper_2505_14742_amd.build` "
                               "(there is no CPU or PyTorch fallback for this path)")
        # PyTorch ships its own copy of the HIP runtime.  The tensors handed to this library live in that runtime's
        # context, so it must be the one libquaff.so binds to: load torch first (a process that loaded libquaff.so
        # before torch got two runtimes and "no device" from the first launch).
        import torch  # noqa: F401
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(status):
    if status != OK:
        raise QuaffError(status)


def padded_outliers(n: int) -> int:
    return int(lib().quaff_padded_outliers(n))


def packed_weight_bytes(c_in: int, c_out: int) -> int:
    return int(lib().quaff_packed_weight_bytes(c_in, c_out))


def packed_weight_offset(c_in: int, c_out: int, k: int, j: int) -> int:
    return int(lib().quaff_packed_weight_offset(c_in, c_out, k, j))


def prepare_workspace_bytes(c_in: int, c_out: int) -> int:
    return int(lib().quaff_prepare_workspace_bytes(c_in, c_out))


def workspace_bytes(t: int, c_in: int, c_out: int, n_outlier: int, lora_rank: int) -> int:
    return int(lib().quaff_workspace_bytes(t, c_in, c_out, n_outlier, lora_rank))


def prepare_weight(W, O, Wq_packed, delta_w, W_O, wmax_O, Wq_plain, workspace):
    c_in, c_out = W.shape
    n = 0 if O is None else O.numel()
    _check(lib().quaff_prepare_weight(_ptr(W), c_in, c_out, W.stride(0), _ptr(O), n, _ptr(Wq_packed), _ptr(delta_w),
                                      _ptr(W_O), _ptr(wmax_O), _ptr(Wq_plain), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream()))


def scale_update(X, O, W_O, wmax_O, c_out, gamma, s_O, colscale, what_int, delta_what, cmax_out, workspace):
    t, c_in = X.shape
    n = 0 if O is None else O.numel()
    _check(lib().quaff_scale_update(_ptr(X), t, c_in, X.stride(0), _ptr(O), n, _ptr(W_O), _ptr(wmax_O), c_out,
                                    float(gamma), _ptr(s_O), _ptr(colscale), _ptr(what_int), _ptr(delta_what),
                                    _ptr(cmax_out), _ptr(workspace),
                                    0 if workspace is None else workspace.numel() * workspace.element_size(),
                                    _stream()))


def check_outliers(O, c_in, result):
    """Enqueue the validity scan of O; `result` is a one-element int32 device tensor (0 = valid, else 1 + position)."""
    n = 0 if O is None else O.numel()
    _check(lib().quaff_check_outliers(_ptr(O), n, c_in, _ptr(result), _stream()))


def scale_update_static_max_outliers() -> int:
    return int(lib().quaff_scale_update_static_max_outliers())


def scale_update_static(X, O, W_O, wmax_O, c_out, gamma, s_O, colscale, what_int, delta_what, cmax_out):
    t, c_in = X.shape
    n = 0 if O is None else O.numel()
    _check(lib().quaff_scale_update_static(_ptr(X), t, c_in, X.stride(0), _ptr(O), n, _ptr(W_O), _ptr(wmax_O), c_out,
                                           float(gamma), _ptr(s_O), _ptr(colscale), _ptr(what_int), _ptr(delta_what),
                                           _ptr(cmax_out), _stream()))


def quant_act(X, colscale, O, Xq, delta, xq_O):
    t, c = X.shape
    n = 0 if O is None else O.numel()
    _check(lib().quaff_quant_act(_ptr(X), t, c, X.stride(0), _ptr(colscale), _ptr(O), n, _ptr(Xq), _ptr(delta),
                                 _ptr(xq_O), _stream()))


def linear_fwd(Xq, delta_x, xq_O, Wq_packed, delta_w, c_in, c_out, what_int, delta_what, n_outlier, X, lora_A, lora_B,
               lora_rank, lora_scale, Y, workspace, bf16_out=False):
    t = Xq.shape[0]
    fn = lib().quaff_linear_fwd_bf16 if bf16_out else lib().quaff_linear_fwd
    _check(fn(_ptr(Xq), _ptr(delta_x), _ptr(xq_O), t, _ptr(Wq_packed), _ptr(delta_w), c_in, c_out,
                                  _ptr(what_int), _ptr(delta_what), n_outlier, _ptr(X),
                                  0 if X is None else X.stride(0), _ptr(lora_A), _ptr(lora_B), lora_rank,
                                  float(lora_scale), _ptr(Y), Y.stride(0), _ptr(workspace),
                                  0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


def linear_fwd_acc(Xq, xq_O, Wq_packed, c_in, c_out, what_int, n_outlier, acc1, acc2):
    t = Xq.shape[0]
    _check(lib().quaff_linear_fwd_acc(_ptr(Xq), _ptr(xq_O), t, _ptr(Wq_packed), c_in, c_out, _ptr(what_int),
                                      n_outlier, _ptr(acc1), _ptr(acc2), _stream()))


def linear_bwd_dx(dY, Wq_packed, delta_w, c_in, c_out, lora_A, lora_B, lora_rank, lora_scale, dX, workspace,
                  bf16_out=False):
    t = dY.shape[0]
    fn = lib().quaff_linear_bwd_dx_bf16 if bf16_out else lib().quaff_linear_bwd_dx
    _check(fn(_ptr(dY), t, dY.stride(0), _ptr(Wq_packed), _ptr(delta_w), c_in, c_out,
                                     _ptr(lora_A), _ptr(lora_B), lora_rank, float(lora_scale), _ptr(dX), dX.stride(0),
                                     _ptr(workspace),
                                     0 if workspace is None else workspace.numel() * workspace.element_size(),
                                     _stream()))


def lora_bwd_workspace_bytes(t, c_in, c_out, lora_rank) -> int:
    return int(lib().quaff_lora_bwd_workspace_bytes(t, c_in, c_out, lora_rank))


def lora_bwd_weights(X, dY, lora_A, lora_B, lora_rank, lora_scale, dA, dB, workspace):
    t, c_in, c_out = X.shape[0], X.shape[1], dY.shape[1]
    _check(lib().quaff_lora_bwd_weights(_ptr(X), X.stride(0), _ptr(dY), dY.stride(0), t, c_in, c_out, _ptr(lora_A),
                                        _ptr(lora_B), lora_rank, float(lora_scale), _ptr(dA), _ptr(dB),
                                        _ptr(workspace),
                                        0 if workspace is None else workspace.numel() * workspace.element_size(),
                                        _stream()))


def bwd_step_workspace_bytes(t, c_in, c_out, lora_rank) -> int:
    return int(lib().quaff_bwd_step_workspace_bytes(t, c_in, c_out, lora_rank))


class SideStream:
    """A second stream and two events (timing disabled) for quaff_linear_bwd_step, owned by the caller."""

    def __init__(self):
        import torch
        self.stream = torch.cuda.Stream()
        self.fork, self.join = torch.cuda.Event(), torch.cuda.Event()
        for ev in (self.fork, self.join):   # torch creates the underlying event at its first record
            ev.record(self.stream)
        self.stream.synchronize()

    def handles(self):
        return self.stream.cuda_stream, self.fork.cuda_event, self.join.cuda_event


def linear_bwd_step(dY, X, Wq_packed, delta_w, c_in, c_out, lora_A, lora_B, lora_rank, lora_scale, dX, dA, dB, workspace,
                    side=None):
    """side: a SideStream (the weight gradients then run beside the input-gradient product) or None."""
    t = dY.shape[0]
    hs, hf, hj = side.handles() if side is not None else (None, None, None)
    _check(lib().quaff_linear_bwd_step(_ptr(dY), t, dY.stride(0), _ptr(X), X.stride(0), _ptr(Wq_packed), _ptr(delta_w),
                                       c_in, c_out, _ptr(lora_A), _ptr(lora_B), lora_rank, float(lora_scale), _ptr(dX),
                                       dX.stride(0), _ptr(dA), _ptr(dB), _ptr(workspace),
                                       0 if workspace is None else workspace.numel() * workspace.element_size(),
                                       _stream(), hs, hf, hj))


def bwd_dx_outlier_workspace_bytes(t, c_out) -> int:
    return int(lib().quaff_bwd_dx_outlier_workspace_bytes(t, c_out))


def bwd_dx_outlier_exact(dY, c_in, O, W_O, lora_A, lora_B, lora_rank, lora_scale, dX, workspace):
    t, c_out = dY.shape[0], dY.shape[1]
    n = 0 if O is None else O.numel()
    _check(lib().quaff_bwd_dx_outlier_exact(_ptr(dY), t, dY.stride(0), c_in, c_out, _ptr(O), n, _ptr(W_O),
                                            _ptr(lora_A), _ptr(lora_B), lora_rank, float(lora_scale), _ptr(dX),
                                            dX.stride(0), _ptr(workspace),
                                            0 if workspace is None else workspace.numel() * workspace.element_size(),
                                            _stream()))


def calibrate_workspace_bytes(c_in, n_samples) -> int:
    return int(lib().quaff_calibrate_workspace_bytes(c_in, n_samples))


def calibrate_outliers(X, sample_offsets, ratio, budget, xi, O, n_outlier, workspace):
    t_total, c_in = X.shape[0], X.shape[1]
    _check(lib().quaff_calibrate_outliers(_ptr(X), t_total, c_in, X.stride(0), _ptr(sample_offsets),
                                          sample_offsets.numel() - 1, float(ratio), budget, _ptr(xi), _ptr(O),
                                          _ptr(n_outlier), _ptr(workspace),
                                          0 if workspace is None else workspace.numel() * workspace.element_size(),
                                          _stream()))


def fwd_step_workspace_bytes(t, c_in, c_out, n_outlier, lora_rank) -> int:
    return int(lib().quaff_fwd_step_workspace_bytes(t, c_in, c_out, n_outlier, lora_rank))


def linear_fwd_step(X, O, W_O, wmax_O, c_out, gamma, s_O, colscale, what_int, delta_what, cmax_out, Xq, delta_x, xq_O,
                    Wq_packed, delta_w, lora_A, lora_B, lora_rank, lora_scale, Y, workspace):
    t, c_in = X.shape[0], X.shape[1]
    n = 0 if O is None else O.numel()
    _check(lib().quaff_linear_fwd_step(_ptr(X), t, c_in, X.stride(0), _ptr(O), n, _ptr(W_O), _ptr(wmax_O), c_out,
                                       float(gamma), _ptr(s_O), _ptr(colscale), _ptr(what_int), _ptr(delta_what),
                                       _ptr(cmax_out), _ptr(Xq), _ptr(delta_x), _ptr(xq_O), _ptr(Wq_packed),
                                       _ptr(delta_w), _ptr(lora_A), _ptr(lora_B), lora_rank, float(lora_scale),
                                       _ptr(Y), Y.stride(0), _ptr(workspace),
                                       0 if workspace is None else workspace.numel() * workspace.element_size(),
                                       _stream()))


def debug_grid_wait_ticks(ticks: int) -> int:
    """Set (ticks >= 0) or read (ticks < 0) the bound of the one-launch forward preparation's grid-wide wait."""
    return int(lib().quaff_debug_grid_wait_ticks(ticks))


def linear_bwd_dx_acc(dY, Wq_packed, delta_w, c_in, c_out, Gq, delta_g, acc):
    t = dY.shape[0]
    _check(lib().quaff_linear_bwd_dx_acc(_ptr(dY), t, dY.stride(0), _ptr(Wq_packed), _ptr(delta_w), c_in, c_out,
                                         _ptr(Gq), _ptr(delta_g), _ptr(acc), _stream()))


def profile_enable(on: bool):
    _check(lib().quaff_profile_enable(1 if on else 0))


def profile_launches():
    """[(kernel kind name, milliseconds), ...] of every launch recorded since profile_enable(True), in order."""
    n = int(lib().quaff_profile_collect())
    if n < 0:
        raise QuaffError(ERR_HIP)
    out = []
    kind, ms = C.c_int(), C.c_float()
    for i in range(n):
        _check(lib().quaff_profile_launch(i, C.byref(kind), C.byref(ms)))
        out.append((lib().quaff_profile_kind_name(kind.value).decode(), float(ms.value)))
    return out


def microbench_mfma_i8(random_operands: bool):
    """(TOP/s, shader clock MHz) of a register-only INT8 MFMA loop on the whole chip."""
    tops, mhz = C.c_double(), C.c_double()
    _check(lib().quaff_microbench_mfma_i8(1 if random_operands else 0, C.byref(tops), C.byref(mhz)))
    return tops.value, mhz.value


def microbench_copy(nbytes: int = 1 << 30) -> float:
    """GB/s (read + write) of a streaming device copy."""
    gbs = C.c_double()
    _check(lib().quaff_microbench_copy(nbytes, C.byref(gbs)))
    return gbs.value
