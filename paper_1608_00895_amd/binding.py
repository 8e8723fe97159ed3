"""Thin ctypes binding of librlstm.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
include/rlstm.h.  Tensors are torch CUDA (ROCm) tensors used purely as device
memory; streams are torch streams or None (the current stream).  Nothing is
computed here, and there is no fallback: if the library is missing, loading
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librlstm.so")

RLSTM_ENGINE_AUTO = 0
RLSTM_ENGINE_PERSISTENT = 1
RLSTM_ENGINE_STEPWISE = 2

EXPORTS = [
    "rlstm_reserve_bytes", "rlstm_workspace_bytes", "rblstm_reserve_bytes", "rblstm_workspace_bytes",
    "lstm_fwd", "lstm_bwd", "lstm_fwd_noalloc", "rlstm_noalloc_scratch_bytes", "rlstm_last_timeout_on",
    "blstm_stack_fwd_bwd", "blstm_stack_fwd", "blstm_stack_bwd",
    "rlstm_ce_workspace_bytes", "softmax_ce_fwd_bwd", "rlstm_sgd_momentum_step", "rlstm_adam_step",
    "rlstm_stream_reserve_bytes", "rlstm_stream_workspace_bytes", "lstm_stream_fwd_bwd",
    "rlstm_gemm_f32", "rlstm_gemm_bf16", "rlstm_to_bf16", "rlstm_to_bf16_2d", "rlstm_gemm_bf16_mem", "rlstm_copy_f32", "rlstm_profile_enable", "rlstm_profile_read", "rlstm_last_timeout", "rlstm_test_hook", "rlstm_test_delay", "rmdlstm_reserve_bytes", "rmdlstm_workspace_bytes", "mdlstm_fwd", "mdlstm_bwd", "rlstm_chunk_plan", "rlstm_chunk_gather", "rblstm_plan", "rlstm_exchange_floor_bytes", "rlstm_exchange_floor", "rlstm_resolve_engine", "rlstm_strerror", "rlstm_version",
]


class rlstm_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("T", "B", "D", "H", "direction", "operand_dtype", "ldx", "ldy", "engine",
                 "batch_groups", "bwd_exchange", "gemm_variant")]


class rblstm_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("L", "T", "B", "D", "H", "operand_dtype", "engine",
                                              "first_piece", "batch_groups", "overlap_mode", "gemm_variant", "bwd_exchange")]


class rlstm_stream_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("L", "S", "Tc", "B", "D", "H", "operand_dtype", "engine",
                                              "batch_groups", "bwd_exchange", "gemm_variant")]


class rmdlstm_desc(ctypes.Structure):
    _fields_ = [("Hh", ctypes.c_int32), ("Ww", ctypes.c_int32), ("B", ctypes.c_int32), ("D", ctypes.c_int32),
                ("H", ctypes.c_int32), ("operand_dtype", ctypes.c_int32), ("engine", ctypes.c_int32)]


class rlstm_profile_entry(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("layer", ctypes.c_int32), ("ndir", ctypes.c_int32),
                ("steps", ctypes.c_int32), ("ms", ctypes.c_float), ("reserved", ctypes.c_float),
                ("flop", ctypes.c_double)]


PROFILE_KINDS = {0: "input_projection", 1: "recurrent_forward", 2: "recurrent_backward",
                 3: "input_gradient", 4: "weight_gradient", 5: "recurrent_weight_gradient",
                 6: "output_layer_product", 7: "softmax_cross_entropy_rows"}


class RlstmError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where} failed: {code} ({strerror(code)})")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads librlstm.so (built in-tree by paper_1608_00895_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python paper_1608_00895_amd/build.py` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, ip = ctypes.c_void_p, ctypes.c_int
        for name in ("rlstm_reserve_bytes", "rlstm_workspace_bytes"):
            getattr(L, name).restype = ctypes.c_size_t
            getattr(L, name).argtypes = [ctypes.POINTER(rlstm_desc)]
        for name in ("rblstm_reserve_bytes", "rblstm_workspace_bytes"):
            getattr(L, name).restype = ctypes.c_size_t
            getattr(L, name).argtypes = [ctypes.POINTER(rblstm_desc)]
        L.lstm_fwd.restype = ip
        L.lstm_fwd.argtypes = [ctypes.POINTER(rlstm_desc)] + [vp] * 14
        L.lstm_bwd.restype = ip
        L.lstm_bwd.argtypes = [ctypes.POINTER(rlstm_desc)] + [vp] * 20
        L.lstm_fwd_noalloc.restype = ip
        L.lstm_fwd_noalloc.argtypes = [ctypes.POINTER(rlstm_desc)] + [vp] * 13
        L.rlstm_noalloc_scratch_bytes.restype = ctypes.c_size_t
        L.rlstm_noalloc_scratch_bytes.argtypes = [ctypes.POINTER(rlstm_desc)]
        L.rlstm_last_timeout_on.restype = ip
        L.rlstm_last_timeout_on.argtypes = [vp, vp]
        L.blstm_stack_fwd_bwd.restype = ip
        L.blstm_stack_fwd_bwd.argtypes = [ctypes.POINTER(rblstm_desc), vp, ctypes.POINTER(vp), vp, vp, vp,
                                          ctypes.POINTER(vp), vp, vp, vp, vp, vp]
        L.blstm_stack_bwd.restype = ip
        L.blstm_stack_bwd.argtypes = [ctypes.POINTER(rblstm_desc), vp, ctypes.POINTER(vp), vp, vp, vp,
                                      ctypes.POINTER(vp), vp, vp, vp, vp, vp]
        for name in ("rlstm_stream_reserve_bytes", "rlstm_stream_workspace_bytes"):
            getattr(L, name).restype = ctypes.c_size_t
            getattr(L, name).argtypes = [ctypes.POINTER(rlstm_stream_desc)]
        L.lstm_stream_fwd_bwd.restype = ip
        L.lstm_stream_fwd_bwd.argtypes = [ctypes.POINTER(rlstm_stream_desc), vp, ctypes.POINTER(vp), vp, vp, vp,
                                          ctypes.POINTER(vp), vp, vp, vp, vp, vp, vp]
        L.rlstm_ce_workspace_bytes.restype = ctypes.c_size_t
        L.rlstm_ce_workspace_bytes.argtypes = [ip, ip, ip, ip]
        L.softmax_ce_fwd_bwd.restype = ip
        L.softmax_ce_fwd_bwd.argtypes = [ip, ip, ip, ip, ip] + [vp] * 11 + [ctypes.c_size_t, vp]
        L.rlstm_sgd_momentum_step.restype = ip
        L.rlstm_sgd_momentum_step.argtypes = [vp, vp, vp, ctypes.c_size_t, ctypes.c_double, ctypes.c_double, vp]
        L.rlstm_adam_step.restype = ip
        L.rlstm_adam_step.argtypes = [vp, vp, vp, vp, ctypes.c_size_t, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                      ctypes.c_double, ip, vp]
        L.blstm_stack_fwd.restype = ip
        L.blstm_stack_fwd.argtypes = [ctypes.POINTER(rblstm_desc), vp, ctypes.POINTER(vp), vp, vp, vp, vp, vp]
        L.rlstm_gemm_f32.restype = ip
        L.rlstm_gemm_f32.argtypes = [ip, ip, ip, ip, ip, vp, ip, vp, ip, vp, ip, vp, ip, vp, ctypes.c_size_t, vp]
        L.rlstm_gemm_bf16.restype = ip
        L.rlstm_gemm_bf16.argtypes = L.rlstm_gemm_f32.argtypes
        L.rlstm_to_bf16.restype = ip
        L.rlstm_to_bf16.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.rlstm_gemm_bf16_mem.restype = ip
        L.rlstm_gemm_bf16_mem.argtypes = [ip, ip, ip, ip, ip, vp, ip, vp, ip, vp, ip, vp, ip, vp, ctypes.c_size_t, vp]
        L.rlstm_to_bf16_2d.restype = ip
        L.rlstm_to_bf16_2d.argtypes = [vp, vp, vp, ip, ip, ip, vp]
        L.rlstm_copy_f32.restype = ip
        L.rlstm_copy_f32.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.rlstm_profile_enable.restype = ip
        L.rlstm_profile_enable.argtypes = [ip]
        L.rlstm_profile_read.restype = ip
        L.rlstm_profile_read.argtypes = [ctypes.POINTER(rlstm_profile_entry), ip]
        L.rlstm_last_timeout.restype = ip
        L.rlstm_last_timeout.argtypes = [vp]
        for name in ("rmdlstm_reserve_bytes", "rmdlstm_workspace_bytes"):
            getattr(L, name).restype = ctypes.c_size_t
            getattr(L, name).argtypes = [ctypes.POINTER(rmdlstm_desc)]
        L.mdlstm_fwd.restype = ip
        L.mdlstm_fwd.argtypes = [ctypes.POINTER(rmdlstm_desc), vp, ctypes.POINTER(vp), vp, vp, vp, vp, vp]
        L.mdlstm_bwd.restype = ip
        L.mdlstm_bwd.argtypes = [ctypes.POINTER(rmdlstm_desc), vp, ctypes.POINTER(vp), vp, vp, vp, vp,
                                 ctypes.POINTER(vp), vp, vp]
        i32p = ctypes.POINTER(ctypes.c_int32)
        L.rlstm_chunk_plan.restype = ctypes.c_longlong
        L.rlstm_chunk_plan.argtypes = [i32p, ip, ip, ip, i32p, i32p, i32p, ctypes.c_longlong]
        L.rlstm_chunk_gather.restype = ip
        L.rlstm_chunk_gather.argtypes = [vp, ip, ip, ip, ip, vp, vp, vp, ip, ip, vp, vp]
        L.rblstm_plan.restype = ip
        L.rblstm_plan.argtypes = [ctypes.POINTER(rblstm_desc), ctypes.POINTER(ctypes.c_int32)]
        L.rlstm_exchange_floor_bytes.restype = ctypes.c_size_t
        L.rlstm_exchange_floor_bytes.argtypes = [ip, ip, ip]
        L.rlstm_exchange_floor.restype = ip
        L.rlstm_exchange_floor.argtypes = [ip, ip, ip, ip, ip, vp, ctypes.c_size_t, ctypes.POINTER(ctypes.c_float), vp]
        L.rlstm_test_hook.restype = ip
        L.rlstm_test_hook.argtypes = [ip, ctypes.c_uint64]
        L.rlstm_test_delay.restype = ip
        L.rlstm_test_delay.argtypes = [ip, ctypes.c_uint32]
        L.rlstm_resolve_engine.restype = ip
        L.rlstm_resolve_engine.argtypes = [ctypes.POINTER(rlstm_desc)]
        L.rlstm_strerror.restype = ctypes.c_char_p
        L.rlstm_strerror.argtypes = [ip]
        L.rlstm_version.restype = ctypes.c_char_p
        L.rlstm_version.argtypes = []
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().rlstm_strerror(int(code)).decode()


def version() -> str:
    return lib().rlstm_version().decode()


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("librlstm takes device pointers: pass a tensor on the GPU")
    return ctypes.c_void_p(t.data_ptr())


def _stream(s) -> ctypes.c_void_p:
    if s is None:
        s = torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _ptr_array(ts: Sequence[torch.Tensor]):
    arr = (ctypes.c_void_p * len(ts))()
    for i, t in enumerate(ts):
        if not t.is_cuda:
            raise ValueError("librlstm takes device pointers: pass tensors on the GPU")
        arr[i] = t.data_ptr()
    return arr


def rlstm_reserve_bytes(desc: rlstm_desc) -> int:
    return int(lib().rlstm_reserve_bytes(ctypes.byref(desc)))


def rlstm_workspace_bytes(desc: rlstm_desc) -> int:
    return int(lib().rlstm_workspace_bytes(ctypes.byref(desc)))


def rblstm_reserve_bytes(desc: rblstm_desc) -> int:
    return int(lib().rblstm_reserve_bytes(ctypes.byref(desc)))


def rblstm_workspace_bytes(desc: rblstm_desc) -> int:
    return int(lib().rblstm_workspace_bytes(ctypes.byref(desc)))


def rlstm_resolve_engine(desc: rlstm_desc) -> int:
    return int(lib().rlstm_resolve_engine(ctypes.byref(desc)))


def rlstm_last_timeout(workspace: torch.Tensor) -> int:
    return int(lib().rlstm_last_timeout(_ptr(workspace)))


RLSTM_NOALLOC_SCRATCH_LIMIT = 16 << 20


def rlstm_last_timeout_on(workspace: Optional[torch.Tensor], stream=None) -> int:
    """workspace None: the flag of lstm_fwd_noalloc on the current device."""
    return int(lib().rlstm_last_timeout_on(_ptr(workspace), _stream(stream)))


def rlstm_noalloc_scratch_bytes(desc: rlstm_desc) -> int:
    return int(lib().rlstm_noalloc_scratch_bytes(ctypes.byref(desc)))


def lstm_fwd_noalloc(desc, x, W, R, b, h0, c0, seq_lens, y, c, hT, cT, reserve, stream=None, check=True) -> int:
    rc = lib().lstm_fwd_noalloc(ctypes.byref(desc), _ptr(x), _ptr(W), _ptr(R), _ptr(b), _ptr(h0), _ptr(c0),
                                _ptr(seq_lens), _ptr(y), _ptr(c), _ptr(hT), _ptr(cT), _ptr(reserve), _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "lstm_fwd_noalloc")
    return rc


def lstm_fwd(desc, x, W, R, b, h0, c0, seq_lens, y, c, hT, cT, reserve, workspace, stream=None, check=True) -> int:
    rc = lib().lstm_fwd(ctypes.byref(desc), _ptr(x), _ptr(W), _ptr(R), _ptr(b), _ptr(h0), _ptr(c0), _ptr(seq_lens),
                        _ptr(y), _ptr(c), _ptr(hT), _ptr(cT), _ptr(reserve), _ptr(workspace), _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "lstm_fwd")
    return rc


def lstm_bwd(desc, x, W, R, seq_lens, h0, c0, y, c, reserve, dy, dhT, dcT, dx, dW, dR, db, dh0, dc0,
             workspace, stream=None, check=True) -> int:
    rc = lib().lstm_bwd(ctypes.byref(desc), _ptr(x), _ptr(W), _ptr(R), _ptr(seq_lens), _ptr(h0), _ptr(c0),
                        _ptr(y), _ptr(c), _ptr(reserve), _ptr(dy), _ptr(dhT), _ptr(dcT),
                        _ptr(dx), _ptr(dW), _ptr(dR), _ptr(db), _ptr(dh0), _ptr(dc0),
                        _ptr(workspace), _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "lstm_bwd")
    return rc


def blstm_stack_fwd_bwd(desc, x, params, seq_lens, dy_top, y_top, grads, dx, reserve, workspace,
                        stream_a=None, stream_b=None, check=True) -> int:
    """params / grads: flat sequences of 6*L tensors (layer-major, forward direction first: W, R, b)."""
    pa, ga = _ptr_array(params), _ptr_array(grads)
    sb = ctypes.c_void_p(stream_b.cuda_stream) if stream_b is not None else None
    rc = lib().blstm_stack_fwd_bwd(ctypes.byref(desc), _ptr(x), pa, _ptr(seq_lens), _ptr(dy_top), _ptr(y_top),
                                   ga, _ptr(dx), _ptr(reserve), _ptr(workspace), _stream(stream_a), sb)
    if check and rc != 0:
        raise RlstmError(rc, "blstm_stack_fwd_bwd")
    return rc


def blstm_stack_bwd(desc, x, params, seq_lens, dy_top, y_top, grads, dx, reserve, workspace,
                    stream_a=None, stream_b=None, check=True) -> int:
    """Backward half alone, after blstm_stack_fwd with the same reserve and workspace."""
    pa, ga = _ptr_array(params), _ptr_array(grads)
    sb = ctypes.c_void_p(stream_b.cuda_stream) if stream_b is not None else None
    rc = lib().blstm_stack_bwd(ctypes.byref(desc), _ptr(x), pa, _ptr(seq_lens), _ptr(dy_top), _ptr(y_top),
                               ga, _ptr(dx), _ptr(reserve), _ptr(workspace), _stream(stream_a), sb)
    if check and rc != 0:
        raise RlstmError(rc, "blstm_stack_bwd")
    return rc


def rlstm_stream_reserve_bytes(desc) -> int:
    return int(lib().rlstm_stream_reserve_bytes(ctypes.byref(desc)))


def rlstm_stream_workspace_bytes(desc) -> int:
    return int(lib().rlstm_stream_workspace_bytes(ctypes.byref(desc)))


def lstm_stream_fwd_bwd(desc, x, params, seq_lens, dy_top, y_top, grads, dx, state, reserve, workspace, stream=None,
                        check=True, stream_b=None) -> int:
    """params / grads: flat sequences of 3*L tensors (W, R, b per layer); state: [L,2,B,H] tensor or None."""
    pa, ga = _ptr_array(params), _ptr_array(grads)
    rc = lib().lstm_stream_fwd_bwd(ctypes.byref(desc), _ptr(x), pa, _ptr(seq_lens), _ptr(dy_top), _ptr(y_top), ga,
                                   _ptr(dx), _ptr(state), _ptr(reserve), _ptr(workspace), _stream(stream),
                                   _stream(stream_b) if stream_b is not None else None)
    if check and rc != 0:
        raise RlstmError(rc, "lstm_stream_fwd_bwd")
    return rc


def rlstm_ce_workspace_bytes(T: int, B: int, F: int, C: int) -> int:
    return int(lib().rlstm_ce_workspace_bytes(T, B, F, C))


def softmax_ce_fwd_bwd(T, B, F, C, operand_dtype, y, Wo, bo, labels, seq_lens, loss, errors, dy, dWo, dbo, workspace,
                       stream=None, check=True) -> int:
    """loss: float32[1], errors: int32[1] device tensors; workspace: uint8 tensor of rlstm_ce_workspace_bytes()."""
    rc = lib().softmax_ce_fwd_bwd(T, B, F, C, operand_dtype, _ptr(y), _ptr(Wo), _ptr(bo), _ptr(labels), _ptr(seq_lens),
                                  _ptr(loss), _ptr(errors), _ptr(dy), _ptr(dWo), _ptr(dbo), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "softmax_ce_fwd_bwd")
    return rc


def rlstm_sgd_momentum_step(param, grad, velocity, learning_rate, momentum, stream=None, check=True) -> int:
    rc = lib().rlstm_sgd_momentum_step(_ptr(param), _ptr(grad), _ptr(velocity), param.numel(), learning_rate, momentum,
                                       _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "rlstm_sgd_momentum_step")
    return rc


def rlstm_adam_step(param, grad, m, v, learning_rate, beta1, beta2, epsilon, step, stream=None, check=True) -> int:
    rc = lib().rlstm_adam_step(_ptr(param), _ptr(grad), _ptr(m), _ptr(v), param.numel(), learning_rate, beta1, beta2,
                               epsilon, step, _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "rlstm_adam_step")
    return rc


def blstm_stack_fwd(desc, x, params, seq_lens, y_top, reserve, workspace, stream_a=None, check=True) -> int:
    pa = _ptr_array(params)
    rc = lib().blstm_stack_fwd(ctypes.byref(desc), _ptr(x), pa, _ptr(seq_lens), _ptr(y_top),
                               _ptr(reserve), _ptr(workspace), _stream(stream_a))
    if check and rc != 0:
        raise RlstmError(rc, "blstm_stack_fwd")
    return rc


def rlstm_gemm_f32(trans_a, trans_b, M, N, K, A, lda, B, ldb, C, ldc, bias=None, splitk_ws=None,
                   stream=None, check=True, variant=0) -> int:
    nbytes = 0 if splitk_ws is None else splitk_ws.numel() * splitk_ws.element_size()
    rc = lib().rlstm_gemm_f32(int(trans_a), int(trans_b), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc,
                              _ptr(bias), int(variant), _ptr(splitk_ws), nbytes, _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "rlstm_gemm_f32")
    return rc


def rlstm_profile_enable(on: bool) -> int:
    return int(lib().rlstm_profile_enable(1 if on else 0))


def rlstm_profile_read(max_entries: int = 4096):
    """Returns the recorded (kind, layer, ndir, ms, steps, flop) entries in launch order and clears the record."""
    buf = (rlstm_profile_entry * max_entries)()
    n = int(lib().rlstm_profile_read(buf, max_entries))
    if n < 0:
        raise RlstmError(n, "rlstm_profile_read")
    return [(buf[i].kind, buf[i].layer, buf[i].ndir, float(buf[i].ms), buf[i].steps, float(buf[i].flop))
            for i in range(min(n, max_entries))]


def rlstm_copy_f32(dst, src, n, stream=None, check=True) -> int:
    rc = lib().rlstm_copy_f32(_ptr(dst), _ptr(src), int(n), _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "rlstm_copy_f32")
    return rc


def rlstm_gemm_bf16(trans_a, trans_b, M, N, K, A, lda, B, ldb, C, ldc, bias=None, splitk_ws=None,
                    stream=None, check=True, variant=0) -> int:
    nbytes = 0 if splitk_ws is None else splitk_ws.numel() * splitk_ws.element_size()
    rc = lib().rlstm_gemm_bf16(int(trans_a), int(trans_b), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc,
                               _ptr(bias), int(variant), _ptr(splitk_ws), nbytes, _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "rlstm_gemm_bf16")
    return rc


def rlstm_to_bf16(dst, src, stream=None, check=True) -> int:
    """dst: int16 / uint16 tensor of src.numel() elements."""
    rc = lib().rlstm_to_bf16(_ptr(dst), _ptr(src), src.numel(), _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "rlstm_to_bf16")
    return rc


def rlstm_to_bf16_2d(dst, dst_t, src, R, C, ld, stream=None, check=True) -> int:
    rc = lib().rlstm_to_bf16_2d(_ptr(dst), _ptr(dst_t), _ptr(src), R, C, ld, _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "rlstm_to_bf16_2d")
    return rc


def rlstm_gemm_bf16_mem(trans_a, trans_b, M, N, K, A16, lda, B16, ldb, C, ldc, bias=None, splitk_ws=None,
                        stream=None, check=True, variant=0) -> int:
    nbytes = 0 if splitk_ws is None else splitk_ws.numel() * splitk_ws.element_size()
    rc = lib().rlstm_gemm_bf16_mem(int(trans_a), int(trans_b), M, N, K, _ptr(A16), lda, _ptr(B16), ldb,
                                   _ptr(C), ldc, _ptr(bias), int(variant), _ptr(splitk_ws), nbytes, _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "rlstm_gemm_bf16_mem")
    return rc


def rlstm_test_delay(slow_workgroup: int = -1, ticks: int = 0) -> int:
    return int(lib().rlstm_test_delay(int(slow_workgroup), int(ticks)))


def rlstm_test_hook(mute_workgroup: int = -1, wait_ticks: int = 0) -> int:
    return int(lib().rlstm_test_hook(int(mute_workgroup), int(wait_ticks)))


def rlstm_exchange_floor_bytes(groups: int, members: int, tile_bytes: int) -> int:
    return int(lib().rlstm_exchange_floor_bytes(int(groups), int(members), int(tile_bytes)))


def rlstm_exchange_floor(groups, members, tile_bytes, read_bytes, steps, workspace, stream=None, check=True):
    """Microseconds per step of the bare exchange (best of three runs)."""
    out = ctypes.c_float(0.0)
    nbytes = workspace.numel() * workspace.element_size()
    rc = lib().rlstm_exchange_floor(int(groups), int(members), int(tile_bytes), int(read_bytes), int(steps),
                                    _ptr(workspace), nbytes, ctypes.byref(out), _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "rlstm_exchange_floor")
    return float(out.value) if rc == 0 else rc


def rblstm_plan(desc) -> dict:
    out = (ctypes.c_int32 * 10)()
    rc = int(lib().rblstm_plan(ctypes.byref(desc), out))
    if rc != 0:
        raise RlstmError(rc, "rblstm_plan")
    keys = ("groups", "sequences_per_group", "rows", "units_per_workgroup", "members_fwd", "members_bwd", "Hp", "Hq",
            "bwd_exchanges_per_step", "recurrent_operand_form")
    return dict(zip(keys, [int(v) for v in out]))


def rmdlstm_reserve_bytes(desc) -> int:
    return int(lib().rmdlstm_reserve_bytes(ctypes.byref(desc)))


def rmdlstm_workspace_bytes(desc) -> int:
    return int(lib().rmdlstm_workspace_bytes(ctypes.byref(desc)))


def mdlstm_fwd(desc, x, params, widths, y, reserve, workspace, stream=None, check=True) -> int:
    rc = lib().mdlstm_fwd(ctypes.byref(desc), _ptr(x), _ptr_array(params), _ptr(widths), _ptr(y), _ptr(reserve),
                          _ptr(workspace), _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "mdlstm_fwd")
    return rc


def mdlstm_bwd(desc, x, params, widths, reserve, dy, dx, grads, workspace, stream=None, check=True) -> int:
    rc = lib().mdlstm_bwd(ctypes.byref(desc), _ptr(x), _ptr_array(params), _ptr(widths), _ptr(reserve), _ptr(dy),
                          _ptr(dx), _ptr_array(grads), _ptr(workspace), _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "mdlstm_bwd")
    return rc


def rlstm_chunk_plan(seq_lens, size: int, step: int):
    """Segment table (host): returns numpy int32 arrays (chunk_seq, chunk_start, chunk_len)."""
    import numpy as np
    sl = np.ascontiguousarray(np.asarray(seq_lens), dtype=np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    n = int(lib().rlstm_chunk_plan(sl.ctypes.data_as(i32p), len(sl), int(size), int(step), None, None, None, 0))
    if n < 0:
        raise RlstmError(n, "rlstm_chunk_plan")
    seq, start, ln = (np.empty(n, np.int32) for _ in range(3))
    m = int(lib().rlstm_chunk_plan(sl.ctypes.data_as(i32p), len(sl), int(size), int(step), seq.ctypes.data_as(i32p),
                                   start.ctypes.data_as(i32p), ln.ctypes.data_as(i32p), n))
    assert m == n
    return seq, start, ln


def rlstm_chunk_gather(x, chunk_seq, chunk_start, chunk_len, size: int, xc, ldx: int = 0, stream=None, check=True) -> int:
    T, B = int(x.shape[0]), int(x.shape[1])
    D = int(xc.shape[2])
    rc = lib().rlstm_chunk_gather(_ptr(x), T, B, D, int(ldx), _ptr(chunk_seq), _ptr(chunk_start), _ptr(chunk_len),
                                  int(chunk_seq.numel()), int(size), _ptr(xc), _stream(stream))
    if check and rc != 0:
        raise RlstmError(rc, "rlstm_chunk_gather")
    return rc
