"""ctypes binding of libconvbn.so: same entry-point names as include/convbn.h.

Argument marshalling only -- every step of the block runs in the library's HIP kernels.
PyTorch supplies device memory and the stream.  There is no fallback: if the compiled
library is missing this module raises on first use.
"""
import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libconvbn.so")

OK, ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_LAUNCH = range(6)
F32, BF16 = 0, 1
LAYOUT_NHWC = 0
MODE_TUNE, MODE_EVAL = 0, 1
PASS_FWD, PASS_BWD = 0, 1

EXPORTS = ["convbn_hout", "convbn_wout", "convbn_workspace_bytes", "convbn_saved_bytes",
           "convbn_tune_fwd", "convbn_tune_bwd", "convbn_eval_fwd", "convbn_eval_bwd",
           "convbn_last_error", "convbn_fold", "convbn_conv_fprop", "convbn_conv_dgrad", "convbn_conv_dgrad_masked",
           "convbn_wgrad_parts", "convbn_rsum_parts", "convbn_conv_wgrad", "convbn_fold_back",
           "convbn_conv_workspace_bytes", "convbn_aux_eltwise", "convbn_aux_add_relu_bwd", "convbn_aux_maxpool_fwd",
           "convbn_aux_maxpool_bwd", "convbn_fold_group_table_bytes", "convbn_fold_group_plan",
           "convbn_fold_group", "convbn_tconv_hout", "convbn_tconv_wout", "convbn_tconv_workspace_bytes",
           "convbn_tconv_tune_fwd", "convbn_tconv_tune_bwd", "convbn_tconv_saved_bytes",
           "convbn_tconv_eval_fwd", "convbn_tconv_eval_bwd", "convbn_dw_workspace_bytes", "convbn_dw_saved_bytes",
           "convbn_dw_tune_fwd", "convbn_dw_tune_bwd", "convbn_dw_eval_fwd", "convbn_dw_eval_bwd",
           "convbn_tune_fwd_scale_epilogue", "convbn_grouped_workspace_bytes", "convbn_grouped_saved_bytes",
           "convbn_grouped_tune_fwd", "convbn_grouped_tune_bwd", "convbn_grouped_eval_fwd", "convbn_grouped_eval_bwd",
           "convbn_tune_fwd_static", "convbn_static_workspace_limit", "convbn_fold_back_group_table_bytes",
           "convbn_fold_back_group_plan", "convbn_fold_back_group", "convbn_tune_bwd_is_fused"]


class Desc(C.Structure):
    """Mirror of convbn_desc."""
    _fields_ = [("N", C.c_int32), ("Cin", C.c_int32), ("Hin", C.c_int32), ("Win", C.c_int32),
                ("Cout", C.c_int32), ("kH", C.c_int32), ("kW", C.c_int32),
                ("stride_h", C.c_int32), ("stride_w", C.c_int32),
                ("pad_h", C.c_int32), ("pad_w", C.c_int32),
                ("eps", C.c_float), ("dtype", C.c_int32), ("layout", C.c_int32), ("act", C.c_int32),
                ("add_out", C.c_void_p), ("add_in", C.c_void_p)]


class FoldItem(C.Structure):
    """Mirror of convbn_fold_item."""
    _fields_ = [("desc", C.POINTER(Desc)), ("W", C.c_void_p), ("b", C.c_void_p), ("gamma", C.c_void_p),
                ("beta", C.c_void_p), ("mean", C.c_void_p), ("var", C.c_void_p), ("w_fprop", C.c_void_p),
                ("w_folded", C.c_void_p), ("b_folded", C.c_void_p), ("identity", C.c_int32)]


class FoldBackItem(C.Structure):
    """Mirror of convbn_fold_back_item."""
    _fields_ = [("desc", C.POINTER(Desc)), ("dw_part", C.c_void_p), ("r_part", C.c_void_p), ("W", C.c_void_p),
                ("b", C.c_void_p), ("gamma", C.c_void_p), ("mean", C.c_void_p), ("var", C.c_void_p),
                ("dW", C.c_void_p), ("db", C.c_void_p), ("dgamma", C.c_void_p), ("dbeta", C.c_void_p)]


class ConvBNError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"convbn status {status}: {message}")
        self.status = status


_lib = None


def lib():
    """The loaded library.  Raises if it has not been built (no silent fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2305_11624_amd.build` "
                "(hipcc, gfx950).  This package has no CPU or PyTorch fallback.")
        L = C.CDLL(LIB_PATH)
        vp, fp = C.c_void_p, C.c_void_p
        dp = C.POINTER(Desc)
        L.convbn_hout.restype = C.c_int32
        L.convbn_hout.argtypes = [dp]
        L.convbn_wout.restype = C.c_int32
        L.convbn_wout.argtypes = [dp]
        L.convbn_workspace_bytes.restype = C.c_size_t
        L.convbn_workspace_bytes.argtypes = [dp, C.c_int, C.c_int]
        L.convbn_saved_bytes.restype = C.c_size_t
        L.convbn_saved_bytes.argtypes = [dp, C.c_int, C.c_int]
        L.convbn_last_error.restype = C.c_char_p
        L.convbn_last_error.argtypes = []
        L.convbn_tune_fwd.restype = C.c_int
        L.convbn_tune_fwd.argtypes = [dp, vp, vp, fp, fp, fp, fp, fp, vp, vp, vp, C.c_size_t, vp]
        L.convbn_tune_bwd.restype = C.c_int
        L.convbn_tune_bwd.argtypes = [dp, vp, vp, fp, fp, fp, fp, vp, vp, vp, vp, fp, fp, fp, vp,
                                      C.c_size_t, vp]
        L.convbn_eval_fwd.restype = C.c_int
        L.convbn_eval_fwd.argtypes = [dp, vp, vp, fp, fp, fp, fp, fp, vp, vp, vp, C.c_size_t, vp]
        L.convbn_eval_bwd.restype = C.c_int
        L.convbn_eval_bwd.argtypes = [dp, vp, vp, fp, fp, fp, fp, vp, vp, vp, vp, fp, fp, fp, vp,
                                      C.c_size_t, vp]
        L.convbn_fold.restype = C.c_int
        L.convbn_fold.argtypes = [dp, vp, fp, fp, fp, fp, fp, vp, vp, fp, vp]
        L.convbn_fold_group_table_bytes.restype = C.c_size_t
        L.convbn_fold_group_table_bytes.argtypes = [C.c_int]
        L.convbn_fold_group_plan.restype = C.c_int
        L.convbn_fold_group_plan.argtypes = [C.c_int, C.POINTER(FoldItem), vp, C.c_size_t, C.POINTER(C.c_int)]
        L.convbn_fold_group.restype = C.c_int
        L.convbn_fold_group.argtypes = [C.c_int, vp, C.c_int, vp]
        L.convbn_conv_fprop.restype = C.c_int
        L.convbn_conv_fprop.argtypes = [dp, vp, vp, fp, vp, vp, C.c_size_t, vp]
        L.convbn_conv_dgrad.restype = C.c_int
        L.convbn_conv_dgrad.argtypes = [dp, vp, vp, vp, vp, C.c_size_t, vp]
        L.convbn_conv_dgrad_masked.restype = C.c_int
        L.convbn_conv_dgrad_masked.argtypes = [dp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.convbn_conv_workspace_bytes.restype = C.c_size_t
        L.convbn_conv_workspace_bytes.argtypes = [dp, C.c_int]
        L.convbn_wgrad_parts.restype = C.c_int32
        L.convbn_wgrad_parts.argtypes = [dp]
        L.convbn_rsum_parts.restype = C.c_int32
        L.convbn_rsum_parts.argtypes = [dp]
        L.convbn_conv_wgrad.restype = C.c_int
        L.convbn_conv_wgrad.argtypes = [dp, vp, vp, fp, fp, vp, C.c_size_t, vp]
        L.convbn_fold_back.restype = C.c_int
        L.convbn_fold_back.argtypes = [dp, fp, fp, vp, fp, fp, fp, fp, vp, fp, fp, fp, vp]
        L.convbn_aux_eltwise.restype = C.c_int
        L.convbn_aux_eltwise.argtypes = [C.c_int, C.c_int, vp, vp, C.c_size_t, vp]
        L.convbn_aux_add_relu_bwd.restype = C.c_int
        L.convbn_aux_add_relu_bwd.argtypes = [C.c_int, vp, vp, vp, C.c_size_t, vp]
        L.convbn_aux_maxpool_fwd.restype = C.c_int
        L.convbn_aux_maxpool_fwd.argtypes = [C.c_int, vp, vp, vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp]
        L.convbn_aux_maxpool_bwd.restype = C.c_int
        L.convbn_aux_maxpool_bwd.argtypes = [C.c_int, vp, vp, vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp]
        L.convbn_tconv_hout.restype = C.c_int32
        L.convbn_tconv_hout.argtypes = [dp]
        L.convbn_tconv_wout.restype = C.c_int32
        L.convbn_tconv_wout.argtypes = [dp]
        L.convbn_tconv_workspace_bytes.restype = C.c_size_t
        L.convbn_tconv_workspace_bytes.argtypes = [dp, C.c_int, C.c_int]
        L.convbn_tconv_saved_bytes.restype = C.c_size_t
        L.convbn_tconv_saved_bytes.argtypes = [dp, C.c_int, C.c_int]
        L.convbn_tconv_eval_fwd.restype = C.c_int
        L.convbn_tconv_eval_fwd.argtypes = L.convbn_eval_fwd.argtypes
        L.convbn_tconv_eval_bwd.restype = C.c_int
        L.convbn_tconv_eval_bwd.argtypes = L.convbn_eval_bwd.argtypes
        L.convbn_tconv_tune_fwd.restype = C.c_int
        L.convbn_tconv_tune_fwd.argtypes = L.convbn_tune_fwd.argtypes
        L.convbn_tconv_tune_bwd.restype = C.c_int
        L.convbn_tconv_tune_bwd.argtypes = L.convbn_tune_bwd.argtypes
        for name in ("convbn_dw_workspace_bytes", "convbn_dw_saved_bytes"):
            getattr(L, name).restype = C.c_size_t
            getattr(L, name).argtypes = [dp, C.c_int, C.c_int]
        for name, like in (("convbn_dw_tune_fwd", L.convbn_tune_fwd), ("convbn_dw_tune_bwd", L.convbn_tune_bwd),
                           ("convbn_dw_eval_fwd", L.convbn_eval_fwd), ("convbn_dw_eval_bwd", L.convbn_eval_bwd)):
            getattr(L, name).restype = C.c_int
            getattr(L, name).argtypes = like.argtypes
        for name in ("convbn_grouped_workspace_bytes", "convbn_grouped_saved_bytes"):
            getattr(L, name).restype = C.c_size_t
            getattr(L, name).argtypes = [dp, C.c_int, C.c_int, C.c_int]
        for name, like in (("convbn_grouped_tune_fwd", L.convbn_tune_fwd), ("convbn_grouped_tune_bwd", L.convbn_tune_bwd),
                           ("convbn_grouped_eval_fwd", L.convbn_eval_fwd), ("convbn_grouped_eval_bwd", L.convbn_eval_bwd)):
            getattr(L, name).restype = C.c_int
            getattr(L, name).argtypes = [like.argtypes[0], C.c_int] + list(like.argtypes[1:])
        L.convbn_tune_fwd_scale_epilogue.restype = C.c_int
        L.convbn_tune_fwd_scale_epilogue.argtypes = [dp, vp, vp, fp, fp, fp, fp, fp, vp, vp]
        L.convbn_tune_bwd_is_fused.restype = C.c_int32
        L.convbn_tune_bwd_is_fused.argtypes = [dp]
        L.convbn_fold_back_group_table_bytes.restype = C.c_size_t
        L.convbn_fold_back_group_table_bytes.argtypes = [C.c_int]
        L.convbn_fold_back_group_plan.restype = C.c_int
        L.convbn_fold_back_group_plan.argtypes = [C.c_int, C.POINTER(FoldBackItem), vp, C.c_size_t, C.POINTER(C.c_int)]
        L.convbn_fold_back_group.restype = C.c_int
        L.convbn_fold_back_group.argtypes = [C.c_int, vp, C.c_int, vp]
        L.convbn_tune_fwd_static.restype = C.c_int
        L.convbn_tune_fwd_static.argtypes = [dp, vp, vp, fp, fp, fp, fp, fp, vp, vp, vp]
        L.convbn_static_workspace_limit.restype = C.c_size_t
        L.convbn_static_workspace_limit.argtypes = []
        _lib = L
    return _lib


ACT_RELU_OUT, ACT_RELU_IN, ACT_ADD_OUT, ACT_ADD_IN = 1, 2, 4, 8


def set_addends(desc, add_out=None, add_in=None):
    """Point the descriptor at the tensors of its ACT_ADD_OUT / ACT_ADD_IN bits (device tensors, or None); the caller
    keeps them alive until the calls that read them have been enqueued."""
    desc.add_out = None if add_out is None else add_out.data_ptr()
    desc.add_in = None if add_in is None else add_in.data_ptr()


def make_desc(N, Cin, Hin, Win, Cout, kH, kW, stride=1, pad=0, eps=1e-5, dtype=BF16,
              layout=LAYOUT_NHWC, stride_w=None, pad_w=None, act=0) -> Desc:
    return Desc(N, Cin, Hin, Win, Cout, kH, kW, stride, stride if stride_w is None else stride_w,
                pad, pad if pad_w is None else pad_w, eps, dtype, layout, act)


def desc_from_shape(s, eps=1e-5) -> Desc:
    """Descriptor for a synth.BlockShape."""
    return make_desc(s.N, s.Cin, s.Hin, s.Win, s.Cout, s.k, s.k, s.stride, s.pad, eps,
                     BF16 if s.dtype == "bf16" else F32)


def torch_dtype(desc: Desc):
    return torch.bfloat16 if desc.dtype == BF16 else torch.float32


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    assert t.is_cuda and t.is_contiguous(), "device, dense tensors only"
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return C.c_void_p(stream.cuda_stream)
    return C.c_void_p(int(stream))


def _check(status: int):
    if status != OK:
        raise ConvBNError(status, lib().convbn_last_error().decode())


def convbn_last_error() -> str:
    return lib().convbn_last_error().decode()


def convbn_hout(desc: Desc) -> int:
    return lib().convbn_hout(C.byref(desc))


def convbn_wout(desc: Desc) -> int:
    return lib().convbn_wout(C.byref(desc))


def convbn_workspace_bytes(desc: Desc, mode: int, pass_: int) -> int:
    return lib().convbn_workspace_bytes(C.byref(desc), mode, pass_)


def convbn_saved_bytes(desc: Desc, mode: int, refold: bool = False) -> int:
    return lib().convbn_saved_bytes(C.byref(desc), mode, int(refold))


def _ws(ws):
    if ws is None:
        return None, 0
    return _ptr(ws), ws.numel() * ws.element_size()


def convbn_tune_fwd(desc, x, W, b, gamma, beta, mean, var, z, w_folded, ws, stream=None,
                    check=True):
    p, n = _ws(ws)
    st = lib().convbn_tune_fwd(C.byref(desc), _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(beta),
                               _ptr(mean), _ptr(var), _ptr(z), _ptr(w_folded), p, n,
                               _stream(stream))
    if check:
        _check(st)
    return st


def convbn_tune_fwd_static(desc, x, W, b, gamma, beta, mean, var, z, w_folded, stream=None, check=True):
    st = lib().convbn_tune_fwd_static(C.byref(desc), _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(beta),
                                      _ptr(mean), _ptr(var), _ptr(z), _ptr(w_folded), _stream(stream))
    if check:
        _check(st)
    return st


def convbn_static_workspace_limit() -> int:
    return lib().convbn_static_workspace_limit()


def convbn_tune_bwd(desc, x, W, b, gamma, mean, var, w_folded, dz, dx, dW, db, dgamma, dbeta, ws,
                    stream=None, check=True):
    p, n = _ws(ws)
    st = lib().convbn_tune_bwd(C.byref(desc), _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(mean),
                               _ptr(var), _ptr(w_folded), _ptr(dz), _ptr(dx), _ptr(dW), _ptr(db),
                               _ptr(dgamma), _ptr(dbeta), p, n, _stream(stream))
    if check:
        _check(st)
    return st


def convbn_eval_fwd(desc, x, W, b, gamma, beta, mean, var, z, y_saved, ws, stream=None,
                    check=True):
    p, n = _ws(ws)
    st = lib().convbn_eval_fwd(C.byref(desc), _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(beta),
                               _ptr(mean), _ptr(var), _ptr(z), _ptr(y_saved), p, n,
                               _stream(stream))
    if check:
        _check(st)
    return st


def convbn_eval_bwd(desc, x, W, b, gamma, mean, var, y_saved, dz, dx, dW, db, dgamma, dbeta, ws,
                    stream=None, check=True):
    p, n = _ws(ws)
    st = lib().convbn_eval_bwd(C.byref(desc), _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(mean),
                               _ptr(var), _ptr(y_saved), _ptr(dz), _ptr(dx), _ptr(dW), _ptr(db),
                               _ptr(dgamma), _ptr(dbeta), p, n, _stream(stream))
    if check:
        _check(st)
    return st


def convbn_fold(desc, W, b, gamma, beta, mean, var, w_fprop, w_folded, b_folded, stream=None,
                check=True):
    st = lib().convbn_fold(C.byref(desc), _ptr(W), _ptr(b), _ptr(gamma), _ptr(beta), _ptr(mean),
                           _ptr(var), _ptr(w_fprop), _ptr(w_folded), _ptr(b_folded),
                           _stream(stream))
    if check:
        _check(st)
    return st


def convbn_fold_group_plan(blocks, device="cuda", check=True):
    """blocks: list of dicts with desc, W, b, gamma, beta, mean, var, w_fprop, w_folded, b_folded (tensors
    or None) and identity.  Returns (n, table tensor on the device, grid_blocks)."""
    n = len(blocks)
    items = (FoldItem * n)()
    for it, blk in zip(items, blocks):
        it.desc = C.pointer(blk["desc"])
        for k in ("W", "b", "gamma", "beta", "mean", "var", "w_fprop", "w_folded", "b_folded"):
            t = blk.get(k)
            setattr(it, k, None if t is None else t.data_ptr())
        it.identity = int(blk.get("identity", 0))
    nbytes = lib().convbn_fold_group_table_bytes(n)
    host = (C.c_ubyte * nbytes)()
    grid = C.c_int(0)
    st = lib().convbn_fold_group_plan(n, items, C.cast(host, C.c_void_p), nbytes, C.byref(grid))
    if check:
        _check(st)
    elif st != OK:
        return st
    table = torch.frombuffer(bytearray(host), dtype=torch.uint8).to(device)
    return n, table, grid.value


def convbn_fold_group(n, table, grid_blocks, stream=None, check=True):
    st = lib().convbn_fold_group(n, _ptr(table), grid_blocks, _stream(stream))
    if check:
        _check(st)
    return st


def convbn_tune_bwd_is_fused(desc) -> bool:
    return bool(lib().convbn_tune_bwd_is_fused(C.byref(desc)))


def convbn_fold_back_group_plan(blocks, device="cuda", check=True):
    """blocks: list of dicts with desc, dw_part, r_part, W, b, gamma, mean, var, dW, db, dgamma, dbeta (tensors or
    None).  Returns (n, table tensor on the device, grid_blocks)."""
    n = len(blocks)
    items = (FoldBackItem * n)()
    for it, blk in zip(items, blocks):
        it.desc = C.pointer(blk["desc"])
        for k in ("dw_part", "r_part", "W", "b", "gamma", "mean", "var", "dW", "db", "dgamma", "dbeta"):
            t = blk.get(k)
            setattr(it, k, None if t is None else t.data_ptr())
    nbytes = lib().convbn_fold_back_group_table_bytes(n)
    host = (C.c_ubyte * nbytes)()
    grid = C.c_int(0)
    st = lib().convbn_fold_back_group_plan(n, items, C.cast(host, C.c_void_p), nbytes, C.byref(grid))
    if check:
        _check(st)
    elif st != OK:
        return st
    table = torch.frombuffer(bytearray(host), dtype=torch.uint8).to(device)
    return n, table, grid.value


def convbn_fold_back_group(n, table, grid_blocks, stream=None, check=True):
    st = lib().convbn_fold_back_group(n, _ptr(table), grid_blocks, _stream(stream))
    if check:
        _check(st)
    return st


def convbn_conv_workspace_bytes(desc, pass_: int) -> int:
    return lib().convbn_conv_workspace_bytes(C.byref(desc), pass_)


def convbn_conv_fprop(desc, x, w, bias, z, ws=None, stream=None, check=True):
    p, n = _ws(ws)
    st = lib().convbn_conv_fprop(C.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(z), p, n,
                                 _stream(stream))
    if check:
        _check(st)
    return st


def convbn_conv_dgrad(desc, dz, w_t, dx, ws=None, stream=None, check=True, x_mask=None):
    p, n = _ws(ws)
    if x_mask is not None:
        st = lib().convbn_conv_dgrad_masked(C.byref(desc), _ptr(dz), _ptr(w_t), _ptr(x_mask), _ptr(dx), p, n,
                                            _stream(stream))
    else:
        st = lib().convbn_conv_dgrad(C.byref(desc), _ptr(dz), _ptr(w_t), _ptr(dx), p, n,
                                     _stream(stream))
    if check:
        _check(st)
    return st


def convbn_wgrad_parts(desc) -> int:
    return lib().convbn_wgrad_parts(C.byref(desc))


def convbn_rsum_parts(desc) -> int:
    return lib().convbn_rsum_parts(C.byref(desc))


def convbn_conv_wgrad(desc, x, dz, dw_part, r_part, ws=None, stream=None, check=True):
    p, n = _ws(ws)
    st = lib().convbn_conv_wgrad(C.byref(desc), _ptr(x), _ptr(dz), _ptr(dw_part), _ptr(r_part), p, n,
                                 _stream(stream))
    if check:
        _check(st)
    return st


def convbn_fold_back(desc, dw_part, r_part, W, b, gamma, mean, var, dW, db, dgamma, dbeta,
                     stream=None, check=True):
    st = lib().convbn_fold_back(C.byref(desc), _ptr(dw_part), _ptr(r_part), _ptr(W), _ptr(b),
                                _ptr(gamma), _ptr(mean), _ptr(var), _ptr(dW), _ptr(db),
                                _ptr(dgamma), _ptr(dbeta), _stream(stream))
    if check:
        _check(st)
    return st


OP_RELU, OP_RELU_BWD, OP_ADD_RELU, OP_ADD = range(4)


def _dtype_code(t: torch.Tensor) -> int:
    return BF16 if t.dtype == torch.bfloat16 else F32


def convbn_aux_eltwise(op, a, b=None, stream=None):
    _check(lib().convbn_aux_eltwise(op, _dtype_code(a), _ptr(a), _ptr(b), a.numel(), _stream(stream)))


def convbn_aux_add_relu_bwd(a, b, y, stream=None):
    _check(lib().convbn_aux_add_relu_bwd(_dtype_code(a), _ptr(a), _ptr(b), _ptr(y), a.numel(), _stream(stream)))


def convbn_aux_maxpool_fwd(x, y, idx, stream=None):
    n, h, w, c = x.shape
    _check(lib().convbn_aux_maxpool_fwd(_dtype_code(x), _ptr(x), _ptr(y), _ptr(idx), n, h, w, c,
                                        _stream(stream)))


def convbn_aux_maxpool_bwd(dy, idx, dx, stream=None):
    n, h, w, c = dx.shape
    _check(lib().convbn_aux_maxpool_bwd(_dtype_code(dx), _ptr(dy), _ptr(idx), _ptr(dx), n, h, w, c,
                                        _stream(stream)))


# ---- layout marshalling between logical NCHW host tensors and the library's
def convbn_tconv_hout(desc: Desc) -> int:
    return int(lib().convbn_tconv_hout(C.byref(desc)))


def convbn_tconv_wout(desc: Desc) -> int:
    return int(lib().convbn_tconv_wout(C.byref(desc)))


def convbn_tconv_workspace_bytes(desc: Desc, mode: int, pass_: int) -> int:
    return int(lib().convbn_tconv_workspace_bytes(C.byref(desc), mode, pass_))


def convbn_tconv_saved_bytes(desc: Desc, mode: int, refold: bool = False) -> int:
    return int(lib().convbn_tconv_saved_bytes(C.byref(desc), mode, int(refold)))


def convbn_tconv_eval_fwd(desc, x, W, b, gamma, beta, mean, var, z, y_saved, ws, stream=None, check=True):
    p, n = _ws(ws)
    st = lib().convbn_tconv_eval_fwd(C.byref(desc), _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(beta),
                                     _ptr(mean), _ptr(var), _ptr(z), _ptr(y_saved), p, n, _stream(stream))
    if check:
        _check(st)
    return st


def convbn_tconv_eval_bwd(desc, x, W, b, gamma, mean, var, y_saved, dz, dx, dW, db, dgamma, dbeta, ws,
                          stream=None, check=True):
    p, n = _ws(ws)
    st = lib().convbn_tconv_eval_bwd(C.byref(desc), _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(mean),
                                     _ptr(var), _ptr(y_saved), _ptr(dz), _ptr(dx), _ptr(dW), _ptr(db),
                                     _ptr(dgamma), _ptr(dbeta), p, n, _stream(stream))
    if check:
        _check(st)
    return st


def convbn_tconv_tune_fwd(desc, x, W, b, gamma, beta, mean, var, z, w_folded, ws, stream=None,
                          check=True):
    p, n = _ws(ws)
    st = lib().convbn_tconv_tune_fwd(C.byref(desc), _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(beta),
                                     _ptr(mean), _ptr(var), _ptr(z), _ptr(w_folded), p, n,
                                     _stream(stream))
    if check:
        _check(st)
    return st


def convbn_tconv_tune_bwd(desc, x, W, b, gamma, mean, var, w_folded, dz, dx, dW, db, dgamma, dbeta, ws,
                          stream=None, check=True):
    p, n = _ws(ws)
    st = lib().convbn_tconv_tune_bwd(C.byref(desc), _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(mean),
                                     _ptr(var), _ptr(w_folded), _ptr(dz), _ptr(dx), _ptr(dW), _ptr(db),
                                     _ptr(dgamma), _ptr(dbeta), p, n, _stream(stream))
    if check:
        _check(st)
    return st


def convbn_tune_fwd_scale_epilogue(desc, x, W, b, gamma, beta, mean, var, z, stream=None, check=True):
    st = lib().convbn_tune_fwd_scale_epilogue(C.byref(desc), _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(beta),
                                              _ptr(mean), _ptr(var), _ptr(z), _stream(stream))
    if check:
        _check(st)
    return st


def convbn_dw_workspace_bytes(desc: Desc, mode: int, pass_: int) -> int:
    return int(lib().convbn_dw_workspace_bytes(C.byref(desc), mode, pass_))


def convbn_dw_saved_bytes(desc: Desc, mode: int, refold: bool = False) -> int:
    return int(lib().convbn_dw_saved_bytes(C.byref(desc), mode, int(refold)))


def _block_fwd(fn, desc, x, W, b, gamma, beta, mean, var, z, keep, ws, stream, check):
    p, n = _ws(ws)
    st = fn(C.byref(desc), _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(beta), _ptr(mean), _ptr(var), _ptr(z),
            _ptr(keep), p, n, _stream(stream))
    if check:
        _check(st)
    return st


def _block_bwd(fn, desc, x, W, b, gamma, mean, var, kept, dz, dx, dW, db, dgamma, dbeta, ws, stream, check):
    p, n = _ws(ws)
    st = fn(C.byref(desc), _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(mean), _ptr(var), _ptr(kept), _ptr(dz),
            _ptr(dx), _ptr(dW), _ptr(db), _ptr(dgamma), _ptr(dbeta), p, n, _stream(stream))
    if check:
        _check(st)
    return st


def convbn_dw_tune_fwd(desc, x, W, b, gamma, beta, mean, var, z, w_folded, ws, stream=None, check=True):
    return _block_fwd(lib().convbn_dw_tune_fwd, desc, x, W, b, gamma, beta, mean, var, z, w_folded, ws, stream, check)


def convbn_dw_tune_bwd(desc, x, W, b, gamma, mean, var, w_folded, dz, dx, dW, db, dgamma, dbeta, ws, stream=None,
                       check=True):
    return _block_bwd(lib().convbn_dw_tune_bwd, desc, x, W, b, gamma, mean, var, w_folded, dz, dx, dW, db, dgamma,
                      dbeta, ws, stream, check)


def convbn_dw_eval_fwd(desc, x, W, b, gamma, beta, mean, var, z, y_saved, ws, stream=None, check=True):
    return _block_fwd(lib().convbn_dw_eval_fwd, desc, x, W, b, gamma, beta, mean, var, z, y_saved, ws, stream, check)


def convbn_dw_eval_bwd(desc, x, W, b, gamma, mean, var, y_saved, dz, dx, dW, db, dgamma, dbeta, ws, stream=None,
                       check=True):
    return _block_bwd(lib().convbn_dw_eval_bwd, desc, x, W, b, gamma, mean, var, y_saved, dz, dx, dW, db, dgamma,
                      dbeta, ws, stream, check)


# ---- grouped block: the same calls with the number of groups after the descriptor ----

def convbn_grouped_workspace_bytes(desc: Desc, groups: int, mode: int, pass_: int) -> int:
    return int(lib().convbn_grouped_workspace_bytes(C.byref(desc), groups, mode, pass_))


def convbn_grouped_saved_bytes(desc: Desc, groups: int, mode: int, refold: bool = False) -> int:
    return int(lib().convbn_grouped_saved_bytes(C.byref(desc), groups, mode, int(refold)))


def _gblock_fwd(fn, desc, groups, x, W, b, gamma, beta, mean, var, z, keep, ws, stream, check):
    p, n = _ws(ws)
    st = fn(C.byref(desc), groups, _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(beta), _ptr(mean), _ptr(var), _ptr(z),
            _ptr(keep), p, n, _stream(stream))
    if check:
        _check(st)
    return st


def _gblock_bwd(fn, desc, groups, x, W, b, gamma, mean, var, kept, dz, dx, dW, db, dgamma, dbeta, ws, stream, check):
    p, n = _ws(ws)
    st = fn(C.byref(desc), groups, _ptr(x), _ptr(W), _ptr(b), _ptr(gamma), _ptr(mean), _ptr(var), _ptr(kept), _ptr(dz),
            _ptr(dx), _ptr(dW), _ptr(db), _ptr(dgamma), _ptr(dbeta), p, n, _stream(stream))
    if check:
        _check(st)
    return st


def convbn_grouped_tune_fwd(desc, groups, x, W, b, gamma, beta, mean, var, z, w_folded, ws, stream=None, check=True):
    return _gblock_fwd(lib().convbn_grouped_tune_fwd, desc, groups, x, W, b, gamma, beta, mean, var, z, w_folded, ws,
                       stream, check)


def convbn_grouped_tune_bwd(desc, groups, x, W, b, gamma, mean, var, w_folded, dz, dx, dW, db, dgamma, dbeta, ws,
                            stream=None, check=True):
    return _gblock_bwd(lib().convbn_grouped_tune_bwd, desc, groups, x, W, b, gamma, mean, var, w_folded, dz, dx, dW, db,
                       dgamma, dbeta, ws, stream, check)


def convbn_grouped_eval_fwd(desc, groups, x, W, b, gamma, beta, mean, var, z, y_saved, ws, stream=None, check=True):
    return _gblock_fwd(lib().convbn_grouped_eval_fwd, desc, groups, x, W, b, gamma, beta, mean, var, z, y_saved, ws,
                       stream, check)


def convbn_grouped_eval_bwd(desc, groups, x, W, b, gamma, mean, var, y_saved, dz, dx, dW, db, dgamma, dbeta, ws,
                            stream=None, check=True):
    return _gblock_bwd(lib().convbn_grouped_eval_bwd, desc, groups, x, W, b, gamma, mean, var, y_saved, dz, dx, dW, db,
                       dgamma, dbeta, ws, stream, check)


# ---- channels-last device buffers (pure permutes and casts) -------------------

def act_to_device(t_nchw: torch.Tensor, dtype, device="cuda") -> torch.Tensor:
    """[N,C,H,W] host tensor -> dense [N,H,W,C] device buffer."""
    return t_nchw.permute(0, 2, 3, 1).contiguous().to(device=device, dtype=dtype)


def act_from_device(t_nhwc: torch.Tensor) -> torch.Tensor:
    """[N,H,W,C] device buffer -> logical [N,C,H,W] fp64 host tensor."""
    return t_nhwc.detach().to("cpu", torch.float64).permute(0, 3, 1, 2).contiguous()


def weight_to_device(w_oihw: torch.Tensor, dtype, device="cuda") -> torch.Tensor:
    """[Cout,Cin,kH,kW] -> [Cout,kH,kW,Cin] device buffer."""
    return w_oihw.permute(0, 2, 3, 1).contiguous().to(device=device, dtype=dtype)


def weight_from_device(w_ohwi: torch.Tensor) -> torch.Tensor:
    return w_ohwi.detach().to("cpu", torch.float64).permute(0, 3, 1, 2).contiguous()


def folded_from_device(w_ihwo: torch.Tensor) -> torch.Tensor:
    """w_folded buffer [Cin,kH,kW,Cout] -> logical [Cout,Cin,kH,kW] fp64 host tensor."""
    return w_ihwo.detach().to("cpu", torch.float64).permute(3, 0, 1, 2).contiguous()


def vec_to_device(v: Optional[torch.Tensor], device="cuda"):
    return None if v is None else v.to(device=device, dtype=torch.float32).contiguous()
