"""ctypes/numpy front end of the C oracle.  Marshalling only: every number is
computed in oracle/convbn_oracle.c."""
import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

_lib = None


class _CDims(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("N", "Cin", "Hin", "Win", "Cout", "kH", "kW", "sh", "sw", "ph", "pw")]


@dataclass(frozen=True)
class Dims:
    """Logical problem size (Sec. 3.1): X is [N,Cin,Hin,Win], W is [Cout,Cin,kH,kW]."""
    N: int
    Cin: int
    Hin: int
    Win: int
    Cout: int
    kH: int
    kW: int
    sh: int = 1
    sw: int = 1
    ph: int = 0
    pw: int = 0

    def c(self):
        return _CDims(self.N, self.Cin, self.Hin, self.Win, self.Cout, self.kH, self.kW,
                      self.sh, self.sw, self.ph, self.pw)


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.cbo_hout.restype = C.c_int
        _lib.cbo_wout.restype = C.c_int
        _lib.cbo_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(_load().cbo_num_threads())


def out_hw(d: Dims):
    lib = _load()
    cd = d.c()
    return int(lib.cbo_hout(C.byref(cd))), int(lib.cbo_wout(C.byref(cd)))


def _p(a):
    if a is None:
        return None
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def _f64(a, shape=None):
    if a is None:
        return None
    a = np.ascontiguousarray(np.asarray(a, dtype=np.float64))
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


def _shapes(d: Dims):
    ho, wo = out_hw(d)
    return ((d.N, d.Cin, d.Hin, d.Win), (d.Cout, d.Cin, d.kH, d.kW), (d.N, d.Cout, ho, wo),
            (d.Cout,))


def conv_fwd(d, X, W, b=None):
    xs, ws, ys, vs = _shapes(d)
    X, W, b = _f64(X, xs), _f64(W, ws), _f64(b, vs)
    Y = np.empty(ys)
    cd = d.c()
    _load().cbo_conv_fwd(C.byref(cd), _p(X), _p(W), _p(b), _p(Y))
    return Y


def conv_dgrad(d, W, dY):
    xs, ws, ys, _ = _shapes(d)
    W, dY = _f64(W, ws), _f64(dY, ys)
    dX = np.empty(xs)
    cd = d.c()
    _load().cbo_conv_dgrad(C.byref(cd), _p(W), _p(dY), _p(dX))
    return dX


def conv_wgrad(d, X, dY):
    xs, ws, ys, _ = _shapes(d)
    X, dY = _f64(X, xs), _f64(dY, ys)
    dW = np.empty(ws)
    cd = d.c()
    _load().cbo_conv_wgrad(C.byref(cd), _p(X), _p(dY), _p(dW))
    return dW


def eval_fwd(d, X, W, b, gamma, beta, mu, var, eps):
    """Returns (Y, Z): conv output kept for backward, and the block output."""
    xs, ws, ys, vs = _shapes(d)
    X, W, b = _f64(X, xs), _f64(W, ws), _f64(b, vs)
    gamma, beta, mu, var = (_f64(v, vs) for v in (gamma, beta, mu, var))
    Y, Z = np.empty(ys), np.empty(ys)
    cd = d.c()
    _load().cbo_eval_fwd(C.byref(cd), _p(X), _p(W), _p(b), _p(gamma), _p(beta), _p(mu), _p(var),
                         C.c_double(eps), _p(Y), _p(Z))
    return Y, Z


def eval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G, need_dx=True):
    """Returns dict with dX, dW, db (None if b is None), dgamma, dbeta."""
    xs, ws, ys, vs = _shapes(d)
    X, W, Y, G = _f64(X, xs), _f64(W, ws), _f64(Y, ys), _f64(G, ys)
    gamma, mu, var = (_f64(v, vs) for v in (gamma, mu, var))
    dX = np.empty(xs) if need_dx else None
    dW = np.empty(ws)
    db = np.empty(vs) if b is not None else None
    dgamma, dbeta = np.empty(vs), np.empty(vs)
    scratch = np.empty(ys)
    cd = d.c()
    _load().cbo_eval_bwd(C.byref(cd), _p(X), _p(W), _p(gamma), _p(mu), _p(var), C.c_double(eps),
                         _p(Y), _p(G), _p(scratch), _p(dX), _p(dW), _p(db), _p(dgamma),
                         _p(dbeta))
    return dict(dX=dX, dW=dW, db=db, dgamma=dgamma, dbeta=dbeta)


def fold(d, W, b, gamma, beta, mu, var, eps):
    _, ws, _, vs = _shapes(d)
    W, b = _f64(W, ws), _f64(b, vs)
    gamma, beta, mu, var = (_f64(v, vs) for v in (gamma, beta, mu, var))
    Wf, bf = np.empty(ws), np.empty(vs)
    cd = d.c()
    _load().cbo_fold(C.byref(cd), _p(W), _p(b), _p(gamma), _p(beta), _p(mu), _p(var),
                     C.c_double(eps), _p(Wf), _p(bf))
    return Wf, bf


def tune_fwd(d, X, W, b, gamma, beta, mu, var, eps):
    """Returns (Wf, bf, Z)."""
    xs, ws, ys, vs = _shapes(d)
    X, W, b = _f64(X, xs), _f64(W, ws), _f64(b, vs)
    gamma, beta, mu, var = (_f64(v, vs) for v in (gamma, beta, mu, var))
    Wf, bf, Z = np.empty(ws), np.empty(vs), np.empty(ys)
    cd = d.c()
    _load().cbo_tune_fwd(C.byref(cd), _p(X), _p(W), _p(b), _p(gamma), _p(beta), _p(mu), _p(var),
                         C.c_double(eps), _p(Wf), _p(bf), _p(Z))
    return Wf, bf, Z


def tune_bwd(d, X, W, b, gamma, mu, var, eps, Wf, G, need_dx=True):
    xs, ws, ys, vs = _shapes(d)
    X, W, Wf, G = _f64(X, xs), _f64(W, ws), _f64(Wf, ws), _f64(G, ys)
    b = _f64(b, vs)
    gamma, mu, var = (_f64(v, vs) for v in (gamma, mu, var))
    dX = np.empty(xs) if need_dx else None
    dWf, dW = np.empty(ws), np.empty(ws)
    db = np.empty(vs) if b is not None else None
    dgamma, dbeta = np.empty(vs), np.empty(vs)
    cd = d.c()
    _load().cbo_tune_bwd(C.byref(cd), _p(X), _p(W), _p(b), _p(gamma), _p(mu), _p(var),
                         C.c_double(eps), _p(Wf), _p(G), _p(dX), _p(dWf), _p(dW), _p(db),
                         _p(dgamma), _p(dbeta))
    return dict(dX=dX, dWf=dWf, dW=dW, db=db, dgamma=dgamma, dbeta=dbeta)


# ---- TransposedConv-BN block (Sec. 3.2.1, closing remark).  W is [Cin, Cout, kH, kW]. ----

def tconv_out_hw(d: Dims):
    lib = _load()
    cd = d.c()
    lib.cbo_thout.restype = C.c_int
    lib.cbo_twout.restype = C.c_int
    return int(lib.cbo_thout(C.byref(cd))), int(lib.cbo_twout(C.byref(cd)))


def _tshapes(d: Dims):
    ho, wo = tconv_out_hw(d)
    return ((d.N, d.Cin, d.Hin, d.Win), (d.Cin, d.Cout, d.kH, d.kW), (d.N, d.Cout, ho, wo),
            (d.Cout,))


def tconv_fwd(d, X, W, b=None):
    xs, ws, ys, vs = _tshapes(d)
    X, W, b = _f64(X, xs), _f64(W, ws), _f64(b, vs)
    Y = np.empty(ys)
    cd = d.c()
    _load().cbo_tconv_fwd(C.byref(cd), _p(X), _p(W), _p(b), _p(Y))
    return Y


def tconv_dgrad(d, W, dY):
    xs, ws, ys, _ = _tshapes(d)
    W, dY = _f64(W, ws), _f64(dY, ys)
    dX = np.empty(xs)
    cd = d.c()
    _load().cbo_tconv_dgrad(C.byref(cd), _p(W), _p(dY), _p(dX))
    return dX


def tconv_wgrad(d, X, dY):
    xs, ws, ys, _ = _tshapes(d)
    X, dY = _f64(X, xs), _f64(dY, ys)
    dW = np.empty(ws)
    cd = d.c()
    _load().cbo_tconv_wgrad(C.byref(cd), _p(X), _p(dY), _p(dW))
    return dW


def teval_fwd(d, X, W, b, gamma, beta, mu, var, eps):
    """Returns (Y, Z) of the transposed block in Eval mode."""
    xs, ws, ys, vs = _tshapes(d)
    X, W, b = _f64(X, xs), _f64(W, ws), _f64(b, vs)
    gamma, beta, mu, var = (_f64(v, vs) for v in (gamma, beta, mu, var))
    Y, Z = np.empty(ys), np.empty(ys)
    cd = d.c()
    _load().cbo_teval_fwd(C.byref(cd), _p(X), _p(W), _p(b), _p(gamma), _p(beta), _p(mu), _p(var),
                          C.c_double(eps), _p(Y), _p(Z))
    return Y, Z


def teval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G, need_dx=True):
    xs, ws, ys, vs = _tshapes(d)
    X, W, Y, G = _f64(X, xs), _f64(W, ws), _f64(Y, ys), _f64(G, ys)
    gamma, mu, var = (_f64(v, vs) for v in (gamma, mu, var))
    dX = np.empty(xs) if need_dx else None
    dW = np.empty(ws)
    db = np.empty(vs) if b is not None else None
    dgamma, dbeta = np.empty(vs), np.empty(vs)
    scratch = np.empty(ys)
    cd = d.c()
    _load().cbo_teval_bwd(C.byref(cd), _p(X), _p(W), _p(gamma), _p(mu), _p(var), C.c_double(eps),
                          _p(Y), _p(G), _p(scratch), _p(dX), _p(dW), _p(db), _p(dgamma), _p(dbeta))
    return dict(dX=dX, dW=dW, db=db, dgamma=dgamma, dbeta=dbeta)


def ttune_fwd(d, X, W, b, gamma, beta, mu, var, eps):
    """Returns (Wf, bf, Z) of the transposed block in Tune mode."""
    xs, ws, ys, vs = _tshapes(d)
    X, W, b = _f64(X, xs), _f64(W, ws), _f64(b, vs)
    gamma, beta, mu, var = (_f64(v, vs) for v in (gamma, beta, mu, var))
    Wf, bf, Z = np.empty(ws), np.empty(vs), np.empty(ys)
    cd = d.c()
    _load().cbo_ttune_fwd(C.byref(cd), _p(X), _p(W), _p(b), _p(gamma), _p(beta), _p(mu), _p(var),
                          C.c_double(eps), _p(Wf), _p(bf), _p(Z))
    return Wf, bf, Z


def ttune_bwd(d, X, W, b, gamma, mu, var, eps, Wf, G, need_dx=True):
    xs, ws, ys, vs = _tshapes(d)
    X, W, Wf, G = _f64(X, xs), _f64(W, ws), _f64(Wf, ws), _f64(G, ys)
    b = _f64(b, vs)
    gamma, mu, var = (_f64(v, vs) for v in (gamma, mu, var))
    dX = np.empty(xs) if need_dx else None
    dWf, dW = np.empty(ws), np.empty(ws)
    db = np.empty(vs) if b is not None else None
    dgamma, dbeta = np.empty(vs), np.empty(vs)
    cd = d.c()
    _load().cbo_ttune_bwd(C.byref(cd), _p(X), _p(W), _p(b), _p(gamma), _p(mu), _p(var),
                          C.c_double(eps), _p(Wf), _p(G), _p(dX), _p(dWf), _p(dW), _p(db),
                          _p(dgamma), _p(dbeta))
    return dict(dX=dX, dWf=dWf, dW=dW, db=db, dgamma=dgamma, dbeta=dbeta)


# ---- depthwise ConvBN block (groups = channels).  W is [C, 1, kH, kW]; Dims.Cin == Dims.Cout == C. ----

def _dwshapes(d: Dims):
    assert d.Cin == d.Cout, "depthwise: one filter per channel"
    ho, wo = out_hw(d)
    return ((d.N, d.Cin, d.Hin, d.Win), (d.Cout, 1, d.kH, d.kW), (d.N, d.Cout, ho, wo), (d.Cout,))


def dw_fwd(d, X, W, b=None):
    xs, ws, ys, vs = _dwshapes(d)
    X, W, b = _f64(X, xs), _f64(W, ws), _f64(b, vs)
    Y = np.empty(ys)
    cd = d.c()
    _load().cbo_dw_fwd(C.byref(cd), _p(X), _p(W), _p(b), _p(Y))
    return Y


def dw_dgrad(d, W, dY):
    xs, ws, ys, _ = _dwshapes(d)
    W, dY = _f64(W, ws), _f64(dY, ys)
    dX = np.empty(xs)
    cd = d.c()
    _load().cbo_dw_dgrad(C.byref(cd), _p(W), _p(dY), _p(dX))
    return dX


def dw_wgrad(d, X, dY):
    xs, ws, ys, _ = _dwshapes(d)
    X, dY = _f64(X, xs), _f64(dY, ys)
    dW = np.empty(ws)
    cd = d.c()
    _load().cbo_dw_wgrad(C.byref(cd), _p(X), _p(dY), _p(dW))
    return dW


def dw_eval_fwd(d, X, W, b, gamma, beta, mu, var, eps):
    xs, ws, ys, vs = _dwshapes(d)
    X, W, b = _f64(X, xs), _f64(W, ws), _f64(b, vs)
    gamma, beta, mu, var = (_f64(v, vs) for v in (gamma, beta, mu, var))
    Y, Z = np.empty(ys), np.empty(ys)
    cd = d.c()
    _load().cbo_dw_eval_fwd(C.byref(cd), _p(X), _p(W), _p(b), _p(gamma), _p(beta), _p(mu), _p(var),
                            C.c_double(eps), _p(Y), _p(Z))
    return Y, Z


def dw_eval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G, need_dx=True):
    xs, ws, ys, vs = _dwshapes(d)
    X, W, Y, G = _f64(X, xs), _f64(W, ws), _f64(Y, ys), _f64(G, ys)
    gamma, mu, var = (_f64(v, vs) for v in (gamma, mu, var))
    dX = np.empty(xs) if need_dx else None
    dW = np.empty(ws)
    db = np.empty(vs) if b is not None else None
    dgamma, dbeta = np.empty(vs), np.empty(vs)
    scratch = np.empty(ys)
    cd = d.c()
    _load().cbo_dw_eval_bwd(C.byref(cd), _p(X), _p(W), _p(gamma), _p(mu), _p(var), C.c_double(eps),
                            _p(Y), _p(G), _p(scratch), _p(dX), _p(dW), _p(db), _p(dgamma), _p(dbeta))
    return dict(dX=dX, dW=dW, db=db, dgamma=dgamma, dbeta=dbeta)


def dw_tune_fwd(d, X, W, b, gamma, beta, mu, var, eps):
    xs, ws, ys, vs = _dwshapes(d)
    X, W, b = _f64(X, xs), _f64(W, ws), _f64(b, vs)
    gamma, beta, mu, var = (_f64(v, vs) for v in (gamma, beta, mu, var))
    Wf, bf, Z = np.empty(ws), np.empty(vs), np.empty(ys)
    cd = d.c()
    _load().cbo_dw_tune_fwd(C.byref(cd), _p(X), _p(W), _p(b), _p(gamma), _p(beta), _p(mu), _p(var),
                            C.c_double(eps), _p(Wf), _p(bf), _p(Z))
    return Wf, bf, Z


def dw_tune_bwd(d, X, W, b, gamma, mu, var, eps, Wf, G, need_dx=True):
    xs, ws, ys, vs = _dwshapes(d)
    X, W, Wf, G = _f64(X, xs), _f64(W, ws), _f64(Wf, ws), _f64(G, ys)
    b = _f64(b, vs)
    gamma, mu, var = (_f64(v, vs) for v in (gamma, mu, var))
    dX = np.empty(xs) if need_dx else None
    dWf, dW = np.empty(ws), np.empty(ws)
    db = np.empty(vs) if b is not None else None
    dgamma, dbeta = np.empty(vs), np.empty(vs)
    cd = d.c()
    _load().cbo_dw_tune_bwd(C.byref(cd), _p(X), _p(W), _p(b), _p(gamma), _p(mu), _p(var),
                            C.c_double(eps), _p(Wf), _p(G), _p(dX), _p(dWf), _p(dW), _p(db),
                            _p(dgamma), _p(dbeta))
    return dict(dX=dX, dWf=dWf, dW=dW, db=db, dgamma=dgamma, dbeta=dbeta)


# ---- grouped ConvBN block.  W is [Cout, Cin/groups, kH, kW]; output channel o reads the input channels of
# ---- group o // (Cout/groups). ----

def _gshapes(d: Dims, groups: int):
    assert groups >= 1 and d.Cin % groups == 0 and d.Cout % groups == 0, "groups must divide both channel counts"
    ho, wo = out_hw(d)
    return ((d.N, d.Cin, d.Hin, d.Win), (d.Cout, d.Cin // groups, d.kH, d.kW), (d.N, d.Cout, ho, wo), (d.Cout,))


def g_fwd(d, groups, X, W, b=None):
    xs, ws, ys, vs = _gshapes(d, groups)
    X, W, b = _f64(X, xs), _f64(W, ws), _f64(b, vs)
    Y = np.empty(ys)
    cd = d.c()
    _load().cbo_g_fwd(C.byref(cd), C.c_int(groups), _p(X), _p(W), _p(b), _p(Y))
    return Y


def g_dgrad(d, groups, W, dY):
    xs, ws, ys, _ = _gshapes(d, groups)
    W, dY = _f64(W, ws), _f64(dY, ys)
    dX = np.empty(xs)
    cd = d.c()
    _load().cbo_g_dgrad(C.byref(cd), C.c_int(groups), _p(W), _p(dY), _p(dX))
    return dX


def g_wgrad(d, groups, X, dY):
    xs, ws, ys, _ = _gshapes(d, groups)
    X, dY = _f64(X, xs), _f64(dY, ys)
    dW = np.empty(ws)
    cd = d.c()
    _load().cbo_g_wgrad(C.byref(cd), C.c_int(groups), _p(X), _p(dY), _p(dW))
    return dW


def g_eval_fwd(d, groups, X, W, b, gamma, beta, mu, var, eps):
    xs, ws, ys, vs = _gshapes(d, groups)
    X, W, b = _f64(X, xs), _f64(W, ws), _f64(b, vs)
    gamma, beta, mu, var = (_f64(v, vs) for v in (gamma, beta, mu, var))
    Y, Z = np.empty(ys), np.empty(ys)
    cd = d.c()
    _load().cbo_g_eval_fwd(C.byref(cd), C.c_int(groups), _p(X), _p(W), _p(b), _p(gamma), _p(beta), _p(mu),
                           _p(var), C.c_double(eps), _p(Y), _p(Z))
    return Y, Z


def g_eval_bwd(d, groups, X, W, b, gamma, mu, var, eps, Y, G, need_dx=True):
    xs, ws, ys, vs = _gshapes(d, groups)
    X, W, Y, G = _f64(X, xs), _f64(W, ws), _f64(Y, ys), _f64(G, ys)
    gamma, mu, var = (_f64(v, vs) for v in (gamma, mu, var))
    dX = np.empty(xs) if need_dx else None
    dW = np.empty(ws)
    db = np.empty(vs) if b is not None else None
    dgamma, dbeta = np.empty(vs), np.empty(vs)
    scratch = np.empty(ys)
    cd = d.c()
    _load().cbo_g_eval_bwd(C.byref(cd), C.c_int(groups), _p(X), _p(W), _p(gamma), _p(mu), _p(var),
                           C.c_double(eps), _p(Y), _p(G), _p(scratch), _p(dX), _p(dW), _p(db), _p(dgamma),
                           _p(dbeta))
    return dict(dX=dX, dW=dW, db=db, dgamma=dgamma, dbeta=dbeta)


def g_tune_fwd(d, groups, X, W, b, gamma, beta, mu, var, eps):
    xs, ws, ys, vs = _gshapes(d, groups)
    X, W, b = _f64(X, xs), _f64(W, ws), _f64(b, vs)
    gamma, beta, mu, var = (_f64(v, vs) for v in (gamma, beta, mu, var))
    Wf, bf, Z = np.empty(ws), np.empty(vs), np.empty(ys)
    cd = d.c()
    _load().cbo_g_tune_fwd(C.byref(cd), C.c_int(groups), _p(X), _p(W), _p(b), _p(gamma), _p(beta), _p(mu),
                           _p(var), C.c_double(eps), _p(Wf), _p(bf), _p(Z))
    return Wf, bf, Z


def g_tune_bwd(d, groups, X, W, b, gamma, mu, var, eps, Wf, G, need_dx=True):
    xs, ws, ys, vs = _gshapes(d, groups)
    X, W, Wf, G = _f64(X, xs), _f64(W, ws), _f64(Wf, ws), _f64(G, ys)
    b = _f64(b, vs)
    gamma, mu, var = (_f64(v, vs) for v in (gamma, mu, var))
    dX = np.empty(xs) if need_dx else None
    dWf, dW = np.empty(ws), np.empty(ws)
    db = np.empty(vs) if b is not None else None
    dgamma, dbeta = np.empty(vs), np.empty(vs)
    cd = d.c()
    _load().cbo_g_tune_bwd(C.byref(cd), C.c_int(groups), _p(X), _p(W), _p(b), _p(gamma), _p(mu), _p(var),
                           C.c_double(eps), _p(Wf), _p(G), _p(dX), _p(dWf), _p(dW), _p(db), _p(dgamma),
                           _p(dbeta))
    return dict(dX=dX, dWf=dWf, dW=dW, db=db, dgamma=dgamma, dbeta=dbeta)
