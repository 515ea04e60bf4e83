"""Shared pieces of the GPU parity tests: run the oracle on a generated input set and
compare tensors with the benchmark's error measure max|a - ref| / max|ref|."""
import numpy as np

import oracle
from oracle import Dims

TOL = {"f32": 1e-4, "bf16": 2e-2}   # stated tolerances: fp32 1e-4, bf16 2e-2 of max|ref|


def dims_of(s):
    return Dims(s.N, s.Cin, s.Hin, s.Win, s.Cout, s.k, s.k, s.stride, s.stride, s.pad, s.pad)


def _np(t):
    return None if t is None else t.double().numpy()


def oracle_block(inp, need_dx=True):
    """Eval-mode definition in fp64 on the generated (already bf16-rounded) values."""
    d = dims_of(inp["shape"])
    a = {k: _np(inp[k]) for k in ("x", "W", "b", "gamma", "beta", "rmean", "rvar", "dy")}
    Y, Z = oracle.eval_fwd(d, a["x"], a["W"], a["b"], a["gamma"], a["beta"], a["rmean"], a["rvar"],
                           inp["eps"])
    g = oracle.eval_bwd(d, a["x"], a["W"], a["b"], a["gamma"], a["rmean"], a["rvar"], inp["eps"], Y,
                        a["dy"], need_dx=need_dx)
    Wf, bf = oracle.fold(d, a["W"], a["b"], a["gamma"], a["beta"], a["rmean"], a["rvar"], inp["eps"])
    g.update(Y=Y, Z=Z, Wf=Wf, bf=bf)
    return g


def oracle_tconv_block(inp, need_dx=True):
    """Eval-mode definition of the TransposedConv-BN block in fp64 (plus the folded weight of its Tune route)."""
    d = dims_of(inp["shape"])
    a = {k: _np(inp[k]) for k in ("x", "W", "b", "gamma", "beta", "rmean", "rvar", "dy")}
    Y, Z = oracle.teval_fwd(d, a["x"], a["W"], a["b"], a["gamma"], a["beta"], a["rmean"], a["rvar"], inp["eps"])
    g = oracle.teval_bwd(d, a["x"], a["W"], a["b"], a["gamma"], a["rmean"], a["rvar"], inp["eps"], Y, a["dy"],
                         need_dx=need_dx)
    Wf, bf, _ = oracle.ttune_fwd(d, a["x"], a["W"], a["b"], a["gamma"], a["beta"], a["rmean"], a["rvar"],
                                 inp["eps"])
    g.update(Y=Y, Z=Z, Wf=Wf, bf=bf)
    return g


def oracle_dw_block(inp, need_dx=True):
    """Eval-mode definition of the depthwise ConvBN block in fp64 (plus the folded filter of its Tune route)."""
    d = dims_of(inp["shape"])
    a = {k: _np(inp[k]) for k in ("x", "W", "b", "gamma", "beta", "rmean", "rvar", "dy")}
    Y, Z = oracle.dw_eval_fwd(d, a["x"], a["W"], a["b"], a["gamma"], a["beta"], a["rmean"], a["rvar"], inp["eps"])
    g = oracle.dw_eval_bwd(d, a["x"], a["W"], a["b"], a["gamma"], a["rmean"], a["rvar"], inp["eps"], Y, a["dy"],
                           need_dx=need_dx)
    Wf, bf, _ = oracle.dw_tune_fwd(d, a["x"], a["W"], a["b"], a["gamma"], a["beta"], a["rmean"], a["rvar"],
                                   inp["eps"])
    g.update(Y=Y, Z=Z, Wf=Wf, bf=bf)
    return g


def oracle_grouped_block(inp, need_dx=True):
    """Eval-mode definition of the grouped ConvBN block in fp64 (plus the folded weight of its Tune route)."""
    d, G = dims_of(inp["shape"]), inp["groups"]
    a = {k: _np(inp[k]) for k in ("x", "W", "b", "gamma", "beta", "rmean", "rvar", "dy")}
    Y, Z = oracle.g_eval_fwd(d, G, a["x"], a["W"], a["b"], a["gamma"], a["beta"], a["rmean"], a["rvar"], inp["eps"])
    g = oracle.g_eval_bwd(d, G, a["x"], a["W"], a["b"], a["gamma"], a["rmean"], a["rvar"], inp["eps"], Y, a["dy"],
                          need_dx=need_dx)
    Wf, bf, _ = oracle.g_tune_fwd(d, G, a["x"], a["W"], a["b"], a["gamma"], a["beta"], a["rmean"], a["rvar"],
                                  inp["eps"])
    g.update(Y=Y, Z=Z, Wf=Wf, bf=bf)
    return g


def rel_err(got, ref):
    got = got.numpy() if hasattr(got, "numpy") else np.asarray(got)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite values in GPU output"
    denom = np.abs(ref).max()
    if denom == 0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / denom)


def compare(res, ref, dtype, keys=("Z", "dX", "dW", "db", "dgamma", "dbeta"), tol=None, tag=""):
    tol = TOL[dtype] if tol is None else tol
    errs = {}
    for k in keys:
        if ref.get(k) is None:
            assert res.get(k) is None, k
            continue
        errs[k] = rel_err(res[k], ref[k])
    print(tag, {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"{tag}: above tolerance {tol}: {bad}"
    return errs
