"""Pins for the depthwise part of the CPU oracle (no GPU): the dense convolution oracle (separately pinned) with
a block-diagonal weight, the library's grouped conv2d + batch_norm with autograd, finite differences, the
adjoint identities and Tune == Eval (Sec. 3.4.1)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import Dims

DCASES = [
    # N C H W C kH kW sh sw ph pw
    Dims(2, 5, 7, 6, 5, 3, 3, 1, 1, 1, 1),
    Dims(1, 4, 9, 8, 4, 3, 3, 2, 2, 1, 1),
    Dims(2, 3, 8, 8, 3, 5, 5, 1, 1, 2, 2),
    Dims(1, 6, 5, 5, 6, 1, 1, 1, 1, 0, 0),
    Dims(1, 2, 7, 9, 2, 3, 2, 2, 1, 0, 1),
]


def _draw(d, seed, bias=True):
    rng = np.random.default_rng(seed)
    ho, wo = oracle.out_hw(d)
    X = rng.standard_normal((d.N, d.Cin, d.Hin, d.Win))
    W = rng.standard_normal((d.Cout, 1, d.kH, d.kW)) * 0.5
    b = rng.standard_normal(d.Cout) * 0.3 if bias else None
    gamma = rng.uniform(0.5, 1.5, d.Cout)
    beta = rng.standard_normal(d.Cout) * 0.1
    mu = rng.standard_normal(d.Cout) * 0.1
    var = rng.uniform(0.5, 2.0, d.Cout)
    G = rng.standard_normal((d.N, d.Cout, ho, wo))
    return X, W, b, gamma, beta, mu, var, G


def _t(a, grad=False):
    return None if a is None else torch.tensor(a, dtype=torch.float64).requires_grad_(grad)


def _dense(d, W):
    Wd = np.zeros((d.Cout, d.Cin, d.kH, d.kW))
    for c in range(d.Cout):
        Wd[c, c] = W[c, 0]
    return Wd


@pytest.mark.parametrize("d", DCASES)
def test_depthwise_is_dense_convolution_with_block_diagonal_weight(d):
    X, W, b, _, _, _, _, G = _draw(d, 2)
    Wd = _dense(d, W)
    np.testing.assert_allclose(oracle.dw_fwd(d, X, W, b), oracle.conv_fwd(d, X, Wd, b), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.dw_dgrad(d, W, G), oracle.conv_dgrad(d, Wd, G), rtol=1e-13, atol=1e-13)
    full = oracle.conv_wgrad(d, X, G)
    diag = np.stack([full[c, c] for c in range(d.Cout)])[:, None]
    np.testing.assert_allclose(oracle.dw_wgrad(d, X, G), diag, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("d", DCASES)
@pytest.mark.parametrize("bias", [True, False])
def test_eval_matches_library_grouped_conv_bn_autograd(d, bias):
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, 11, bias)
    Y, Z = oracle.dw_eval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    g = oracle.dw_eval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G)
    tX, tW, tb, tg, tbeta = _t(X, True), _t(W, True), _t(b, bias), _t(gamma, True), _t(beta, True)
    tY = F.conv2d(tX, tW, tb, stride=(d.sh, d.sw), padding=(d.ph, d.pw), groups=d.Cin)
    tZ = F.batch_norm(tY, _t(mu), _t(var), tg, tbeta, training=False, eps=eps)
    tZ.backward(_t(G))
    np.testing.assert_allclose(Y, tY.detach().numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(Z, tZ.detach().numpy(), rtol=1e-12, atol=1e-12)
    for k, t in (("dX", tX), ("dW", tW), ("dgamma", tg), ("dbeta", tbeta)):
        np.testing.assert_allclose(g[k], t.grad.numpy(), rtol=1e-11, atol=1e-11)
    if bias:
        np.testing.assert_allclose(g["db"], tb.grad.numpy(), rtol=1e-11, atol=1e-11)
    else:
        assert g["db"] is None


@pytest.mark.parametrize("d", DCASES)
def test_adjoint_identities(d):
    X, W, _, _, _, _, _, G = _draw(d, 5)
    lhs = np.sum(G * oracle.dw_fwd(d, X, W))
    np.testing.assert_allclose(lhs, np.sum(oracle.dw_dgrad(d, W, G) * X), rtol=1e-12)
    np.testing.assert_allclose(lhs, np.sum(oracle.dw_wgrad(d, X, G) * W), rtol=1e-12)


@pytest.mark.parametrize("d", DCASES[:3])
def test_eval_backward_vs_central_differences(d):
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, 21)
    Y, _ = oracle.dw_eval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    g = oracle.dw_eval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G)
    args = dict(X=X, W=W, b=b, gamma=gamma, beta=beta)
    names = dict(X="dX", W="dW", b="db", gamma="dgamma", beta="dbeta")
    J = lambda a: float(np.sum(G * oracle.dw_eval_fwd(d, a["X"], a["W"], a["b"], a["gamma"], a["beta"], mu, var, eps)[1]))
    h = 1e-5
    rng = np.random.default_rng(1)
    for key, gname in names.items():
        a = args[key]
        for _ in range(6):
            idx = tuple(int(rng.integers(0, n)) for n in a.shape)
            ap, am = a.copy(), a.copy()
            ap[idx] += h
            am[idx] -= h
            fd = (J({**args, key: ap}) - J({**args, key: am})) / (2 * h)
            assert abs(fd - g[gname][idx]) <= 1e-6 * max(1.0, abs(fd)), (key, idx, fd, g[gname][idx])


@pytest.mark.parametrize("d", DCASES)
@pytest.mark.parametrize("bias", [True, False])
def test_tune_equals_eval(d, bias):
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, 31, bias)
    Y, Z = oracle.dw_eval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    ge = oracle.dw_eval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G)
    Wf, bf, Zt = oracle.dw_tune_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    gt = oracle.dw_tune_bwd(d, X, W, b, gamma, mu, var, eps, Wf, G)
    np.testing.assert_allclose(Zt, Z, rtol=1e-12, atol=1e-12)
    s = gamma / np.sqrt(var + eps)
    np.testing.assert_allclose(Wf, W * s[:, None, None, None], rtol=1e-14)
    for k in ("dX", "dW", "dgamma", "dbeta"):
        np.testing.assert_allclose(gt[k], ge[k], rtol=1e-11, atol=1e-11)
    if bias:
        np.testing.assert_allclose(gt["db"], ge["db"], rtol=1e-11, atol=1e-11)
