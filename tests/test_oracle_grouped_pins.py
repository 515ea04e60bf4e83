"""Pins for the grouped part of the CPU oracle (no GPU): the dense convolution oracle (separately pinned) with a
block-diagonal weight, its two limits (one group = the dense block, groups = channels = the depthwise block), the
library's grouped conv2d + batch_norm with autograd, finite differences, the adjoint identities and Tune == Eval
(Sec. 3.4.1)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import Dims

GCASES = [
    # (N Cin H W Cout kH kW sh sw ph pw), groups
    (Dims(2, 6, 7, 6, 6, 3, 3, 1, 1, 1, 1), 3),
    (Dims(1, 8, 9, 8, 4, 3, 3, 2, 2, 1, 1), 2),     # Cin/G = 4, Cout/G = 2
    (Dims(2, 4, 8, 8, 12, 5, 5, 1, 1, 2, 2), 4),    # Cin/G = 1, Cout/G = 3 (channel multiplier)
    (Dims(1, 6, 5, 5, 9, 1, 1, 1, 1, 0, 0), 3),
    (Dims(1, 10, 7, 9, 4, 3, 2, 2, 1, 0, 1), 2),
]
IDS = [f"g{g}_{d.Cin}to{d.Cout}_k{d.kH}x{d.kW}_s{d.sh}{d.sw}" for d, g in GCASES]


def _draw(d, groups, seed, bias=True):
    rng = np.random.default_rng(seed)
    ho, wo = oracle.out_hw(d)
    X = rng.standard_normal((d.N, d.Cin, d.Hin, d.Win))
    W = rng.standard_normal((d.Cout, d.Cin // groups, d.kH, d.kW)) * 0.5
    b = rng.standard_normal(d.Cout) * 0.3 if bias else None
    gamma = rng.uniform(0.5, 1.5, d.Cout)
    beta = rng.standard_normal(d.Cout) * 0.1
    mu = rng.standard_normal(d.Cout) * 0.1
    var = rng.uniform(0.5, 2.0, d.Cout)
    G = rng.standard_normal((d.N, d.Cout, ho, wo))
    return X, W, b, gamma, beta, mu, var, G


def _t(a, grad=False):
    return None if a is None else torch.tensor(a, dtype=torch.float64).requires_grad_(grad)


def _dense(d, groups, W):
    cg, og = d.Cin // groups, d.Cout // groups
    Wd = np.zeros((d.Cout, d.Cin, d.kH, d.kW))
    for o in range(d.Cout):
        g = o // og
        Wd[o, g * cg:(g + 1) * cg] = W[o]
    return Wd


def _diag(d, groups, full):
    cg, og = d.Cin // groups, d.Cout // groups
    return np.stack([full[o, (o // og) * cg:(o // og + 1) * cg] for o in range(d.Cout)])


@pytest.mark.parametrize("d,groups", GCASES, ids=IDS)
def test_grouped_is_dense_convolution_with_block_diagonal_weight(d, groups):
    X, W, b, _, _, _, _, G = _draw(d, groups, 2)
    Wd = _dense(d, groups, W)
    np.testing.assert_allclose(oracle.g_fwd(d, groups, X, W, b), oracle.conv_fwd(d, X, Wd, b), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.g_dgrad(d, groups, W, G), oracle.conv_dgrad(d, Wd, G), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.g_wgrad(d, groups, X, G), _diag(d, groups, oracle.conv_wgrad(d, X, G)),
                               rtol=1e-13, atol=1e-13)


def test_one_group_is_the_dense_block_and_all_groups_the_depthwise_block():
    eps = 1e-5
    d = Dims(2, 5, 6, 7, 4, 3, 3, 2, 1, 1, 1)
    X, W, b, gamma, beta, mu, var, G = _draw(d, 1, 8)
    Y, Z = oracle.g_eval_fwd(d, 1, X, W, b, gamma, beta, mu, var, eps)
    Yd, Zd = oracle.eval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    np.testing.assert_array_equal(Z, Zd)
    g, gd = (oracle.g_eval_bwd(d, 1, X, W, b, gamma, mu, var, eps, Y, G),
             oracle.eval_bwd(d, X, W, b, gamma, mu, var, eps, Yd, G))
    for k in ("dX", "dW", "db", "dgamma", "dbeta"):
        np.testing.assert_allclose(g[k], gd[k], rtol=1e-13, atol=1e-13)
    d = Dims(2, 5, 6, 7, 5, 3, 3, 1, 2, 1, 0)
    X, W, b, gamma, beta, mu, var, G = _draw(d, 5, 9)
    Y, Z = oracle.g_eval_fwd(d, 5, X, W, b, gamma, beta, mu, var, eps)
    Yd, Zd = oracle.dw_eval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    np.testing.assert_array_equal(Z, Zd)
    g, gd = (oracle.g_eval_bwd(d, 5, X, W, b, gamma, mu, var, eps, Y, G),
             oracle.dw_eval_bwd(d, X, W, b, gamma, mu, var, eps, Yd, G))
    for k in ("dX", "dW", "db", "dgamma", "dbeta"):
        np.testing.assert_allclose(g[k], gd[k], rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("d,groups", GCASES, ids=IDS)
@pytest.mark.parametrize("bias", [True, False])
def test_eval_matches_library_grouped_conv_bn_autograd(d, groups, bias):
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, groups, 11, bias)
    Y, Z = oracle.g_eval_fwd(d, groups, X, W, b, gamma, beta, mu, var, eps)
    g = oracle.g_eval_bwd(d, groups, X, W, b, gamma, mu, var, eps, Y, G)
    tX, tW, tb, tg, tbeta = _t(X, True), _t(W, True), _t(b, bias), _t(gamma, True), _t(beta, True)
    tY = F.conv2d(tX, tW, tb, stride=(d.sh, d.sw), padding=(d.ph, d.pw), groups=groups)
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


@pytest.mark.parametrize("d,groups", GCASES, ids=IDS)
def test_adjoint_identities(d, groups):
    X, W, _, _, _, _, _, G = _draw(d, groups, 5)
    lhs = np.sum(G * oracle.g_fwd(d, groups, X, W))
    np.testing.assert_allclose(lhs, np.sum(oracle.g_dgrad(d, groups, W, G) * X), rtol=1e-12)
    np.testing.assert_allclose(lhs, np.sum(oracle.g_wgrad(d, groups, X, G) * W), rtol=1e-12)


def test_groups_do_not_mix():
    """An input channel moves only the outputs of its own group; an output's gradient reaches only its group's inputs."""
    d, groups = Dims(1, 6, 5, 5, 9, 3, 3, 1, 1, 1, 1), 3
    X, W, b, _, _, _, _, G = _draw(d, groups, 3)
    Y0 = oracle.g_fwd(d, groups, X, W, b)
    X2 = X.copy()
    X2[:, 2:4] += 1.0                       # group 1's input channels
    diff = np.abs(oracle.g_fwd(d, groups, X2, W, b) - Y0).reshape(d.N, groups, 3, -1).max(axis=(0, 2, 3))
    assert diff[0] == 0 and diff[2] == 0 and diff[1] > 0
    G1 = np.zeros_like(G)
    G1[:, 7] = G[:, 7]                      # an output of group 2
    dX = np.abs(oracle.g_dgrad(d, groups, W, G1)).reshape(d.N, groups, 2, -1).max(axis=(0, 2, 3))
    assert dX[0] == 0 and dX[1] == 0 and dX[2] > 0


@pytest.mark.parametrize("d,groups", GCASES[:3], ids=IDS[:3])
def test_eval_backward_vs_central_differences(d, groups):
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, groups, 21)
    Y, _ = oracle.g_eval_fwd(d, groups, X, W, b, gamma, beta, mu, var, eps)
    g = oracle.g_eval_bwd(d, groups, X, W, b, gamma, mu, var, eps, Y, G)
    args = dict(X=X, W=W, b=b, gamma=gamma, beta=beta)
    names = dict(X="dX", W="dW", b="db", gamma="dgamma", beta="dbeta")
    J = lambda a: float(np.sum(G * oracle.g_eval_fwd(d, groups, a["X"], a["W"], a["b"], a["gamma"], a["beta"], mu, var,
                                                     eps)[1]))
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


@pytest.mark.parametrize("d,groups", GCASES, ids=IDS)
@pytest.mark.parametrize("bias", [True, False])
def test_tune_equals_eval(d, groups, bias):
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, groups, 31, bias)
    Y, Z = oracle.g_eval_fwd(d, groups, X, W, b, gamma, beta, mu, var, eps)
    ge = oracle.g_eval_bwd(d, groups, X, W, b, gamma, mu, var, eps, Y, G)
    Wf, bf, Zt = oracle.g_tune_fwd(d, groups, X, W, b, gamma, beta, mu, var, eps)
    gt = oracle.g_tune_bwd(d, groups, X, W, b, gamma, mu, var, eps, Wf, G)
    np.testing.assert_allclose(Zt, Z, rtol=1e-12, atol=1e-12)
    s = gamma / np.sqrt(var + eps)
    np.testing.assert_allclose(Wf, W * s[:, None, None, None], rtol=1e-14)
    for k in ("dX", "dW", "dgamma", "dbeta"):
        np.testing.assert_allclose(gt[k], ge[k], rtol=1e-11, atol=1e-11)
    if bias:
        np.testing.assert_allclose(gt["db"], ge["db"], rtol=1e-11, atol=1e-11)
