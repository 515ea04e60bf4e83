"""Pins for the TransposedConv-BN part of the CPU oracle (no GPU).  Sec. 3.2.1 only states that the
associative law carries over to transposed convolution; the operator itself is pinned here to things
other than the oracle's own loops: the adjoint identity against the (separately pinned) convolution,
the library's conv_transpose2d + batch_norm with autograd, a closed form for non-overlapping
patches, finite differences, and Tune == Eval (Sec. 3.4.1)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import Dims

TCASES = [
    # N Cin Hin Win Cout kH kW sh sw ph pw      (Cin/Hin/Win describe the input of the transposed block)
    Dims(2, 3, 5, 4, 4, 3, 3, 1, 1, 1, 1),
    Dims(1, 2, 4, 5, 3, 4, 4, 2, 2, 1, 1),      # the usual 2x upsampling block
    Dims(2, 3, 3, 3, 2, 2, 2, 2, 2, 0, 0),      # non-overlapping patches
    Dims(1, 4, 5, 5, 3, 1, 1, 1, 1, 0, 0),      # 1x1
    Dims(1, 2, 4, 3, 3, 3, 3, 2, 2, 0, 0),      # overlapping, no padding
    Dims(1, 2, 3, 4, 2, 3, 2, 2, 1, 1, 0),      # non-square kernel/stride/pad
    Dims(1, 2, 3, 3, 2, 3, 3, 3, 3, 1, 1),      # stride 3
]


def _draw(d, seed, bias=True):
    rng = np.random.default_rng(seed)
    ho, wo = oracle.tconv_out_hw(d)
    X = rng.standard_normal((d.N, d.Cin, d.Hin, d.Win))
    W = rng.standard_normal((d.Cin, d.Cout, d.kH, d.kW)) * 0.5
    b = rng.standard_normal(d.Cout) * 0.3 if bias else None
    gamma = rng.uniform(0.5, 1.5, d.Cout)
    beta = rng.standard_normal(d.Cout) * 0.1
    mu = rng.standard_normal(d.Cout) * 0.1
    var = rng.uniform(0.5, 2.0, d.Cout)
    G = rng.standard_normal((d.N, d.Cout, ho, wo))
    return X, W, b, gamma, beta, mu, var, G


def _t(a, grad=False):
    if a is None:
        return None
    return torch.tensor(a, dtype=torch.float64).requires_grad_(grad)


def _conv_dims(d):
    """The convolution whose adjoint the transposed block is: it maps the block's output back to its input."""
    ho, wo = oracle.tconv_out_hw(d)
    return Dims(d.N, d.Cout, ho, wo, d.Cin, d.kH, d.kW, d.sh, d.sw, d.ph, d.pw)


def test_output_size_rule():
    assert oracle.tconv_out_hw(Dims(1, 1, 7, 7, 1, 4, 4, 2, 2, 1, 1)) == (14, 14)
    assert oracle.tconv_out_hw(Dims(1, 1, 5, 6, 1, 3, 3, 1, 1, 1, 1)) == (5, 6)
    assert oracle.tconv_out_hw(Dims(1, 1, 3, 3, 1, 2, 2, 2, 2, 0, 0)) == (6, 6)


@pytest.mark.parametrize("d", TCASES)
def test_transposed_is_adjoint_of_convolution(d):
    """<tconv(X, W), G> = <X, conv(G, W)> with the same weight array read as [Cout_conv, Cin_conv, kH, kW],
    and the oracle's convolution input gradient is the transposed convolution itself."""
    X, W, _, _, _, _, _, G = _draw(d, 3)
    c = _conv_dims(d)
    assert oracle.out_hw(c) == (d.Hin, d.Win)
    Y = oracle.tconv_fwd(d, X, W)
    back = oracle.conv_fwd(c, G, W)
    np.testing.assert_allclose(np.sum(Y * G), np.sum(X * back), rtol=1e-12)
    np.testing.assert_allclose(Y, oracle.conv_dgrad(c, W, X), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.tconv_dgrad(d, W, G), back, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.tconv_wgrad(d, X, G), oracle.conv_wgrad(c, G, X), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("d", TCASES)
@pytest.mark.parametrize("bias", [True, False])
def test_eval_matches_library_conv_transpose_bn_autograd(d, bias):
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, 11, bias)
    Y, Z = oracle.teval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    g = oracle.teval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G)
    tX, tW, tb, tg, tbeta = _t(X, True), _t(W, True), _t(b, bias), _t(gamma, True), _t(beta, True)
    tY = F.conv_transpose2d(tX, tW, tb, stride=(d.sh, d.sw), padding=(d.ph, d.pw))
    tZ = F.batch_norm(tY, _t(mu), _t(var), tg, tbeta, training=False, eps=eps)
    tZ.backward(_t(G))
    np.testing.assert_allclose(Y, tY.detach().numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(Z, tZ.detach().numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(g["dX"], tX.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g["dW"], tW.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g["dgamma"], tg.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g["dbeta"], tbeta.grad.numpy(), rtol=1e-11, atol=1e-11)
    if bias:
        np.testing.assert_allclose(g["db"], tb.grad.numpy(), rtol=1e-11, atol=1e-11)
    else:
        assert g["db"] is None


def test_non_overlapping_patches_closed_form():
    """Stride = kernel size, no padding: output pixel (s h + i, s w + j) is W[:, :, i, j]^T X[:, h, w]."""
    d = Dims(2, 3, 3, 4, 5, 2, 2, 2, 2, 0, 0)
    rng = np.random.default_rng(5)
    X = rng.standard_normal((2, 3, 3, 4))
    W = rng.standard_normal((3, 5, 2, 2))
    Y = oracle.tconv_fwd(d, X, W)
    ref = np.einsum("coij,nchw->nohiwj", W, X).reshape(2, 5, 6, 8)
    np.testing.assert_allclose(Y, ref, rtol=1e-13, atol=1e-13)


def test_1x1_is_matrix_product():
    d = Dims(2, 4, 3, 5, 6, 1, 1)
    rng = np.random.default_rng(6)
    X = rng.standard_normal((2, 4, 3, 5))
    W = rng.standard_normal((4, 6, 1, 1))
    b = rng.standard_normal(6)
    Y = oracle.tconv_fwd(d, X, W, b)
    ref = np.einsum("co,nchw->nohw", W[:, :, 0, 0], X) + b[None, :, None, None]
    np.testing.assert_allclose(Y, ref, rtol=1e-13, atol=1e-13)


def _J(d, X, W, b, gamma, beta, mu, var, eps, G):
    _, Z = oracle.teval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    return float(np.sum(G * Z))


@pytest.mark.parametrize("d", TCASES[:3])
def test_eval_backward_vs_central_differences(d):
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, 21)
    Y, _ = oracle.teval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    g = oracle.teval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G)
    args = dict(X=X, W=W, b=b, gamma=gamma, beta=beta)
    names = dict(X="dX", W="dW", b="db", gamma="dgamma", beta="dbeta")
    h = 1e-5
    rng = np.random.default_rng(1)
    for key, gname in names.items():
        a = args[key]
        for _ in range(6):
            idx = tuple(int(rng.integers(0, n)) for n in a.shape)
            ap, am = a.copy(), a.copy()
            ap[idx] += h
            am[idx] -= h
            jp = _J(d, **{**args, key: ap}, mu=mu, var=var, eps=eps, G=G)
            jm = _J(d, **{**args, key: am}, mu=mu, var=var, eps=eps, G=G)
            fd = (jp - jm) / (2 * h)
            assert abs(fd - g[gname][idx]) <= 1e-6 * max(1.0, abs(fd)), (key, idx, fd, g[gname][idx])


@pytest.mark.parametrize("d", TCASES)
@pytest.mark.parametrize("bias", [True, False])
def test_tune_equals_eval(d, bias):
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, 31, bias)
    Y, Z = oracle.teval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    ge = oracle.teval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G)
    Wf, bf, Zt = oracle.ttune_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    gt = oracle.ttune_bwd(d, X, W, b, gamma, mu, var, eps, Wf, G)
    np.testing.assert_allclose(Zt, Z, rtol=1e-12, atol=1e-12)
    s = gamma / np.sqrt(var + eps)
    np.testing.assert_allclose(Wf, W * s[None, :, None, None], rtol=1e-14)
    for k in ("dX", "dW", "dgamma", "dbeta"):
        np.testing.assert_allclose(gt[k], ge[k], rtol=1e-11, atol=1e-11)
    if bias:
        np.testing.assert_allclose(gt["db"], ge["db"], rtol=1e-11, atol=1e-11)
