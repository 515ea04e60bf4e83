"""Pins for the CPU oracle (no GPU).  Each test fixes the oracle to something other
than itself: a library routine it does not call (torch CPU conv2d / batch_norm with
autograd), a textbook special case (1x1 conv = matrix product, delta kernel,
impulse response), finite differences, the adjoint identities, or the paper's own
identity Tune == Eval (Sec. 3.4.1)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import Dims

CASES = [
    # N Cin Hin Win Cout kH kW sh sw ph pw
    Dims(2, 3, 7, 6, 4, 3, 3, 1, 1, 1, 1),
    Dims(1, 2, 9, 8, 3, 3, 3, 2, 2, 1, 1),     # stride 2, Hin not divisible
    Dims(2, 3, 11, 10, 2, 7, 7, 2, 2, 3, 3),   # stem-like
    Dims(2, 4, 5, 5, 3, 1, 1, 1, 1, 0, 0),     # 1x1
    Dims(1, 2, 8, 8, 2, 1, 1, 2, 2, 0, 0),     # 1x1 stride 2 (shortcut projection)
    Dims(1, 2, 6, 7, 3, 3, 3, 1, 1, 0, 0),     # no padding
    Dims(1, 1, 6, 6, 2, 3, 2, 2, 1, 1, 0),     # non-square kernel/stride/pad
]


def _draw(d, seed, bias=True):
    rng = np.random.default_rng(seed)
    ho, wo = oracle.out_hw(d)
    X = rng.standard_normal((d.N, d.Cin, d.Hin, d.Win))
    W = rng.standard_normal((d.Cout, d.Cin, d.kH, d.kW)) * 0.5
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
    t = torch.tensor(a, dtype=torch.float64)
    return t.requires_grad_(grad)


@pytest.mark.parametrize("d", CASES)
@pytest.mark.parametrize("bias", [True, False])
def test_eval_matches_library_conv_bn_autograd(d, bias):
    """Special case that reduces to library routines: conv2d followed by
    inference-mode batch_norm, gradients by reverse-mode autodiff (fp64, CPU)."""
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, 11, bias)
    Y, Z = oracle.eval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    g = oracle.eval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G)

    tX, tW, tb, tg, tbeta = _t(X, True), _t(W, True), _t(b, bias), _t(gamma, True), _t(beta, True)
    tY = F.conv2d(tX, tW, tb, stride=(d.sh, d.sw), padding=(d.ph, d.pw))
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


def test_conv_1x1_is_matrix_product():
    d = Dims(3, 5, 4, 6, 7, 1, 1)
    rng = np.random.default_rng(0)
    X = rng.standard_normal((3, 5, 4, 6))
    W = rng.standard_normal((7, 5, 1, 1))
    Y = oracle.conv_fwd(d, X, W)
    ref = np.einsum("oc,nchw->nohw", W[:, :, 0, 0], X)
    np.testing.assert_allclose(Y, ref, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("k", [1, 3, 5])
def test_delta_kernel_is_identity(k):
    c = 4
    d = Dims(2, c, 6, 7, c, k, k, 1, 1, k // 2, k // 2)
    W = np.zeros((c, c, k, k))
    for o in range(c):
        W[o, o, k // 2, k // 2] = 1.0
    X = np.random.default_rng(1).standard_normal((2, c, 6, 7))
    np.testing.assert_array_equal(oracle.conv_fwd(d, X, W), X)


def test_impulse_response_is_unflipped_kernel_placed_backwards():
    """A single-pixel input at (h0,w0): cross-correlation gives
    Y[o,ho,wo] = W[o,c0,h0-ho*s+p,w0-wo*s+p] where that index is in range (a true,
    flipped, convolution would place W the other way round)."""
    d = Dims(1, 2, 9, 9, 3, 3, 3, 2, 2, 1, 1)
    rng = np.random.default_rng(2)
    W = rng.standard_normal((3, 2, 3, 3))
    X = np.zeros((1, 2, 9, 9))
    c0, h0, w0 = 1, 4, 5
    X[0, c0, h0, w0] = 1.0
    Y = oracle.conv_fwd(d, X, W)
    ho_n, wo_n = oracle.out_hw(d)
    assert (ho_n, wo_n) == (5, 5)
    ref = np.zeros_like(Y)
    for o in range(3):
        for ho in range(ho_n):
            for wo in range(wo_n):
                i, j = h0 - ho * 2 + 1, w0 - wo * 2 + 1
                if 0 <= i < 3 and 0 <= j < 3:
                    ref[0, o, ho, wo] = W[o, c0, i, j]
    np.testing.assert_array_equal(Y, ref)
    assert np.count_nonzero(Y) > 0


def test_output_size_rule():
    assert oracle.out_hw(Dims(1, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3)) == (112, 112)
    assert oracle.out_hw(Dims(1, 1, 28, 28, 1, 3, 3, 2, 2, 1, 1)) == (14, 14)
    assert oracle.out_hw(Dims(1, 1, 56, 56, 1, 1, 1, 2, 2, 0, 0)) == (28, 28)
    assert oracle.out_hw(Dims(1, 1, 9, 8, 1, 3, 3, 2, 2, 1, 1)) == (5, 4)


def test_bn_identity_and_constant_closed_form():
    d = Dims(2, 3, 5, 5, 4, 3, 3, 1, 1, 1, 1)
    X, W, b, gamma, beta, mu, var, _ = _draw(d, 3)
    eps = 1e-3
    # gamma = sqrt(var+eps), beta = mu = 0  =>  Z == Y up to one rounding
    Y, Z = oracle.eval_fwd(d, X, W, b, np.sqrt(var + eps), 0 * beta, 0 * mu, var, eps)
    np.testing.assert_allclose(Z, Y, rtol=1e-15, atol=0)
    # constant input through a 1x1 conv: Z = gamma (c*sum_ci W + b - mu)/sqrt(var+eps) + beta
    d1 = Dims(1, 3, 4, 4, 4, 1, 1)
    W1 = np.random.default_rng(4).standard_normal((4, 3, 1, 1))
    X1 = np.full((1, 3, 4, 4), 0.75)
    _, Z1 = oracle.eval_fwd(d1, X1, W1, b, gamma, beta, mu, var, eps)
    ref = gamma * (0.75 * W1[:, :, 0, 0].sum(1) + b - mu) / np.sqrt(var + eps) + beta
    np.testing.assert_allclose(Z1, np.broadcast_to(ref[None, :, None, None], Z1.shape), rtol=1e-13)


def _J(d, X, W, b, gamma, beta, mu, var, eps, G):
    _, Z = oracle.eval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    return float((G * Z).sum())


@pytest.mark.parametrize("d", CASES[:4])
def test_eval_backward_vs_central_differences(d):
    """J = <G, Z> is at most bilinear in each argument, so central differences are
    exact up to rounding; every entry of every gradient is checked."""
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, 5)
    Y, _ = oracle.eval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    g = oracle.eval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G)
    args = dict(X=X, W=W, b=b, gamma=gamma, beta=beta)
    names = dict(X="dX", W="dW", b="db", gamma="dgamma", beta="dbeta")
    h = 1e-3
    for key, arr in args.items():
        num = np.zeros_like(arr)
        flat = arr.reshape(-1)
        for idx in range(flat.size):
            old = flat[idx]
            flat[idx] = old + h
            jp = _J(d, args["X"], args["W"], args["b"], args["gamma"], args["beta"], mu, var, eps, G)
            flat[idx] = old - h
            jm = _J(d, args["X"], args["W"], args["b"], args["gamma"], args["beta"], mu, var, eps, G)
            flat[idx] = old
            num.reshape(-1)[idx] = (jp - jm) / (2 * h)
        scale = np.abs(num).max() + 1e-30
        assert np.abs(g[names[key]] - num).max() / scale < 1e-8, key


@pytest.mark.parametrize("d", CASES)
def test_adjoint_identities(d):
    """<G, conv(W,X)> = <dgrad(W,G), X> = <wgrad(X,G), W>: needs no reference."""
    X, W, _, _, _, _, _, G = _draw(d, 6, bias=False)
    lhs = (G * oracle.conv_fwd(d, X, W)).sum()
    a = (oracle.conv_dgrad(d, W, G) * X).sum()
    b = (oracle.conv_wgrad(d, X, G) * W).sum()
    assert abs(lhs - a) <= 1e-11 * abs(lhs) + 1e-11
    assert abs(lhs - b) <= 1e-11 * abs(lhs) + 1e-11


@pytest.mark.parametrize("d", CASES)
@pytest.mark.parametrize("bias", [True, False])
def test_tune_equals_eval(d, bias):
    """Sec. 3.4.1: same function of (w, b, gamma, beta) => same output and the
    same gradients.  Also the Deploy relation dW' = dW / s (Sec. 3.3) and the
    bilinearity identity <dW'[c], W[c]> = sum G_c (W (*) X)_c."""
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, 7, bias)
    Y, Z = oracle.eval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    ge = oracle.eval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G)
    Wf, bf, Zt = oracle.tune_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    gt = oracle.tune_bwd(d, X, W, b, gamma, mu, var, eps, Wf, G)
    np.testing.assert_allclose(Zt, Z, rtol=1e-11, atol=1e-11)
    for k in ("dX", "dW", "dgamma", "dbeta") + (("db",) if bias else ()):
        np.testing.assert_allclose(gt[k], ge[k], rtol=1e-10, atol=1e-10, err_msg=k)
    s = gamma / np.sqrt(var + eps)
    np.testing.assert_allclose(gt["dWf"], ge["dW"] / s[:, None, None, None], rtol=1e-10, atol=1e-11)
    conv_nobias = oracle.conv_fwd(d, X, W)
    lhs = (gt["dWf"] * W).sum(axis=(1, 2, 3))
    rhs = (G * conv_nobias).sum(axis=(0, 2, 3))
    np.testing.assert_allclose(lhs, rhs, rtol=1e-10, atol=1e-10)


def test_tune_handles_zero_and_large_scale():
    """gamma = 0 channels: Tune never divides by gamma (unlike Deploy)."""
    d = CASES[0]
    eps = 1e-5
    X, W, b, gamma, beta, mu, var, G = _draw(d, 8)
    gamma = np.array([0.0, 30.0, 1e-3, 2.0]) * np.sqrt(var + eps)
    Y, Z = oracle.eval_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    ge = oracle.eval_bwd(d, X, W, b, gamma, mu, var, eps, Y, G)
    Wf, _, Zt = oracle.tune_fwd(d, X, W, b, gamma, beta, mu, var, eps)
    gt = oracle.tune_bwd(d, X, W, b, gamma, mu, var, eps, Wf, G)
    np.testing.assert_allclose(Zt, Z, rtol=1e-10, atol=1e-10)
    for k in ("dX", "dW", "db", "dgamma", "dbeta"):
        assert np.isfinite(gt[k]).all()
        np.testing.assert_allclose(gt[k], ge[k], rtol=1e-9, atol=1e-9, err_msg=k)
    assert np.all(gt["dW"][0] == 0) and np.all(ge["dX"] == ge["dX"])


def test_config0_oracle_matches_library():
    """The small benchmark configuration itself, through the shared generator."""
    from paper_2305_11624_amd import synth
    inp = synth.make_inputs(synth.CONFIGS["c0"])
    s = inp["shape"]
    d = Dims(s.N, s.Cin, s.Hin, s.Win, s.Cout, s.k, s.k, s.stride, s.stride, s.pad, s.pad)
    f = lambda t: None if t is None else t.double().numpy()
    Y, Z = oracle.eval_fwd(d, f(inp["x"]), f(inp["W"]), None, f(inp["gamma"]), f(inp["beta"]),
                           f(inp["rmean"]), f(inp["rvar"]), inp["eps"])
    g = oracle.eval_bwd(d, f(inp["x"]), f(inp["W"]), None, f(inp["gamma"]), f(inp["rmean"]),
                        f(inp["rvar"]), inp["eps"], Y, f(inp["dy"]))
    tX = inp["x"].double().requires_grad_(True)
    tW = inp["W"].double().requires_grad_(True)
    tg = inp["gamma"].double().requires_grad_(True)
    tb = inp["beta"].double().requires_grad_(True)
    tZ = F.batch_norm(F.conv2d(tX, tW, None, stride=1, padding=1), inp["rmean"].double(),
                      inp["rvar"].double(), tg, tb, training=False, eps=inp["eps"])
    tZ.backward(inp["dy"].double())
    np.testing.assert_allclose(Z, tZ.detach().numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g["dX"], tX.grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(g["dW"], tW.grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(g["dgamma"], tg.grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(g["dbeta"], tb.grad.numpy(), rtol=1e-10, atol=1e-10)
