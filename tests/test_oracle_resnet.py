"""Pins for the backbone oracle (oracle/resnet.py): its hand-derived backward through ReLU,
residual adds and the max-pool is checked against reverse-mode autodiff of an independent
forward written with library ops (conv2d, batch_norm in inference mode, relu, max_pool2d)."""
import numpy as np
import torch
import torch.nn.functional as F

from paper_2305_11624_amd import synth
from oracle.resnet import ResNet50Oracle, maxpool_bwd, maxpool_fwd

STAGES = [[f"l{st}.{i}" for i in range(n)] for st, n in enumerate((3, 4, 6, 3), start=1)]


def test_maxpool_matches_library():
    rng = np.random.default_rng(0)
    for shape in [(2, 3, 9, 8), (1, 4, 7, 7), (2, 2, 1, 5)]:
        x = rng.standard_normal(shape)
        y, idx = maxpool_fwd(x)
        tx = torch.tensor(x, requires_grad=True)
        ty = F.max_pool2d(tx, 3, 2, 1)
        assert np.array_equal(y, ty.detach().numpy())
        g = rng.standard_normal(y.shape)
        ty.backward(torch.tensor(g))
        assert np.allclose(maxpool_bwd(g, idx, x.shape), tx.grad.numpy(), rtol=0, atol=1e-13)


def test_backbone_backward_matches_autodiff():
    N, image = 1, 32
    params, tp = {}, {}
    for s in synth.resnet50_blocks(N, image, "f32"):
        p = synth.make_params(s)
        params[s.name] = {k: (v.double().numpy() if hasattr(v, "numpy") else v) for k, v in p.items()}
        tp[s.name] = {k: p[k].double().clone().requires_grad_(k in ("W", "gamma", "beta"))
                      for k in ("W", "gamma", "beta", "rmean", "rvar")}
        tp[s.name]["s"] = s
    g = torch.Generator().manual_seed(5)
    x = torch.randn(N, 3, image, image, generator=g, dtype=torch.float64)
    dout = torch.randn(N, 2048, 1, 1, generator=g, dtype=torch.float64)

    def blk(name, t):
        q = tp[name]
        s = q["s"]
        y = F.conv2d(t, q["W"], None, s.stride, s.pad)
        return F.batch_norm(y, q["rmean"], q["rvar"], q["gamma"], q["beta"], False, 0.0, 1e-5)

    cur = F.max_pool2d(F.relu(blk("stem", x)), 3, 2, 1)
    for names in STAGES:
        for n in names:
            o = blk(n + ".c", F.relu(blk(n + ".b", F.relu(blk(n + ".a", cur)))))
            sc = blk(n + ".ds", cur) if (n + ".ds") in tp else cur
            cur = F.relu(o + sc)
    cur.backward(dout)

    ref = ResNet50Oracle(params, STAGES)
    out = ref.forward(x.numpy())
    assert np.allclose(out, cur.detach().numpy(), rtol=1e-9, atol=1e-9 * np.abs(out).max())
    ref.backward(dout.numpy())
    for name in ("stem", "l1.0.ds", "l1.0.a", "l1.2.b", "l2.0.b", "l2.3.c", "l3.0.ds", "l3.5.a", "l4.0.c", "l4.2.c"):
        for k_ref, k_t in (("dW", "W"), ("dgamma", "gamma"), ("dbeta", "beta")):
            a, b = ref.grads[name][k_ref], tp[name][k_t].grad.numpy()
            assert np.abs(a - b).max() <= 1e-8 * np.abs(b).max(), (name, k_ref)
