"""CPU oracle of the ResNet-50 backbone step used by the end-to-end measurement (test
infrastructure only): 53 ConvBN blocks through the Eval-mode definition of this package, with
ReLU, bottleneck residual adds and a 3x3/2 max-pool written out in numpy, fp64, logical NCHW.
Backward is hand-derived: ReLU passes the gradient where its output is positive, the add copies
it to both branches, the max-pool routes it to the first maximum of each window."""
import numpy as np

from . import oracle as O


def _dims(s):
    return O.Dims(s.N, s.Cin, s.Hin, s.Win, s.Cout, s.k, s.k, s.stride, s.stride, s.pad, s.pad)


def maxpool_fwd(x):
    n, c, h, w = x.shape
    ho, wo = (h - 1) // 2 + 1, (w - 1) // 2 + 1
    xp = np.full((n, c, h + 2, w + 2), -np.inf)
    xp[:, :, 1:h + 1, 1:w + 1] = x
    wins = np.stack([xp[:, :, di:di + 2 * ho:2, dj:dj + 2 * wo:2] for di in range(3) for dj in range(3)], axis=-1)
    idx = wins.argmax(axis=-1)            # first maximum in row-major window order
    return wins.max(axis=-1), idx


def maxpool_gap(x):
    """Smallest gap between the largest and second-largest *positive* entry of any 3x3/2 window
    (a window whose maximum is 0 after a ReLU passes no gradient whichever entry wins)."""
    n, c, h, w = x.shape
    ho, wo = (h - 1) // 2 + 1, (w - 1) // 2 + 1
    xp = np.full((n, c, h + 2, w + 2), -np.inf)
    xp[:, :, 1:h + 1, 1:w + 1] = x
    wins = np.sort(np.stack([xp[:, :, di:di + 2 * ho:2, dj:dj + 2 * wo:2] for di in range(3) for dj in range(3)],
                            axis=-1), axis=-1)
    top, second = wins[..., -1], wins[..., -2]
    gap = np.where(top > 0, top - second, np.inf)
    return gap.min()


def maxpool_bwd(dy, idx, shape):
    n, c, h, w = shape
    dxp = np.zeros((n, c, h + 2, w + 2))
    ho, wo = dy.shape[2], dy.shape[3]
    for k in range(9):
        di, dj = divmod(k, 3)
        dxp[:, :, di:di + 2 * ho:2, dj:dj + 2 * wo:2] += dy * (idx == k)
    return dxp[:, :, 1:h + 1, 1:w + 1]


class ResNet50Oracle:
    """params: dict name -> dict(shape, W, gamma, beta, rmean, rvar, eps) of numpy fp64 arrays."""

    def __init__(self, params, stages):
        self.p, self.stages = params, stages
        self.tape = None
        self.grads = {}
        # ReLU inputs within `tau` (relative to the tensor's largest magnitude) of zero: a lower
        # precision or another summation order can put them on either side, and both are valid
        self.tau = 1e-6
        self.close = []            # (site, index tuple)
        self.pool_margin = np.inf  # smallest winner/runner-up gap of the max-pool, same scale

    def _relu(self, site, v):
        for i in np.argwhere(np.abs(v) < self.tau * np.abs(v).max()):
            self.close.append((site, tuple(int(k) for k in i)))
        return np.maximum(v, 0)

    def _mask(self, site, act, flips):
        m = act > 0
        for s_, i in flips:
            if s_ == site:
                m[i] = ~m[i]
        return m

    def _fwd(self, name, x):
        q = self.p[name]
        y, z = O.eval_fwd(_dims(q["shape"]), x, q["W"], None, q["gamma"], q["beta"], q["rmean"], q["rvar"], q["eps"])
        return y, z

    def _bwd(self, name, x, y, g, need_dx=True):
        q = self.p[name]
        r = O.eval_bwd(_dims(q["shape"]), x, q["W"], None, q["gamma"], q["rmean"], q["rvar"], q["eps"], y, g,
                       need_dx=need_dx)
        self.grads[name] = r
        return r["dX"]

    def forward(self, x):
        t = {}
        y0, z0 = self._fwd("stem", x)
        z0 = self._relu("stem", z0)
        p, idx = maxpool_fwd(z0)
        self.pool_margin = float(maxpool_gap(z0) / np.abs(z0).max())
        t.update(x=x, y0=y0, z0=z0, idx=idx, units=[])
        cur = p
        for names in self.stages:
            for name in names:
                ya, a = self._fwd(name + ".a", cur); a = self._relu(name + ".a", a)
                yb, b = self._fwd(name + ".b", a); b = self._relu(name + ".b", b)
                yc, c = self._fwd(name + ".c", b)
                has_ds = (name + ".ds") in self.p
                yd, sc = self._fwd(name + ".ds", cur) if has_ds else (None, cur)
                out = self._relu(name, c + sc)
                t["units"].append((name, has_ds, cur, ya, a, yb, b, yc, yd, out))
                cur = out
        self.tape = t
        return cur

    def backward(self, dout, flips=()):
        """flips: entries of self.close whose ReLU decision is inverted (the other valid choice)."""
        t = self.tape
        self.grads = {}
        g = dout.copy()
        for name, has_ds, xin, ya, a, yb, b, yc, yd, out in reversed(t["units"]):
            g = g * self._mask(name, out, flips)
            gb = self._bwd(name + ".c", b, yc, g) * self._mask(name + ".b", b, flips)
            ga = self._bwd(name + ".b", a, yb, gb) * self._mask(name + ".a", a, flips)
            gin = self._bwd(name + ".a", xin, ya, ga)
            gin = gin + (self._bwd(name + ".ds", xin, yd, g) if has_ds else g)
            g = gin
        gz0 = maxpool_bwd(g, t["idx"], t["z0"].shape) * self._mask("stem", t["z0"], flips)
        self._bwd("stem", t["x"], t["y0"], gz0, need_dx=False)
