"""GPU parity of every single step of the Tune-mode block (the hot-path rows: fold, forward
conv, input gradient, weight gradient + channel sums, fold-back), each called through its own
C-ABI entry point and compared with the corresponding oracle function."""
import numpy as np
import pytest
import torch

import oracle
from paper_2305_11624_amd import synth
from paper_2305_11624_amd.synth import BlockShape

from helpers import TOL, dims_of, rel_err

pytestmark = pytest.mark.gpu

SHAPES = [
    BlockShape("s_3x3", 3, 64, 20, 18, 72, 3, 1, 1, "bf16", 51),
    BlockShape("s_1x1", 2, 128, 14, 14, 256, 1, 1, 0, "bf16", 52),
    BlockShape("s_3x3_s2", 2, 64, 17, 17, 64, 3, 2, 1, "bf16", 53),
    BlockShape("s_1x1_s2", 2, 64, 16, 16, 128, 1, 2, 0, "bf16", 54),
    BlockShape("s_deep7", 8, 256, 7, 7, 256, 3, 1, 1, "bf16", 55),
    BlockShape("s_f32", 2, 12, 10, 10, 20, 3, 1, 1, "f32", 56),
    BlockShape("s_stem", 2, 3, 40, 40, 64, 7, 2, 3, "bf16", 58),       # 3 input channels: the first-layer kernels
]


def _np(t):
    return None if t is None else t.double().numpy()


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
def test_each_step_against_oracle(shape):
    from paper_2305_11624_amd import binding as B
    inp = synth.make_inputs(shape, bias=True)
    s = shape
    d = dims_of(s)
    desc = B.desc_from_shape(s, eps=inp["eps"])
    dt = B.torch_dtype(desc)
    tol = TOL[s.dtype]
    dev = "cuda"
    x = B.act_to_device(inp["x"], dt)
    W = B.weight_to_device(inp["W"], dt)
    dz = B.act_to_device(inp["dy"], dt)
    b, gamma, beta = (B.vec_to_device(inp[k]) for k in ("b", "gamma", "beta"))
    mean, var = B.vec_to_device(inp["rmean"]), B.vec_to_device(inp["rvar"])
    a = {k: _np(inp[k]) for k in ("x", "W", "b", "gamma", "beta", "rmean", "rvar", "dy")}
    eps = inp["eps"]

    # a1 fold
    w_fprop = torch.full((s.Cout, s.k, s.k, s.Cin), float("nan"), dtype=dt, device=dev)
    w_t = torch.full((s.Cin, s.k, s.k, s.Cout), float("nan"), dtype=dt, device=dev)
    bfold = torch.full((s.Cout,), float("nan"), dtype=torch.float32, device=dev)
    B.convbn_fold(desc, W, b, gamma, beta, mean, var, w_fprop, w_t, bfold)
    Wf, bf = oracle.fold(d, a["W"], a["b"], a["gamma"], a["beta"], a["rmean"], a["rvar"], eps)
    assert rel_err(B.weight_from_device(w_fprop), Wf) <= tol
    assert rel_err(B.folded_from_device(w_t), Wf) <= tol
    assert torch.equal(B.weight_from_device(w_fprop), B.folded_from_device(w_t))   # same values, two orders
    assert rel_err(bfold.double().cpu(), bf) <= 1e-5

    # The later steps are checked with the GPU's own (rounded) w' as the oracle's weight, so
    # that each step's error is its own.
    Wf_gpu = B.weight_from_device(w_fprop).numpy()
    bf_gpu = bfold.double().cpu().numpy()

    def ws(pass_):
        n = B.convbn_conv_workspace_bytes(desc, pass_)
        return torch.empty(max(n, 16), dtype=torch.uint8, device=dev)

    # a2 forward conv
    z = torch.full((s.N, s.Hout, s.Wout, s.Cout), float("nan"), dtype=dt, device=dev)
    B.convbn_conv_fprop(desc, x, w_fprop, bfold, z, ws(B.PASS_FWD))
    assert rel_err(B.act_from_device(z), oracle.conv_fwd(d, a["x"], Wf_gpu, bf_gpu)) <= tol

    # a3 input gradient
    dx = torch.full((s.N, s.Hin, s.Win, s.Cin), float("nan"), dtype=dt, device=dev)
    B.convbn_conv_dgrad(desc, dz, w_t, dx, ws(B.PASS_BWD))
    assert rel_err(B.act_from_device(dx), oracle.conv_dgrad(d, Wf_gpu, a["dy"])) <= tol

    # a4 weight gradient partials and channel-sum partials
    ns, nr = B.convbn_wgrad_parts(desc), B.convbn_rsum_parts(desc)
    P = s.Cout * s.K
    dw_part = torch.full((ns, s.Cout, s.k, s.k, s.Cin), float("nan"), dtype=torch.float32, device=dev)
    r_part = torch.full((nr, s.Cout), float("nan"), dtype=torch.float32, device=dev)
    B.convbn_conv_wgrad(desc, x, dz, dw_part, r_part, ws(B.PASS_BWD))
    dwf = dw_part.double().sum(0).cpu().permute(0, 3, 1, 2).contiguous()
    dwf_ref = oracle.conv_wgrad(d, a["x"], a["dy"])
    assert rel_err(dwf, dwf_ref) <= (1e-4 if s.dtype == "f32" else 1e-5)      # fp32 accumulation of exact products
    r_ref = a["dy"].sum(axis=(0, 2, 3))
    assert rel_err(r_part.double().sum(0).cpu(), r_ref) <= 1e-5

    # a5 fold-back, from the GPU's own partials
    dW = torch.full((s.Cout, s.k, s.k, s.Cin), float("nan"), dtype=dt, device=dev)
    db, dgamma, dbeta = (torch.full((s.Cout,), float("nan"), dtype=torch.float32, device=dev) for _ in range(3))
    B.convbn_fold_back(desc, dw_part, r_part, W, b, gamma, mean, var, dW, db, dgamma, dbeta)
    # reference: the oracle's Tune-mode backward (Table 2 "Tune") on the same inputs; its dw' and r agree with the
    # GPU's summed partials to 1e-5 (checked above), so the fold-back's own error is what is measured here
    tb = oracle.tune_bwd(d, a["x"], a["W"], a["b"], a["gamma"], a["rmean"], a["rvar"], eps, Wf, a["dy"], need_dx=False)
    assert rel_err(B.weight_from_device(dW), tb["dW"]) <= tol
    assert rel_err(dgamma.double().cpu(), tb["dgamma"]) <= 1e-4
    assert rel_err(db.double().cpu(), tb["db"]) <= 1e-4
    assert rel_err(dbeta.double().cpu(), tb["dbeta"]) <= 1e-5
    # dbeta is r itself (Table 2 "Tune": the gradient of beta is the channel sum of dZ)
    assert rel_err(dbeta.double().cpu(), r_part.double().sum(0).cpu().numpy()) <= 1e-6


def test_outputs_are_deterministic():
    """Partial sums are combined in a fixed order: two runs give identical bits."""
    from paper_2305_11624_amd.runner import BlockRun
    inp = synth.make_inputs(BlockShape("det", 4, 64, 28, 28, 64, 3, 1, 1, "bf16", 57))
    r1, r2 = BlockRun(inp, "tune"), BlockRun(inp, "tune")
    r1.step(); r2.step(); r1.step()
    a, b = r1.results(), r2.results()
    for k in ("Z", "dX", "dW", "dgamma", "dbeta"):
        assert torch.equal(a[k], b[k]), k


def test_fold_group_matches_single_folds():
    """Several blocks folded in one launch: bit-identical to one convbn_fold call per block, including an
    identity (re-ordering only) item; shapes the group does not take are refused on the host."""
    from paper_2305_11624_amd import binding as B
    shapes = [BlockShape("g_3x3", 2, 64, 8, 8, 72, 3, 1, 1, "bf16", 81),
              BlockShape("g_1x1", 2, 256, 4, 4, 200, 1, 1, 0, "bf16", 82),
              BlockShape("g_7x7", 1, 8, 16, 16, 64, 7, 2, 3, "bf16", 83),
              BlockShape("g_big", 1, 512, 4, 4, 512, 3, 1, 1, "bf16", 84)]
    blocks, refs = [], []
    for i, sh in enumerate(shapes):
        inp = synth.make_inputs(sh, bias=(i == 0))
        d = B.desc_from_shape(sh, eps=inp["eps"])
        W = B.weight_to_device(inp["W"], torch.bfloat16, "cuda")
        vec = {k: B.vec_to_device(inp[k], "cuda") for k in ("b", "gamma", "beta", "rmean", "rvar")}
        P = sh.Cout * sh.K
        identity = int(i == 2)
        outs = [dict(w_fprop=torch.full((P,), float("nan"), dtype=torch.bfloat16, device="cuda"),
                     w_folded=torch.full((P,), float("nan"), dtype=torch.bfloat16, device="cuda"),
                     b_folded=torch.full((sh.Cout,), float("nan"), dtype=torch.float32, device="cuda")) for _ in range(2)]
        if identity:   # re-ordering only: what the Eval-mode backward asks for
            for o in outs:
                o["w_fprop"] = o["b_folded"] = None
        common = dict(desc=d, W=W, b=vec["b"], gamma=vec["gamma"], beta=vec["beta"], mean=vec["rmean"], var=vec["rvar"],
                      identity=identity)
        blocks.append(dict(common, **outs[0]))
        refs.append(dict(common, **outs[1]))
    n, table, grid = B.convbn_fold_group_plan(blocks)
    B.convbn_fold_group(n, table, grid)
    for r in refs:
        if r["identity"]:   # the re-ordering [Cout][kH][kW][Cin] -> [Cin][kH][kW][Cout], exact
            d = r["desc"]
            r["w_folded"] = r["W"].reshape(d.Cout, d.kH, d.kW, d.Cin).permute(3, 1, 2, 0).contiguous().flatten()
        else:
            B.convbn_fold(r["desc"], r["W"], r["b"], r["gamma"], r["beta"], r["mean"], r["var"], r["w_fprop"],
                          r["w_folded"], r["b_folded"])
    torch.cuda.synchronize()
    for blk, r in zip(blocks, refs):
        for k in ("w_fprop", "w_folded", "b_folded"):
            if r[k] is None:
                continue
            assert not torch.isnan(blk[k].float()).any(), k
            assert torch.equal(blk[k], r[k]), (blk["desc"].Cout, k)
    # a block the group does not take (Cout not a multiple of 8) is refused before anything is launched
    sh = BlockShape("g_odd", 1, 8, 6, 6, 12, 3, 1, 1, "bf16", 85)
    inp = synth.make_inputs(sh)
    d = B.desc_from_shape(sh, eps=inp["eps"])
    bad = dict(desc=d, W=B.weight_to_device(inp["W"], torch.bfloat16, "cuda"), b=None,
               gamma=B.vec_to_device(inp["gamma"], "cuda"), beta=B.vec_to_device(inp["beta"], "cuda"),
               mean=B.vec_to_device(inp["rmean"], "cuda"), var=B.vec_to_device(inp["rvar"], "cuda"),
               w_fprop=None, w_folded=None, b_folded=None)
    assert B.convbn_fold_group_plan([bad], check=False) == B.ERR_UNSUPPORTED


def test_fold_back_group_matches_single_fold_backs():
    """Several blocks' fold-backs in one launch: bit-identical to one convbn_fold_back call per block where that call
    runs its 256-thread kernel (more than 128 output channels, or fewer than 16 partial copies), equal up to the order
    of the partial sums otherwise."""
    from paper_2305_11624_amd import binding as B
    shapes = [BlockShape("fb_3x3", 2, 64, 12, 12, 192, 3, 1, 1, "bf16", 86),
              BlockShape("fb_1x1", 4, 256, 8, 8, 256, 1, 1, 0, "bf16", 87),
              BlockShape("fb_few", 16, 64, 28, 28, 64, 3, 1, 1, "bf16", 88),     # few channels, many partial copies
              BlockShape("fb_s2", 2, 128, 14, 14, 136, 3, 2, 1, "bf16", 89)]
    blocks, singles = [], []
    for i, sh in enumerate(shapes):
        inp = synth.make_inputs(sh, bias=(i == 1))
        d = B.desc_from_shape(sh, eps=inp["eps"])
        dt = torch.bfloat16
        x, W, dz = B.act_to_device(inp["x"], dt), B.weight_to_device(inp["W"], dt), B.act_to_device(inp["dy"], dt)
        vec = {k: B.vec_to_device(inp[k]) for k in ("b", "gamma", "rmean", "rvar")}
        ns, nr = B.convbn_wgrad_parts(d), B.convbn_rsum_parts(d)
        P = sh.Cout * sh.K
        dw_part = torch.empty(ns * P, dtype=torch.float32, device="cuda")
        r_part = torch.empty(nr * sh.Cout, dtype=torch.float32, device="cuda")
        ws = torch.empty(max(16, B.convbn_conv_workspace_bytes(d, B.PASS_BWD)), dtype=torch.uint8, device="cuda")
        B.convbn_conv_wgrad(d, x, dz, dw_part, r_part, ws)
        outs = []
        for _ in range(2):
            outs.append(dict(dW=torch.full((P,), float("nan"), dtype=dt, device="cuda"),
                             db=torch.full((sh.Cout,), float("nan"), device="cuda") if vec["b"] is not None else None,
                             dgamma=torch.full((sh.Cout,), float("nan"), device="cuda"),
                             dbeta=torch.full((sh.Cout,), float("nan"), device="cuda")))
        common = dict(desc=d, dw_part=dw_part, r_part=r_part, W=W, b=vec["b"], gamma=vec["gamma"], mean=vec["rmean"],
                      var=vec["rvar"])
        blocks.append(dict(common, **outs[0]))
        singles.append(dict(common, **outs[1], exact=(sh.Cout > 128 or ns < 16)))
    n, table, grid = B.convbn_fold_back_group_plan(blocks)
    B.convbn_fold_back_group(n, table, grid)
    for r in singles:
        B.convbn_fold_back(r["desc"], r["dw_part"], r["r_part"], r["W"], r["b"], r["gamma"], r["mean"], r["var"], r["dW"],
                           r["db"], r["dgamma"], r["dbeta"])
    torch.cuda.synchronize()
    for g, r in zip(blocks, singles):
        for k in ("dW", "db", "dgamma", "dbeta"):
            if r[k] is None:
                continue
            assert torch.isfinite(g[k].float()).all(), k
            if r["exact"]:
                assert torch.equal(g[k], r[k]), (g["desc"].Cout, k)
            else:
                a, b_ = r[k].double(), g[k].double()
                assert float((a - b_).abs().max() / a.abs().max()) <= (8e-3 if k == "dW" else 1e-5), k


@pytest.mark.parametrize("name", ["c2a", "c2b", "c1"])
def test_scale_in_the_epilogue_forward_matches_the_oracle(name):
    """Forward with the unfolded weight and the BatchNorm scale applied in the convolution's epilogue (the ablation
    of folding first): the same Z as the definition, for a batch small enough for the oracle."""
    import dataclasses
    from paper_2305_11624_amd import binding as B, synth
    from paper_2305_11624_amd.runner import BlockRun
    from helpers import compare, oracle_block
    shape = dataclasses.replace(synth.CONFIGS[name], N={"c2a": 4, "c2b": 64, "c1": 16}[name])
    inp = synth.make_inputs(shape, bias=True, wide_scale=(name == "c2a"))
    ref = oracle_block(inp, need_dx=False)
    r = BlockRun(inp, "tune", poison=True)
    B.convbn_tune_fwd_scale_epilogue(r.desc, r.x, r.W, r.b, r.gamma, r.beta, r.mean, r.var, r.z)
    torch.cuda.synchronize()
    compare({"Z": B.act_from_device(r.z)}, ref, "bf16", keys=("Z",), tag=name + "/scale-epilogue")


def test_scale_in_the_epilogue_forward_refuses_other_shapes():
    from paper_2305_11624_amd import binding as B
    d = B.make_desc(2, 3, 32, 32, 64, 7, 7, 2, 3)     # a first layer (3 input channels) has kernels of its own, without this variant
    x = torch.zeros(1 << 16, device="cuda", dtype=torch.bfloat16)
    v = torch.zeros(64, device="cuda")
    assert B.convbn_tune_fwd_scale_epilogue(d, x, x, None, v, v, v, v, x, check=False) == B.ERR_UNSUPPORTED
