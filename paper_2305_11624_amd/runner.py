"""Device-buffer holder for one ConvBN block: allocates the library's inputs, outputs and
workspaces through PyTorch and calls the C ABI.  Used by the tests, the smoke check and
the benchmark.  No arithmetic of the method happens here."""
from typing import Dict, Optional

import torch

from . import binding as B


class BlockRun:
    """One block on the GPU in `mode` ("tune" or "eval").

    keep_folded: Tune mode only -- keep w' between forward and backward (the paper's
    choice, Sec. 3.4.2) or fold again in backward.
    """

    def __init__(self, inp: Dict[str, object], mode: str = "tune", keep_folded: bool = True,
                 need_dx: bool = True, device: str = "cuda", poison: bool = False, act: int = 0,
                 add_out=None, add_in=None):
        assert mode in ("tune", "eval")
        s = inp["shape"]
        self.shape, self.mode, self.keep_folded, self.need_dx = s, mode, keep_folded, need_dx
        self.desc = B.desc_from_shape(s, eps=inp["eps"])
        self.desc.act = act   # binding.ACT_* bits: a ReLU and / or a residual sum behind and / or in front of the block
        self.add_out, self.add_in = add_out, add_in   # device tensors of the ACT_ADD_* bits (kept alive here)
        B.set_addends(self.desc, add_out, add_in)
        dt = B.torch_dtype(self.desc)
        self.dt = dt
        self.x = B.act_to_device(inp["x"], dt, device)
        self.W = B.weight_to_device(inp["W"], dt, device)
        self.dz = B.act_to_device(inp["dy"], dt, device)
        self.b = B.vec_to_device(inp["b"], device)
        self.gamma, self.beta = B.vec_to_device(inp["gamma"], device), B.vec_to_device(inp["beta"], device)
        self.mean, self.var = B.vec_to_device(inp["rmean"], device), B.vec_to_device(inp["rvar"], device)

        def out(shape, dtype):
            t = torch.empty(shape, dtype=dtype, device=device)
            if poison:
                t.fill_(float("nan"))
            return t

        self.z = out((s.N, s.Hout, s.Wout, s.Cout), dt)
        self.dx = out((s.N, s.Hin, s.Win, s.Cin), dt) if need_dx else None
        self.dW = out((s.Cout, s.k, s.k, s.Cin), dt)
        self.db = out((s.Cout,), torch.float32) if self.b is not None else None
        self.dgamma, self.dbeta = out((s.Cout,), torch.float32), out((s.Cout,), torch.float32)
        m = B.MODE_TUNE if mode == "tune" else B.MODE_EVAL
        self.ws_fwd = self._ws(B.convbn_workspace_bytes(self.desc, m, B.PASS_FWD), device)
        self.ws_bwd = self._ws(B.convbn_workspace_bytes(self.desc, m, B.PASS_BWD), device)
        self.w_folded = None
        self.y_saved = None
        if mode == "tune" and keep_folded:
            self.w_folded = out((s.Cin, s.k, s.k, s.Cout), dt)
        if mode == "eval":
            self.y_saved = out((s.N, s.Hout, s.Wout, s.Cout), dt)

    @staticmethod
    def _ws(nbytes: int, device) -> Optional[torch.Tensor]:
        return torch.empty(nbytes, dtype=torch.uint8, device=device) if nbytes else None

    def saved_bytes(self) -> int:
        m = B.MODE_TUNE if self.mode == "tune" else B.MODE_EVAL
        return B.convbn_saved_bytes(self.desc, m, not self.keep_folded)

    def forward(self, stream=None):
        if self.mode == "tune":
            B.convbn_tune_fwd(self.desc, self.x, self.W, self.b, self.gamma, self.beta, self.mean,
                              self.var, self.z, self.w_folded, self.ws_fwd, stream)
        else:
            B.convbn_eval_fwd(self.desc, self.x, self.W, self.b, self.gamma, self.beta, self.mean,
                              self.var, self.z, self.y_saved, self.ws_fwd, stream)

    def backward(self, stream=None):
        if self.mode == "tune":
            B.convbn_tune_bwd(self.desc, self.x, self.W, self.b, self.gamma, self.mean, self.var,
                              self.w_folded, self.dz, self.dx, self.dW, self.db, self.dgamma,
                              self.dbeta, self.ws_bwd, stream)
        else:
            B.convbn_eval_bwd(self.desc, self.x, self.W, self.b, self.gamma, self.mean, self.var,
                              self.y_saved, self.dz, self.dx, self.dW, self.db, self.dgamma,
                              self.dbeta, self.ws_bwd, stream)

    def step(self, stream=None):
        self.forward(stream)
        self.backward(stream)

    def results(self) -> Dict[str, Optional[torch.Tensor]]:
        """Outputs as logical-NCHW fp64 host tensors."""
        torch.cuda.synchronize()
        f = lambda t: None if t is None else t.detach().to("cpu", torch.float64)
        return dict(
            Z=B.act_from_device(self.z),
            dX=B.act_from_device(self.dx) if self.dx is not None else None,
            dW=B.weight_from_device(self.dW),
            db=f(self.db), dgamma=f(self.dgamma), dbeta=f(self.dbeta),
            Wf=B.folded_from_device(self.w_folded) if self.w_folded is not None else None,
            Y=B.act_from_device(self.y_saved) if self.y_saved is not None else None)


class TconvRun:
    """One TransposedConv-BN block on the GPU in `mode` ("tune" or "eval"; inputs from synth.make_tconv_inputs)."""

    def __init__(self, inp: Dict[str, object], mode: str = "tune", keep_folded: bool = True, need_dx: bool = True,
                 params: bool = True, device: str = "cuda", poison: bool = False):
        assert mode in ("tune", "eval")
        s = inp["shape"]
        self.shape, self.mode, self.keep_folded = s, mode, keep_folded
        self.desc = B.desc_from_shape(s, eps=inp["eps"])
        dt = B.torch_dtype(self.desc)
        self.dt = dt
        ho, wo = B.convbn_tconv_hout(self.desc), B.convbn_tconv_wout(self.desc)
        self.x = B.act_to_device(inp["x"], dt, device)
        self.W = B.weight_to_device(inp["W"], dt, device)        # [Cin, Cout, k, k] -> [Cin][k][k][Cout]
        self.dz = B.act_to_device(inp["dy"], dt, device)
        self.b = B.vec_to_device(inp["b"], device)
        self.gamma, self.beta = B.vec_to_device(inp["gamma"], device), B.vec_to_device(inp["beta"], device)
        self.mean, self.var = B.vec_to_device(inp["rmean"], device), B.vec_to_device(inp["rvar"], device)

        def out(shape, dtype):
            t = torch.empty(shape, dtype=dtype, device=device)
            if poison:
                t.fill_(float("nan"))
            return t

        self.z = out((s.N, ho, wo, s.Cout), dt)
        self.dx = out((s.N, s.Hin, s.Win, s.Cin), dt) if need_dx else None
        self.dW = out((s.Cin, s.k, s.k, s.Cout), dt) if params else None
        self.db = out((s.Cout,), torch.float32) if (self.b is not None and params) else None
        self.dgamma = out((s.Cout,), torch.float32) if params else None
        self.dbeta = out((s.Cout,), torch.float32) if params else None
        m = B.MODE_TUNE if mode == "tune" else B.MODE_EVAL
        self.ws_fwd = BlockRun._ws(B.convbn_tconv_workspace_bytes(self.desc, m, B.PASS_FWD), device)
        self.ws_bwd = BlockRun._ws(B.convbn_tconv_workspace_bytes(self.desc, m, B.PASS_BWD), device)
        self.w_folded = out((s.Cin, s.k, s.k, s.Cout), dt) if (keep_folded and mode == "tune") else None
        self.y_saved = out((s.N, ho, wo, s.Cout), dt) if mode == "eval" else None

    def saved_bytes(self) -> int:
        m = B.MODE_TUNE if self.mode == "tune" else B.MODE_EVAL
        return B.convbn_tconv_saved_bytes(self.desc, m, not self.keep_folded)

    def forward(self, stream=None):
        if self.mode == "tune":
            B.convbn_tconv_tune_fwd(self.desc, self.x, self.W, self.b, self.gamma, self.beta, self.mean, self.var,
                                    self.z, self.w_folded, self.ws_fwd, stream)
        else:
            B.convbn_tconv_eval_fwd(self.desc, self.x, self.W, self.b, self.gamma, self.beta, self.mean, self.var,
                                    self.z, self.y_saved, self.ws_fwd, stream)

    def backward(self, stream=None):
        if self.mode == "tune":
            B.convbn_tconv_tune_bwd(self.desc, self.x, self.W, self.b, self.gamma, self.mean, self.var,
                                    self.w_folded, self.dz, self.dx, self.dW, self.db, self.dgamma, self.dbeta,
                                    self.ws_bwd, stream)
        else:
            B.convbn_tconv_eval_bwd(self.desc, self.x, self.W, self.b, self.gamma, self.mean, self.var,
                                    self.y_saved, self.dz, self.dx, self.dW, self.db, self.dgamma, self.dbeta,
                                    self.ws_bwd, stream)

    def step(self, stream=None):
        self.forward(stream)
        self.backward(stream)

    def results(self) -> Dict[str, Optional[torch.Tensor]]:
        torch.cuda.synchronize()
        f = lambda t: None if t is None else t.detach().to("cpu", torch.float64)
        return dict(
            Z=B.act_from_device(self.z),
            dX=B.act_from_device(self.dx) if self.dx is not None else None,
            dW=B.weight_from_device(self.dW) if self.dW is not None else None,
            db=f(self.db), dgamma=f(self.dgamma), dbeta=f(self.dbeta),
            Wf=B.weight_from_device(self.w_folded) if self.w_folded is not None else None,
            Y=B.act_from_device(self.y_saved) if self.y_saved is not None else None)


class DepthwiseRun:
    """One depthwise ConvBN block on the GPU in `mode` ("tune" or "eval"; inputs from synth.make_dw_inputs)."""

    def __init__(self, inp: Dict[str, object], mode: str = "tune", keep_folded: bool = True, need_dx: bool = True,
                 params: bool = True, device: str = "cuda", poison: bool = False):
        assert mode in ("tune", "eval")
        s = inp["shape"]
        self.shape, self.mode, self.keep_folded = s, mode, keep_folded
        self.desc = B.desc_from_shape(s, eps=inp["eps"])
        dt = B.torch_dtype(self.desc)
        self.dt = dt
        self.x = B.act_to_device(inp["x"], dt, device)
        self.W = inp["W"].reshape(s.Cout, s.k, s.k).contiguous().to(device=device, dtype=dt)   # [C, 1, k, k] -> [C][k][k]
        self.dz = B.act_to_device(inp["dy"], dt, device)
        self.b = B.vec_to_device(inp["b"], device)
        self.gamma, self.beta = B.vec_to_device(inp["gamma"], device), B.vec_to_device(inp["beta"], device)
        self.mean, self.var = B.vec_to_device(inp["rmean"], device), B.vec_to_device(inp["rvar"], device)

        def out(shape, dtype):
            t = torch.empty(shape, dtype=dtype, device=device)
            if poison:
                t.fill_(float("nan"))
            return t

        self.z = out((s.N, s.Hout, s.Wout, s.Cout), dt)
        self.dx = out((s.N, s.Hin, s.Win, s.Cin), dt) if need_dx else None
        self.dW = out((s.Cout, s.k, s.k), dt) if params else None
        self.db = out((s.Cout,), torch.float32) if (self.b is not None and params) else None
        self.dgamma = out((s.Cout,), torch.float32) if params else None
        self.dbeta = out((s.Cout,), torch.float32) if params else None
        m = B.MODE_TUNE if mode == "tune" else B.MODE_EVAL
        self.ws_fwd = BlockRun._ws(B.convbn_dw_workspace_bytes(self.desc, m, B.PASS_FWD), device)
        self.ws_bwd = BlockRun._ws(B.convbn_dw_workspace_bytes(self.desc, m, B.PASS_BWD), device)
        self.w_folded = out((s.k, s.k, s.Cout), dt) if (keep_folded and mode == "tune") else None
        self.y_saved = out((s.N, s.Hout, s.Wout, s.Cout), dt) if mode == "eval" else None

    def saved_bytes(self) -> int:
        m = B.MODE_TUNE if self.mode == "tune" else B.MODE_EVAL
        return B.convbn_dw_saved_bytes(self.desc, m, not self.keep_folded)

    def forward(self, stream=None):
        if self.mode == "tune":
            B.convbn_dw_tune_fwd(self.desc, self.x, self.W, self.b, self.gamma, self.beta, self.mean, self.var,
                                 self.z, self.w_folded, self.ws_fwd, stream)
        else:
            B.convbn_dw_eval_fwd(self.desc, self.x, self.W, self.b, self.gamma, self.beta, self.mean, self.var,
                                 self.z, self.y_saved, self.ws_fwd, stream)

    def backward(self, stream=None):
        if self.mode == "tune":
            B.convbn_dw_tune_bwd(self.desc, self.x, self.W, self.b, self.gamma, self.mean, self.var, self.w_folded,
                                 self.dz, self.dx, self.dW, self.db, self.dgamma, self.dbeta, self.ws_bwd, stream)
        else:
            B.convbn_dw_eval_bwd(self.desc, self.x, self.W, self.b, self.gamma, self.mean, self.var, self.y_saved,
                                 self.dz, self.dx, self.dW, self.db, self.dgamma, self.dbeta, self.ws_bwd, stream)

    def step(self, stream=None):
        self.forward(stream)
        self.backward(stream)

    def results(self) -> Dict[str, Optional[torch.Tensor]]:
        torch.cuda.synchronize()
        s = self.shape
        f = lambda t: None if t is None else t.detach().to("cpu", torch.float64)
        return dict(
            Z=B.act_from_device(self.z),
            dX=B.act_from_device(self.dx) if self.dx is not None else None,
            dW=f(self.dW).reshape(s.Cout, 1, s.k, s.k) if self.dW is not None else None,
            db=f(self.db), dgamma=f(self.dgamma), dbeta=f(self.dbeta),
            Wf=f(self.w_folded).permute(2, 0, 1).reshape(s.Cout, 1, s.k, s.k).contiguous()
            if self.w_folded is not None else None,
            Y=B.act_from_device(self.y_saved) if self.y_saved is not None else None)


class GroupedRun:
    """One grouped ConvBN block on the GPU in `mode` ("tune" or "eval"; inputs from synth.make_grouped_inputs)."""

    def __init__(self, inp: Dict[str, object], mode: str = "tune", keep_folded: bool = True, need_dx: bool = True,
                 params: bool = True, device: str = "cuda", poison: bool = False):
        assert mode in ("tune", "eval")
        s = inp["shape"]
        self.groups = G = int(inp["groups"])
        self.shape, self.mode, self.keep_folded = s, mode, keep_folded
        self.desc = B.desc_from_shape(s, eps=inp["eps"])
        dt = B.torch_dtype(self.desc)
        self.dt = dt
        cg = s.Cin // G
        self.x = B.act_to_device(inp["x"], dt, device)
        self.W = B.weight_to_device(inp["W"], dt, device)              # [Cout, cg, k, k] -> [Cout][k][k][cg]
        self.dz = B.act_to_device(inp["dy"], dt, device)
        self.b = B.vec_to_device(inp["b"], device)
        self.gamma, self.beta = B.vec_to_device(inp["gamma"], device), B.vec_to_device(inp["beta"], device)
        self.mean, self.var = B.vec_to_device(inp["rmean"], device), B.vec_to_device(inp["rvar"], device)

        def out(shape, dtype):
            t = torch.empty(shape, dtype=dtype, device=device)
            if poison:
                t.fill_(float("nan"))
            return t

        self.z = out((s.N, s.Hout, s.Wout, s.Cout), dt)
        self.dx = out((s.N, s.Hin, s.Win, s.Cin), dt) if need_dx else None
        self.dW = out((s.Cout, s.k, s.k, cg), dt) if params else None
        self.db = out((s.Cout,), torch.float32) if (self.b is not None and params) else None
        self.dgamma = out((s.Cout,), torch.float32) if params else None
        self.dbeta = out((s.Cout,), torch.float32) if params else None
        m = B.MODE_TUNE if mode == "tune" else B.MODE_EVAL
        self.ws_fwd = BlockRun._ws(B.convbn_grouped_workspace_bytes(self.desc, G, m, B.PASS_FWD), device)
        self.ws_bwd = BlockRun._ws(B.convbn_grouped_workspace_bytes(self.desc, G, m, B.PASS_BWD), device)
        self.w_folded = out((cg, s.k, s.k, s.Cout), dt) if (keep_folded and mode == "tune") else None
        self.y_saved = out((s.N, s.Hout, s.Wout, s.Cout), dt) if mode == "eval" else None

    def saved_bytes(self) -> int:
        m = B.MODE_TUNE if self.mode == "tune" else B.MODE_EVAL
        return B.convbn_grouped_saved_bytes(self.desc, self.groups, m, not self.keep_folded)

    def forward(self, stream=None):
        if self.mode == "tune":
            B.convbn_grouped_tune_fwd(self.desc, self.groups, self.x, self.W, self.b, self.gamma, self.beta, self.mean,
                                      self.var, self.z, self.w_folded, self.ws_fwd, stream)
        else:
            B.convbn_grouped_eval_fwd(self.desc, self.groups, self.x, self.W, self.b, self.gamma, self.beta, self.mean,
                                      self.var, self.z, self.y_saved, self.ws_fwd, stream)

    def backward(self, stream=None):
        if self.mode == "tune":
            B.convbn_grouped_tune_bwd(self.desc, self.groups, self.x, self.W, self.b, self.gamma, self.mean, self.var,
                                      self.w_folded, self.dz, self.dx, self.dW, self.db, self.dgamma, self.dbeta,
                                      self.ws_bwd, stream)
        else:
            B.convbn_grouped_eval_bwd(self.desc, self.groups, self.x, self.W, self.b, self.gamma, self.mean, self.var,
                                      self.y_saved, self.dz, self.dx, self.dW, self.db, self.dgamma, self.dbeta,
                                      self.ws_bwd, stream)

    def step(self, stream=None):
        self.forward(stream)
        self.backward(stream)

    def results(self) -> Dict[str, Optional[torch.Tensor]]:
        torch.cuda.synchronize()
        f = lambda t: None if t is None else t.detach().to("cpu", torch.float64)
        return dict(
            Z=B.act_from_device(self.z),
            dX=B.act_from_device(self.dx) if self.dx is not None else None,
            dW=B.weight_from_device(self.dW) if self.dW is not None else None,
            db=f(self.db), dgamma=f(self.dgamma), dbeta=f(self.dbeta),
            # [cg][kH][kW][Cout] -> logical [Cout, cg, kH, kW]
            Wf=f(self.w_folded).permute(3, 0, 1, 2).contiguous() if self.w_folded is not None else None,
            Y=B.act_from_device(self.y_saved) if self.y_saved is not None else None)
