"""ResNet-50 backbone (53 ConvBN blocks, ReLU, bottleneck residual adds, 3x3/2 max-pool) chained on
the GPU through the library, forward + backward with frozen BatchNorm statistics, in Tune or
Eval mode -- the workload of the paper's end-to-end time / memory table (App. D).

Everything numeric runs in the library's kernels (blocks: convbn_tune_* / convbn_eval_*; glue:
convbn_aux_*).  PyTorch allocates the buffers, which is also how the peak activation memory is
measured (caching-allocator high-water mark above the parameters, gradients and workspace).
"""
from typing import Dict, List, Optional

import torch

from . import binding as B
from . import synth


class _Block:
    def __init__(self, shape, device, mode, act=0):
        self.shape, self.mode = shape, mode
        p = synth.make_params(shape)
        self.desc = B.desc_from_shape(shape, eps=p["eps"])
        self.act = act        # the ReLUs next to the block that its convolutions apply on the way out
        self.desc.act = act
        dt = B.torch_dtype(self.desc)
        self.dt = dt
        self.W = B.weight_to_device(p["W"], dt, device)
        self.gamma, self.beta = B.vec_to_device(p["gamma"], device), B.vec_to_device(p["beta"], device)
        self.mean, self.var = B.vec_to_device(p["rmean"], device), B.vec_to_device(p["rvar"], device)
        self.dW = torch.empty_like(self.W)
        self.dgamma, self.dbeta = torch.empty_like(self.gamma), torch.empty_like(self.beta)
        m = B.MODE_TUNE if mode == "tune" else B.MODE_EVAL
        self.ws_bytes = max(B.convbn_workspace_bytes(self.desc, m, B.PASS_FWD),
                            B.convbn_workspace_bytes(self.desc, m, B.PASS_BWD))
        # Tune keeps w' unless it is larger than the Y that Eval would keep (then backward re-folds)
        self.keep_folded = mode == "tune" and shape.P <= shape.A_z
        self.x = self.saved = None
        self.grouped = None      # buffers of the network's grouped fold (Tune mode, optional)
        self.unit = None         # buffers of this block inside its unit's grouped fold / fold-back (Tune mode)

    def forward(self, x, ws, add=None):
        """add: the other branch of a residual sum that joins behind this block; the block then returns
        max(z + add, 0) (the descriptor's addend and ReLU bits, for this call)."""
        s = self.shape
        z = torch.empty((s.N, s.Hout, s.Wout, s.Cout), dtype=self.dt, device=x.device)
        self.x = x
        if add is not None:
            B.set_addends(self.desc, add_out=add)
            self.desc.act = self.act | B.ACT_ADD_OUT | B.ACT_RELU_OUT
        try:
            return self._forward(x, z, ws)
        finally:
            self.desc.act = self.act
            B.set_addends(self.desc)

    def _forward(self, x, z, ws):
        s = self.shape
        if self.unit is not None:
            # w' of this block was produced by its unit's grouped fold: only the convolution is left
            B.convbn_conv_fprop(self.desc, x, self.unit["w_fprop"], self.unit["b_folded"], z, ws)
            self.saved = self.unit["w_folded"]
        elif self.grouped is not None:
            # w' of this block was produced by the network's grouped fold: only the convolution is left
            B.convbn_conv_fprop(self.desc, x, self.grouped["w_fprop"], self.grouped["b_folded"], z, ws)
            self.saved = self.grouped["w_folded"]
        elif self.mode == "tune":
            self.saved = torch.empty((s.Cin, s.k, s.k, s.Cout), dtype=self.dt, device=x.device) \
                if self.keep_folded else None
            B.convbn_tune_fwd(self.desc, x, self.W, None, self.gamma, self.beta, self.mean, self.var, z,
                              self.saved, ws)
        else:
            self.saved = torch.empty_like(z)
            B.convbn_eval_fwd(self.desc, x, self.W, None, self.gamma, self.beta, self.mean, self.var, z,
                              self.saved, ws)
        return z

    def backward(self, dz, ws, need_dx=True, add=None, relu_in=False):
        """add: the gradient that reaches this block's input through another branch; the block then returns
        dx + add, zeroed where its input is not positive if relu_in (the input is a ReLU's output)."""
        if add is not None:
            B.set_addends(self.desc, add_in=add)
            self.desc.act = self.act | B.ACT_ADD_IN | (B.ACT_RELU_IN if relu_in else 0)
        try:
            return self._backward(dz, ws, need_dx)
        finally:
            self.desc.act = self.act
            B.set_addends(self.desc)

    def _backward(self, dz, ws, need_dx):
        dx = torch.empty_like(self.x) if need_dx else None
        if self.unit is not None and not self.unit["fused"]:
            # this block's fold-back runs with its unit's, in one launch: only the two gradient convolutions here
            u = self.unit
            B.convbn_conv_dgrad(self.desc, dz, u["w_t"], dx, ws,
                                x_mask=self.x if self.desc.act & B.ACT_RELU_IN else None)
            B.convbn_conv_wgrad(self.desc, self.x, dz, u["dw_part"], u["r_part"], ws)
            self.x = self.saved = None
            return dx
        if self.mode == "tune":
            B.convbn_tune_bwd(self.desc, self.x, self.W, None, self.gamma, self.mean, self.var, self.saved,
                              dz, dx, self.dW, None, self.dgamma, self.dbeta, ws)
        else:
            B.convbn_eval_bwd(self.desc, self.x, self.W, None, self.gamma, self.mean, self.var, self.saved,
                              dz, dx, self.dW, None, self.dgamma, self.dbeta, ws)
        self.x = self.saved = None
        return dx


class ResNet50:
    def __init__(self, N: int = 32, image: int = 224, dtype: str = "bf16", mode: str = "tune",
                 device: str = "cuda", group_fold: bool = False, group_units: bool = False,
                 fuse_residual: bool = True):
        """group_fold (Tune mode): fold all blocks in one launch at the start of forward instead of one
        launch per block.  Faster, but every w' (in both orders) then lives for the whole step.
        group_units (Tune mode): one fold launch and one fold-back launch per bottleneck unit (its three or four
        blocks) instead of one per block; the forward-order w' and the fp32 partial sums live in arenas the size of
        the largest unit."""
        assert mode in ("tune", "eval")
        self.N, self.image, self.mode, self.device = N, image, mode, device
        # the residual sum of a unit (and the ReLU behind it) applied by the unit's last convolution, the sum of the two
        # gradient branches at its input (and that ReLU's backward) by the first block's input gradient -- both modes
        self.fuse_residual = fuse_residual
        self.group_fold = group_fold and mode == "tune"
        self.group_units = group_units and mode == "tune" and not self.group_fold
        self._group = None
        self.group_bytes = 0
        self.arena_bytes = self.kept_bytes = 0   # per-unit grouping: the shared arena (workspace) and the kept w'
        shapes = synth.resnet50_blocks(N, image, dtype)
        # inside a bottleneck unit: ReLU behind the first two blocks, hence in front of the last two (the ReLU behind
        # the unit follows the residual sum and stays an element-wise pass, like the stem's in front of the max-pool)
        act = {"a": B.ACT_RELU_OUT, "b": B.ACT_RELU_OUT | B.ACT_RELU_IN, "c": B.ACT_RELU_IN}
        self.blocks: Dict[str, _Block] = {s.name: _Block(s, device, mode, act.get(s.name.rsplit(".", 1)[-1], 0))
                                          for s in shapes}
        self.order: List[str] = [s.name for s in shapes]
        self.ws = torch.empty(max(b.ws_bytes for b in self.blocks.values()) + 256, dtype=torch.uint8, device=device)
        self.dt = self.blocks["stem"].dt
        self.stages = []
        for st, nblk in enumerate((3, 4, 6, 3), start=1):
            self.stages.append([f"l{st}.{i}" for i in range(nblk)])
        self._tape = None
        self.units = None
        if self.group_units:
            self._build_units()

    def _build_units(self):
        """Tables and arenas of the per-unit grouped fold and fold-back.  Everything the tables point to is allocated
        once: the kept w' of every block (what Tune mode keeps anyway), and three arenas the size of the largest
        unit -- the forward-order w' + b', the w' folded again in backward for blocks that keep nothing, and the
        fp32 partial sums of the weight gradients."""
        bl, dev = self.blocks, self.device
        names = [[u + sfx for sfx in (".c", ".b", ".a", ".ds") if (u + sfx) in bl] for st in self.stages for u in st]
        need = dict(fwd=0, refold=0, part=0)
        plans = []
        for unit in names:
            off = dict(fwd=0, refold=0, part=0)
            rows = []
            for nme in unit:
                b = bl[nme]
                s = b.shape
                P = s.Cout * s.K
                # blocks whose backward is one launch anyway, or whose fp32 partial sums are large (they would set the
                # size of the arena), keep their own backward call
                big = B.convbn_wgrad_parts(b.desc) * P * 4 > (16 << 20)
                row = dict(block=b, fwd=off["fwd"], fused=B.convbn_tune_bwd_is_fused(b.desc) or big)
                off["fwd"] += (P * 2 + 255) // 256 * 256 + (s.Cout * 4 + 255) // 256 * 256
                if not b.keep_folded and not row["fused"]:
                    row["refold"] = off["refold"]
                    off["refold"] += (P * 2 + 255) // 256 * 256
                if not row["fused"]:
                    row["part"] = off["part"]
                    ns, nr = B.convbn_wgrad_parts(b.desc), B.convbn_rsum_parts(b.desc)
                    row["ns"], row["nr"] = ns, nr
                    off["part"] += (ns * P * 4 + 255) // 256 * 256 + (nr * s.Cout * 4 + 255) // 256 * 256
                rows.append(row)
            plans.append(rows)
            for k in need:
                need[k] = max(need[k], off[k])
        # one arena: the forward-order w' of a unit lives in it during forward, the re-folded w' and the partial sums
        # of a unit during backward
        need["refold"] = (need["refold"] + 255) // 256 * 256
        one = torch.empty(max(need["fwd"], need["refold"] + need["part"], 256), dtype=torch.uint8, device=dev)
        arena = dict(fwd=one, refold=one, part=one[need["refold"]:])

        def view(buf, off, nbytes, dtype):
            return buf[off:off + nbytes].view(dtype)

        self.units = {}
        kept_bytes = 0
        for unit, rows in zip(names, plans):
            fold_items, refold_items, back_items = [], [], []
            for row in rows:
                b = row["block"]
                s = b.shape
                P = s.Cout * s.K
                u = dict(fused=row["fused"])
                u["w_fprop"] = view(arena["fwd"], row["fwd"], P * 2, self.dt)
                u["b_folded"] = view(arena["fwd"], row["fwd"] + (P * 2 + 255) // 256 * 256, s.Cout * 4, torch.float32)
                u["w_folded"] = torch.empty(P, dtype=self.dt, device=dev) if b.keep_folded else None
                kept_bytes += P * 2 if b.keep_folded else 0
                fold_items.append(dict(desc=b.desc, W=b.W, b=None, gamma=b.gamma, beta=b.beta, mean=b.mean, var=b.var,
                                       w_fprop=u["w_fprop"], w_folded=u["w_folded"], b_folded=u["b_folded"]))
                if not row["fused"]:
                    if b.keep_folded:
                        u["w_t"] = u["w_folded"]
                    else:
                        u["w_t"] = view(arena["refold"], row["refold"], P * 2, self.dt)
                        refold_items.append(dict(desc=b.desc, W=b.W, b=None, gamma=b.gamma, beta=None, mean=b.mean,
                                                 var=b.var, w_fprop=None, w_folded=u["w_t"], b_folded=None))
                    u["dw_part"] = view(arena["part"], row["part"], row["ns"] * P * 4, torch.float32)
                    u["r_part"] = view(arena["part"], row["part"] + (row["ns"] * P * 4 + 255) // 256 * 256,
                                       row["nr"] * s.Cout * 4, torch.float32)
                    back_items.append(dict(desc=b.desc, dw_part=u["dw_part"], r_part=u["r_part"], W=b.W, b=None,
                                           gamma=b.gamma, mean=b.mean, var=b.var, dW=b.dW, db=None, dgamma=b.dgamma,
                                           dbeta=b.dbeta))
                b.unit = u
            key = unit[0].rsplit(".", 1)[0]
            self.units[key] = dict(
                fold=B.convbn_fold_group_plan(fold_items, device=dev),
                refold=B.convbn_fold_group_plan(refold_items, device=dev) if refold_items else None,
                back=B.convbn_fold_back_group_plan(back_items, device=dev) if back_items else None)
        self._unit_keep = (arena, plans)
        # what the grouping adds to the memory a step holds: the arenas (the kept w' is counted as before)
        self.group_bytes = one.numel() + kept_bytes
        self.arena_bytes, self.kept_bytes = one.numel(), kept_bytes

    def fold_group_table(self, alloc=True):
        """(n, table, grid, bytes moved) of the grouped fold over every block the group takes (all but
        blocks whose channel counts are not multiples of 8, i.e. the stem)."""
        items, byts = [], 0
        for name in self.order:
            b = self.blocks[name]
            s = b.shape
            if s.Cout % 8 or s.K % 8:
                continue
            P = s.Cout * s.K
            g = dict(w_fprop=torch.empty(P, dtype=self.dt, device=self.device),
                     w_folded=torch.empty(P, dtype=self.dt, device=self.device),
                     b_folded=torch.empty(s.Cout, dtype=torch.float32, device=self.device))
            items.append((b, g))
            byts += 3 * P * 2 + 24 * s.Cout
        n, table, grid = B.convbn_fold_group_plan(
            [dict(desc=b.desc, W=b.W, b=None, gamma=b.gamma, beta=b.beta, mean=b.mean, var=b.var, **g)
             for b, g in items], device=self.device)
        return items, n, table, grid, byts

    def _fold_all(self):
        # the buffers and the table are made once (the table holds pointers); `group_bytes` is what they
        # add to the memory a Tune-mode step keeps -- the caller adds it to the measured peak
        if self._group is None:
            items, n, table, grid, _ = self.fold_group_table()
            self._group = (items, n, table, grid)
            self.group_bytes = sum(sum(t.numel() * t.element_size() for t in g.values()) for _, g in items)
        items, n, table, grid = self._group
        B.convbn_fold_group(n, table, grid)
        for b, g in items:
            b.grouped = g

    def saved_bytes_model(self) -> int:
        """Analytic bytes kept between forward and backward besides the block inputs."""
        m = B.MODE_TUNE if self.mode == "tune" else B.MODE_EVAL
        return sum(B.convbn_saved_bytes(b.desc, m, self.mode == "tune" and not b.keep_folded)
                   for b in self.blocks.values())

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        """x: [N][image][image][3] device tensor (channels-last).  Returns [N][h][w][2048]."""
        ws, bl = self.ws, self.blocks
        if self.group_fold:
            self._fold_all()
        z0 = bl["stem"].forward(x, ws)
        B.convbn_aux_eltwise(B.OP_RELU, z0)
        n, h, w, c = z0.shape
        p = torch.empty((n, (h - 1) // 2 + 1, (w - 1) // 2 + 1, c), dtype=self.dt, device=x.device)
        idx = torch.empty(p.shape, dtype=torch.uint8, device=x.device)
        B.convbn_aux_maxpool_fwd(z0, p, idx)
        tape = dict(z0=z0, idx=idx, units=[])
        cur = p
        for names in self.stages:
            for name in names:
                if self.units is not None:
                    B.convbn_fold_group(*self.units[name]["fold"])
                a = bl[name + ".a"].forward(cur, ws)     # (ReLU applied by the block: its act bits)
                b = bl[name + ".b"].forward(a, ws)
                has_ds = (name + ".ds") in bl
                sc = bl[name + ".ds"].forward(cur, ws) if has_ds else cur
                if self.fuse_residual:
                    c_ = bl[name + ".c"].forward(b, ws, add=sc)   # max(z + shortcut, 0) on the convolution's way out
                else:
                    c_ = bl[name + ".c"].forward(b, ws)
                    B.convbn_aux_eltwise(B.OP_ADD_RELU, c_, sc)
                tape["units"].append((name, has_ds, c_))   # (a and b live on as the next blocks' inputs)
                del a, b
                del sc
                cur = c_
        self._tape = tape
        return cur

    def backward(self, dout: torch.Tensor, need_input_grad: bool = False) -> Optional[torch.Tensor]:
        ws, bl, tape = self.ws, self.blocks, self._tape
        g = dout.clone()
        units = tape["units"]
        B.convbn_aux_eltwise(B.OP_RELU_BWD, g, units[-1][2])   # the last unit's ReLU; the others' ride on the adds below
        while units:
            # a unit's entry leaves the tape when its turn comes: its activations are freed as its blocks finish
            name, has_ds, out = units.pop()
            del out
            first = not units   # the first unit's input comes from the max-pool, not from a ReLU
            if self.units is not None and self.units[name]["refold"] is not None:
                B.convbn_fold_group(*self.units[name]["refold"])   # blocks that kept nothing: w' again, for this unit
            gb = bl[name + ".c"].backward(g, ws)     # (masked with b > 0 by the block: its act bits)
            ga = bl[name + ".b"].backward(gb, ws)    # (masked with a > 0)
            del gb
            # the two branches meet at the unit's input, which is the output of the previous unit's ReLU (of the
            # max-pool for the first unit): sum and ReLU backward on the way out of the first block's input gradient,
            # or in one element-wise pass
            if self.fuse_residual:
                other = bl[name + ".ds"].backward(g, ws) if has_ds else g
                gin = bl[name + ".a"].backward(ga, ws, add=other, relu_in=not first)
                del ga
            else:
                gin = bl[name + ".a"].backward(ga, ws)
                del ga
                other = bl[name + ".ds"].backward(g, ws) if has_ds else g
                if not first:
                    B.convbn_aux_add_relu_bwd(gin, other, units[-1][2])
                else:
                    B.convbn_aux_eltwise(B.OP_ADD, gin, other)
            del other
            if self.units is not None and self.units[name]["back"] is not None:
                B.convbn_fold_back_group(*self.units[name]["back"])   # dW, dgamma, dbeta of the unit's blocks
            g = gin
        z0, idx = tape["z0"], tape["idx"]
        gz0 = torch.empty_like(z0)
        B.convbn_aux_maxpool_bwd(g, idx, gz0)
        del g
        B.convbn_aux_eltwise(B.OP_RELU_BWD, gz0, z0)
        gx = bl["stem"].backward(gz0, ws, need_dx=need_input_grad)
        self._tape = None
        if self._group is not None:
            for b, _ in self._group[0]:
                b.grouped = None
        return gx

    def grads(self, name: str) -> Dict[str, torch.Tensor]:
        b = self.blocks[name]
        return dict(dW=B.weight_from_device(b.dW), dgamma=b.dgamma.double().cpu(), dbeta=b.dbeta.double().cpu())
