"""Seeded synthetic inputs for the ConvBN block (shared by the tests, the smoke
check and the benchmark; feeds both the CPU oracle and the GPU library).

This module holds none of the method's arithmetic: it only draws random tensors
with the shapes and value distributions of the workloads (ResNet-50 layer shapes
standing in for the paper's pretrained backbones) and, for bf16 problems, rounds
the tensors that the library receives in bf16 so that both sides see identical
values.

Draw order (CPU generator, fp32): x ~ N(0,1) [N,Cin,Hin,Win]; W ~ N(0, 2/(Cin kH kW))
(fan-in Kaiming normal); gamma ~ U(0.5,1.5); beta ~ N(0,0.1^2); running mean
~ N(0,0.1^2); running var ~ U(0.5,2); dy ~ N(0,1) [N,Cout,Hout,Wout]; then, if
asked for, a conv bias b ~ N(0,0.1^2).  eps = 1e-5.
"""
from dataclasses import dataclass, replace
from typing import Dict, List, Optional

import torch


@dataclass(frozen=True)
class BlockShape:
    """Logical size of one ConvBN block (Sec. 3.1 notation)."""
    name: str
    N: int
    Cin: int
    Hin: int
    Win: int
    Cout: int
    k: int
    stride: int = 1
    pad: int = 0
    dtype: str = "bf16"      # "f32" or "bf16": storage type of x, W, z, dz, dx, dW
    seed: int = 0

    @property
    def Hout(self) -> int:
        return (self.Hin + 2 * self.pad - self.k) // self.stride + 1

    @property
    def Wout(self) -> int:
        return (self.Win + 2 * self.pad - self.k) // self.stride + 1

    @property
    def M(self) -> int:
        return self.N * self.Hout * self.Wout

    @property
    def K(self) -> int:
        return self.Cin * self.k * self.k

    @property
    def P(self) -> int:
        return self.Cout * self.K

    @property
    def A_x(self) -> int:
        return self.N * self.Cin * self.Hin * self.Win

    @property
    def A_z(self) -> int:
        return self.N * self.Cout * self.Hout * self.Wout

    @property
    def fwd_flop(self) -> float:
        return 2.0 * self.M * self.K * self.Cout

    @property
    def step_flop(self) -> float:
        """fprop + dgrad + wgrad, useful MACs only."""
        return 3.0 * self.fwd_flop

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4


# The benchmark configurations (single blocks).
CONFIGS: Dict[str, BlockShape] = {
    "c0": BlockShape("c0", 2, 16, 16, 16, 32, 3, 1, 1, "f32", 0),
    "c1": BlockShape("c1", 32, 256, 56, 56, 64, 1, 1, 0, "bf16", 1),
    "c2a": BlockShape("c2a", 32, 64, 56, 56, 64, 3, 1, 1, "bf16", 2),
    "c2b": BlockShape("c2b", 64, 512, 7, 7, 512, 3, 1, 1, "bf16", 2),
    "c3a": BlockShape("c3a", 32, 3, 224, 224, 64, 7, 2, 3, "bf16", 3),
    "c3b": BlockShape("c3b", 32, 256, 28, 28, 256, 3, 2, 1, "bf16", 3),
}


def round_bf16(t: torch.Tensor) -> torch.Tensor:
    """Round to nearest-even bf16 and widen back to fp32 (value-preserving)."""
    return t.to(torch.bfloat16).to(torch.float32)


def make_inputs(shape: BlockShape, seed: Optional[int] = None, bias: bool = False,
                wide_scale: bool = False, batch: Optional[int] = None) -> Dict[str, object]:
    """Draw one block's tensors on the CPU, logical NCHW, fp32 storage.

    For bf16 problems x, W and dy are rounded to bf16 first (still returned as
    fp32 tensors holding bf16-representable values).  `wide_scale` draws the BN
    scale gamma/sqrt(var+eps) uniformly from [0, 30] with some exact zeros, the
    range the paper reports for pretrained backbones (Fig. 2a).  `batch`
    overrides N (used to bound the CPU-baseline sample).
    """
    if batch is not None:
        shape = replace(shape, N=batch)
    g = torch.Generator(device="cpu")
    g.manual_seed(shape.seed if seed is None else seed)
    s = shape
    x = torch.randn(s.N, s.Cin, s.Hin, s.Win, generator=g)
    W = torch.randn(s.Cout, s.Cin, s.k, s.k, generator=g) * (2.0 / (s.Cin * s.k * s.k)) ** 0.5
    gamma = torch.rand(s.Cout, generator=g) + 0.5
    beta = torch.randn(s.Cout, generator=g) * 0.1
    rmean = torch.randn(s.Cout, generator=g) * 0.1
    rvar = torch.rand(s.Cout, generator=g) * 1.5 + 0.5
    dy = torch.randn(s.N, s.Cout, s.Hout, s.Wout, generator=g)
    b = torch.randn(s.Cout, generator=g) * 0.1 if bias else None
    eps = 1e-5
    if wide_scale:
        scale = torch.rand(s.Cout, generator=g) * 30.0
        scale[:: max(1, s.Cout // 4)] = 0.0
        gamma = scale * torch.sqrt(rvar + eps)
    if s.dtype == "bf16":
        x, W, dy = round_bf16(x), round_bf16(W), round_bf16(dy)
    return dict(shape=s, x=x, W=W, b=b, gamma=gamma, beta=beta, rmean=rmean, rvar=rvar, dy=dy,
                eps=eps)


def tconv_out(shape: BlockShape):
    """(Hout, Wout) of a transposed convolution with the shape's window, stride and padding."""
    return ((shape.Hin - 1) * shape.stride - 2 * shape.pad + shape.k,
            (shape.Win - 1) * shape.stride - 2 * shape.pad + shape.k)


def make_tconv_inputs(shape: BlockShape, seed: Optional[int] = None, bias: bool = False,
                      wide_scale: bool = False) -> Dict[str, object]:
    """Tensors of a TransposedConv-BN block (Sec. 3.2.1): the shape's fields describe the block's input and
    its operator, W is the logical [Cin, Cout, k, k] ~ N(0, 2 stride^2 / (Cin k^2)) (every output pixel sums
    about Cin (k/stride)^2 products), dy has the transposed convolution's output size.  Same draw order and
    distributions as make_inputs otherwise."""
    g = torch.Generator(device="cpu")
    g.manual_seed(shape.seed if seed is None else seed)
    s = shape
    ho, wo = tconv_out(s)
    x = torch.randn(s.N, s.Cin, s.Hin, s.Win, generator=g)
    W = torch.randn(s.Cin, s.Cout, s.k, s.k, generator=g) * (2.0 * s.stride ** 2 / (s.Cin * s.k * s.k)) ** 0.5
    gamma = torch.rand(s.Cout, generator=g) + 0.5
    beta = torch.randn(s.Cout, generator=g) * 0.1
    rmean = torch.randn(s.Cout, generator=g) * 0.1
    rvar = torch.rand(s.Cout, generator=g) * 1.5 + 0.5
    dy = torch.randn(s.N, s.Cout, ho, wo, generator=g)
    b = torch.randn(s.Cout, generator=g) * 0.1 if bias else None
    eps = 1e-5
    if wide_scale:
        scale = torch.rand(s.Cout, generator=g) * 30.0
        scale[:: max(1, s.Cout // 4)] = 0.0
        gamma = scale * torch.sqrt(rvar + eps)
    if s.dtype == "bf16":
        x, W, dy = round_bf16(x), round_bf16(W), round_bf16(dy)
    return dict(shape=s, x=x, W=W, b=b, gamma=gamma, beta=beta, rmean=rmean, rvar=rvar, dy=dy,
                eps=eps)


def make_dw_inputs(shape: BlockShape, seed: Optional[int] = None, bias: bool = False,
                   wide_scale: bool = False) -> Dict[str, object]:
    """Tensors of a depthwise ConvBN block (Cin == Cout, one filter per channel): W is the logical [C, 1, k, k]
    ~ N(0, 2/k^2) (fan-in k^2); everything else as make_inputs."""
    assert shape.Cin == shape.Cout
    g = torch.Generator(device="cpu")
    g.manual_seed(shape.seed if seed is None else seed)
    s = shape
    x = torch.randn(s.N, s.Cin, s.Hin, s.Win, generator=g)
    W = torch.randn(s.Cout, 1, s.k, s.k, generator=g) * (2.0 / (s.k * s.k)) ** 0.5
    gamma = torch.rand(s.Cout, generator=g) + 0.5
    beta = torch.randn(s.Cout, generator=g) * 0.1
    rmean = torch.randn(s.Cout, generator=g) * 0.1
    rvar = torch.rand(s.Cout, generator=g) * 1.5 + 0.5
    dy = torch.randn(s.N, s.Cout, s.Hout, s.Wout, generator=g)
    b = torch.randn(s.Cout, generator=g) * 0.1 if bias else None
    eps = 1e-5
    if wide_scale:
        scale = torch.rand(s.Cout, generator=g) * 30.0
        scale[:: max(1, s.Cout // 4)] = 0.0
        gamma = scale * torch.sqrt(rvar + eps)
    if s.dtype == "bf16":
        x, W, dy = round_bf16(x), round_bf16(W), round_bf16(dy)
    return dict(shape=s, x=x, W=W, b=b, gamma=gamma, beta=beta, rmean=rmean, rvar=rvar, dy=dy,
                eps=eps)


def make_grouped_inputs(shape: BlockShape, groups: int, seed: Optional[int] = None, bias: bool = False,
                        wide_scale: bool = False, batch: Optional[int] = None) -> Dict[str, object]:
    """Tensors of a grouped ConvBN block (`groups` divides Cin and Cout): W is the logical
    [Cout, Cin/groups, k, k] ~ N(0, 2 / fan-in) with fan-in (Cin/groups) k^2; everything else as make_inputs."""
    if batch is not None:
        shape = replace(shape, N=batch)
    assert shape.Cin % groups == 0 and shape.Cout % groups == 0
    g = torch.Generator(device="cpu")
    g.manual_seed(shape.seed if seed is None else seed)
    s = shape
    cg = s.Cin // groups
    x = torch.randn(s.N, s.Cin, s.Hin, s.Win, generator=g)
    W = torch.randn(s.Cout, cg, s.k, s.k, generator=g) * (2.0 / (cg * s.k * s.k)) ** 0.5
    gamma = torch.rand(s.Cout, generator=g) + 0.5
    beta = torch.randn(s.Cout, generator=g) * 0.1
    rmean = torch.randn(s.Cout, generator=g) * 0.1
    rvar = torch.rand(s.Cout, generator=g) * 1.5 + 0.5
    dy = torch.randn(s.N, s.Cout, s.Hout, s.Wout, generator=g)
    b = torch.randn(s.Cout, generator=g) * 0.1 if bias else None
    eps = 1e-5
    if wide_scale:
        scale = torch.rand(s.Cout, generator=g) * 30.0
        scale[:: max(1, s.Cout // 4)] = 0.0
        gamma = scale * torch.sqrt(rvar + eps)
    if s.dtype == "bf16":
        x, W, dy = round_bf16(x), round_bf16(W), round_bf16(dy)
    return dict(shape=s, groups=groups, x=x, W=W, b=b, gamma=gamma, beta=beta, rmean=rmean, rvar=rvar, dy=dy,
                eps=eps)


def make_params(shape: BlockShape, seed: Optional[int] = None) -> Dict[str, object]:
    """Only the parameters of a block (same distributions and draw order as make_inputs, but
    without the activation-sized tensors): W, gamma, beta, running mean, running var."""
    g = torch.Generator(device="cpu")
    g.manual_seed(shape.seed if seed is None else seed)
    s = shape
    W = torch.randn(s.Cout, s.Cin, s.k, s.k, generator=g) * (2.0 / (s.Cin * s.k * s.k)) ** 0.5
    gamma = torch.rand(s.Cout, generator=g) + 0.5
    beta = torch.randn(s.Cout, generator=g) * 0.1
    rmean = torch.randn(s.Cout, generator=g) * 0.1
    rvar = torch.rand(s.Cout, generator=g) * 1.5 + 0.5
    if s.dtype == "bf16":
        W = round_bf16(W)
    return dict(shape=s, W=W, gamma=gamma, beta=beta, rmean=rmean, rvar=rvar, eps=1e-5)


def resnet50_blocks(N: int = 32, image: int = 224, dtype: str = "bf16") -> List[BlockShape]:
    """The 53 ConvBN blocks of a ResNet-50 backbone (stride on the 3x3 conv of each
    stage's first bottleneck, 1x1 stride-s projection on the shortcut), in forward
    order.  Names: stem, l{stage}.{block}.{a,b,c,ds}."""
    out: List[BlockShape] = []
    h = image
    out.append(BlockShape("stem", N, 3, h, h, 64, 7, 2, 3, dtype, 100))
    h = (h + 2 * 3 - 7) // 2 + 1          # conv stem
    h = (h + 2 * 1 - 3) // 2 + 1          # 3x3/2 max-pool
    cin = 64
    seed = 101
    for stage, (width, nblk) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3)), start=1):
        for blk in range(nblk):
            s = 2 if (blk == 0 and stage > 1) else 1
            pre = f"l{stage}.{blk}"
            out.append(BlockShape(pre + ".a", N, cin, h, h, width, 1, 1, 0, dtype, seed))
            out.append(BlockShape(pre + ".b", N, width, h, h, width, 3, s, 1, dtype, seed + 1))
            ho = (h + 2 - 3) // s + 1
            out.append(BlockShape(pre + ".c", N, width, ho, ho, width * 4, 1, 1, 0, dtype,
                                  seed + 2))
            if blk == 0:
                out.append(BlockShape(pre + ".ds", N, cin, h, h, width * 4, 1, s, 0, dtype,
                                      seed + 3))
            seed += 4
            cin = width * 4
            h = ho
    return out
