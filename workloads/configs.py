"""Descriptors of the synthetic workloads (shapes only, no arithmetic).

A network is K modules; module k is a stack of residual blocks with its own
weights (Sec. 4.1, the feature-flow equation of the decoupled forward pass).
The input layer S (stem) belongs to module 0 and the output layer T (head) to
module K-1 (footnote of Sec. 4.2.1).  Auxiliary variable x_k is module k's input.
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

CONFIG_NAMES = ("tiny", "resnet20", "resnet56", "wrn28_10", "resnet50")


@dataclass
class Block:
    kind: str          # "basic" (3x3,3x3) or "bottleneck" (1x1,3x3,1x1)
    cin: int
    cout: int
    width: int         # bottleneck inner width (basic: == cout)
    stride: int        # stride of the block (basic: first 3x3; bottleneck: the 3x3)
    proj: bool         # 1x1 conv(stride)+BN on the skip path
    proj_bn: bool = True       # False: the projection is the bare conv1x1(stride), no BN (conv-BN-ReLU order only)
    post_relu: bool = False    # True: ReLU after the residual sum, X_{m+1} = ReLU(skip + F) (conv-BN-ReLU order only)


@dataclass
class ModuleDesc:
    stem: int          # 0 none, 1 conv3x3(3->stem_cout)+BN+ReLU, 2 conv7x7 s2 +BN+ReLU+maxpool3x3 s2
    stem_cout: int
    blocks: List[Block]
    head: bool         # global avgpool + linear(+bias)
    n_classes: int
    N: int
    H: int
    W: int
    C: int             # dims of the module input x_k, NHWC
    order: str = "post"  # "post": conv-BN-ReLU-conv-BN + skip;  "pre": BN-ReLU-conv-BN-ReLU-conv + skip (Fig. 2);
                         # with "pre" the stem is the bare conv3x3 and the head is BN-ReLU-avgpool-linear

    def out_shape(self) -> Tuple[int, int, int, int]:
        n, h, w, c = self.N, self.H, self.W, self.C
        if self.stem == 1:
            c = self.stem_cout
        elif self.stem == 2:
            h, w, c = h // 4, w // 4, self.stem_cout
        for b in self.blocks:
            h, w, c = h // b.stride, w // b.stride, b.cout
        return n, h, w, c


@dataclass
class AuxDesc:
    cin: int
    cout: int
    stride: int
    relu: bool
    from_prev: bool = False   # block j reads x_j (chained AuxNets, x_{j+1} = AuxNet_j(x_j)) instead of the mini-batch
    mid: Tuple[Tuple[int, int], ...] = ()   # (cout, stride) of the conv3x3-BN-ReLU blocks in front of the last block


def aux_blocks(a: "AuxDesc"):
    """The stack of an AuxNet as (cin, cout, stride, relu) per block: the `mid` blocks end in ReLU, the last block maps
    to `cout` with `stride` and the AuxNet's own ReLU flag."""
    out, c = [], a.cin
    for co, sd in a.mid:
        out.append((c, co, sd, True))
        c = co
    out.append((c, a.cout, a.stride, bool(a.relu)))
    return out


@dataclass
class NetDesc:
    name: str
    K: int
    modules: List[ModuleDesc]
    aux: Optional[List[AuxDesc]]     # K-1 entries (x_1..x_{K-1} from the image) or None
    dtype: str                       # "f32" or "bf16" (storage type; accumulation is fp32)
    bn_eps: float = 1e-5
    al: bool = False                 # augmented Lagrangian (multipliers present) vs penalty
    rho: float = 1.0
    lam_sigma: float = 0.0
    noise_sigma: float = 0.1
    step: float = 0.1                # multiplier step (learning rate / rho)
    seed: int = 0


@dataclass
class TensorSpec:
    name: str
    kind: str          # "conv" | "bn_gamma" | "bn_beta" | "fc_w" | "fc_b"
    shape: Tuple[int, ...]
    fan_in: int = 0
    block: int = -1    # -1 stem, n_blocks head, else block index
    slot: int = 0      # conv slot inside the block: 0,1,2 main path; 3 projection


def _split(blocks: List[Block], counts: List[int]) -> List[List[Block]]:
    out, i = [], 0
    for c in counts:
        out.append(blocks[i:i + c])
        i += c
    assert i == len(blocks)
    return out


def _basic_stages(c0: int, widths: List[int], per_stage: int) -> List[Block]:
    blocks, cin = [], c0
    for si, c in enumerate(widths):
        for bi in range(per_stage):
            stride = 2 if (si > 0 and bi == 0) else 1
            blocks.append(Block("basic", cin, c, c, stride, proj=(stride != 1 or cin != c)))
            cin = c
    return blocks


def _assemble(name, per_module, n, h, w, c_img, stem, stem_cout, n_classes, order="post", **kw) -> NetDesc:
    mods = []
    K = len(per_module)
    shape = (n, h, w, c_img)
    for k, blks in enumerate(per_module):
        m = ModuleDesc(stem=stem if k == 0 else 0, stem_cout=stem_cout if k == 0 else 0,
                       blocks=blks, head=(k == K - 1), n_classes=n_classes,
                       N=shape[0], H=shape[1], W=shape[2], C=shape[3], order=order)
        shape = m.out_shape()
        mods.append(m)
    return NetDesc(name=name, K=K, modules=mods, aux=None, dtype="f32", **kw)


def with_order(net: NetDesc, order: str) -> NetDesc:
    """The same network with every module in the given block order (parameter tensors change with it)."""
    for m in net.modules:
        m.order = order
    return net


def chain_aux(net: NetDesc, relu: bool = False) -> NetDesc:
    """AuxNet blocks that read the previous auxiliary variable: block j maps x_j (module j's input) to x_{j+1}."""
    net.aux = [AuxDesc(cin=net.modules[j].C, cout=net.modules[j + 1].C, stride=net.modules[j].H // net.modules[j + 1].H,
                       relu=relu, from_prev=True) for j in range(net.K - 1)]
    return net


def reaux(net: NetDesc, relu: bool = False) -> NetDesc:
    """Recursive AuxNets (Sec. 4.4): x_{j+1} is generated from the mini-batch by a stack of j+1 blocks of its own, block
    i of the stack mapping the shape of x_i to the shape of x_{i+1}."""
    ms = net.modules
    hop = lambda i: (ms[i + 1].C, ms[i].H // ms[i + 1].H)
    net.aux = [AuxDesc(cin=ms[0].C, cout=ms[j + 1].C, stride=ms[j].H // ms[j + 1].H, relu=relu,
                       mid=tuple(hop(i) for i in range(j))) for j in range(net.K - 1)]
    return net


def deepen_aux(net: NetDesc, extra: int = 1) -> NetDesc:
    """Every AuxNet gets `extra` more blocks in front of its last one: the first block does the change of shape, the
    others keep it (conv3x3 stride 1 at the width of the output)."""
    for a in net.aux:
        a.mid = ((a.cout, a.stride),) + ((a.cout, 1),) * (extra - 1)
        a.stride = 1
    return net


def make_config(name: str, batch: Optional[int] = None, split: Optional[List[int]] = None) -> NetDesc:
    """The five synthetic workloads; `batch` overrides the mini-batch size only, `split` the number of residual
    blocks per module (same network, other K: `[12]` is the layer-serial K=1 form of the 12-block networks)."""
    if split is not None:
        net = make_config(name, batch)
        blocks = [b for m in net.modules for b in m.blocks]
        m0 = net.modules[0]
        out = _assemble(name, _split(blocks, list(split)), m0.N, m0.H, m0.W, m0.C, m0.stem, m0.stem_cout,
                        net.modules[-1].n_classes, order=m0.order, seed=net.seed, al=net.al, lam_sigma=net.lam_sigma, rho=net.rho,
                        step=net.step, bn_eps=net.bn_eps)
        out.dtype = net.dtype
        if net.aux is not None:
            out.aux = [AuxDesc(cin=m0.C, cout=m.C, stride=m0.H // m.H, relu=False) for m in out.modules[1:]]
        return out
    if name == "tiny":
        n = batch or 4
        blk = lambda: Block("basic", 16, 16, 16, 1, False)
        net = _assemble("tiny", [[blk()], [blk()]], n, 8, 8, 16, 0, 0, 10, seed=0)
        return net
    if name == "resnet20":
        n = batch or 128
        blocks = _basic_stages(16, [16, 32, 64], 3)
        net = _assemble("resnet20", _split(blocks, [3, 2, 2, 2]), n, 32, 32, 3, 1, 16, 10, seed=1)
        return net
    if name == "resnet56":
        n = batch or 128
        blocks = _basic_stages(16, [16, 32, 64], 9)
        net = _assemble("resnet56", _split(blocks, [4, 4, 4, 3, 3, 3, 3, 3]), n, 32, 32, 3, 1, 16, 100,
                        seed=2, al=True, lam_sigma=0.01)
        net.dtype = "bf16"
        net.aux = []
        for m in net.modules[1:]:
            net.aux.append(AuxDesc(cin=3, cout=m.C, stride=32 // m.H, relu=False))
        return net
    if name == "wrn28_10":
        n = batch or 128
        blocks = _basic_stages(16, [160, 320, 640], 4)
        net = _assemble("wrn28_10", _split(blocks, [3, 3, 3, 3]), n, 32, 32, 3, 1, 16, 100,
                        seed=3, al=True, lam_sigma=0.01)
        net.dtype = "bf16"
        return net
    if name == "resnet50":
        n = batch or 64
        blocks, cin = [], 64
        for si, (w, cnt) in enumerate(zip([64, 128, 256, 512], [3, 4, 6, 3])):
            for bi in range(cnt):
                stride = 2 if (si > 0 and bi == 0) else 1
                blocks.append(Block("bottleneck", cin, 4 * w, w, stride, proj=(bi == 0)))
                cin = 4 * w
        net = _assemble("resnet50", _split(blocks, [3, 4, 6, 3]), n, 224, 224, 3, 2, 64, 1000, seed=4)
        net.dtype = "bf16"
        return net
    raise ValueError(f"unknown config {name!r}; choose from {CONFIG_NAMES}")


def block_convs(b: Block):
    """(slot, R, cin, cout, stride, pad) of each convolution of a block, main path first."""
    if b.kind == "basic":
        convs = [(0, 3, b.cin, b.cout, b.stride, 1), (1, 3, b.cout, b.cout, 1, 1)]
    else:
        convs = [(0, 1, b.cin, b.width, 1, 0), (1, 3, b.width, b.width, b.stride, 1),
                 (2, 1, b.width, b.cout, 1, 0)]
    if b.proj:
        convs.append((3, 1, b.cin, b.cout, b.stride, 0))
    return convs


def module_tensor_specs(m: ModuleDesc) -> List[TensorSpec]:
    """Parameter tensors of one module in packing order.  Filters are KRSC."""
    t: List[TensorSpec] = []
    if m.order == "pre":
        assert m.stem in (0, 1) and all(b.kind == "basic" for b in m.blocks), "pre-activation: conv3x3 stem, basic blocks"
        if m.stem:
            t.append(TensorSpec("stem.conv", "conv", (m.stem_cout, 3, 3, m.C), 9 * m.C, -1, 0))
        for i, b in enumerate(m.blocks):
            for slot, r, ci, co, _, _ in block_convs(b):
                nm = f"block{i}." + ("proj" if slot == 3 else f"conv{slot + 1}")
                if slot != 3:          # the BN in front of the conv normalises the conv's input channels
                    t.append(TensorSpec(nm + ".bn.gamma", "bn_gamma", (ci,), 0, i, slot))
                    t.append(TensorSpec(nm + ".bn.beta", "bn_beta", (ci,), 0, i, slot))
                t.append(TensorSpec(nm, "conv", (co, r, r, ci), r * r * ci, i, slot))
        if m.head:
            c = m.out_shape()[3]
            nb = len(m.blocks)
            t.append(TensorSpec("head.bn.gamma", "bn_gamma", (c,), 0, nb, 0))
            t.append(TensorSpec("head.bn.beta", "bn_beta", (c,), 0, nb, 0))
            t.append(TensorSpec("head.fc.w", "fc_w", (m.n_classes, c), c, nb, 0))
            t.append(TensorSpec("head.fc.b", "fc_b", (m.n_classes,), c, nb, 0))
        return t
    if m.stem:
        r = 3 if m.stem == 1 else 7
        t.append(TensorSpec("stem.conv", "conv", (m.stem_cout, r, r, m.C), r * r * m.C, -1, 0))
        t.append(TensorSpec("stem.bn.gamma", "bn_gamma", (m.stem_cout,), 0, -1, 0))
        t.append(TensorSpec("stem.bn.beta", "bn_beta", (m.stem_cout,), 0, -1, 0))
    for i, b in enumerate(m.blocks):
        for slot, r, ci, co, _, _ in block_convs(b):
            nm = f"block{i}." + ("proj" if slot == 3 else f"conv{slot + 1}")
            t.append(TensorSpec(nm, "conv", (co, r, r, ci), r * r * ci, i, slot))
            if slot == 3 and not b.proj_bn:
                continue                   # a bare projection has no BN parameters
            t.append(TensorSpec(nm + ".bn.gamma", "bn_gamma", (co,), 0, i, slot))
            t.append(TensorSpec(nm + ".bn.beta", "bn_beta", (co,), 0, i, slot))
    if m.head:
        c = m.out_shape()[3]
        nb = len(m.blocks)
        t.append(TensorSpec("head.fc.w", "fc_w", (m.n_classes, c), c, nb, 0))
        t.append(TensorSpec("head.fc.b", "fc_b", (m.n_classes,), c, nb, 0))
    return t


def aux_tensor_specs(a: AuxDesc) -> List[TensorSpec]:
    """Filter, BN gamma, BN beta of every block of the stack, in order (slot = index of the block)."""
    blocks = aux_blocks(a)
    out = []
    for i, (ci, co, _, _) in enumerate(blocks):
        pre = "aux" if len(blocks) == 1 else f"aux.b{i}"
        out += [TensorSpec(f"{pre}.conv", "conv", (co, 3, 3, ci), 9 * ci, -1, i),
                TensorSpec(f"{pre}.bn.gamma", "bn_gamma", (co,), 0, -1, i),
                TensorSpec(f"{pre}.bn.beta", "bn_beta", (co,), 0, -1, i)]
    return out


def module_conv_shapes(m: ModuleDesc):
    """List of (M, Ngemm, Kgemm, needs_dgrad) for every convolution of the module."""
    out = []
    n, h, w, c = m.N, m.H, m.W, m.C
    if m.stem == 1:
        out.append((n * h * w, m.stem_cout, 9 * c, False))
        c = m.stem_cout
    elif m.stem == 2:
        out.append((n * (h // 2) * (w // 2), m.stem_cout, 49 * c, False))
        h, w, c = h // 4, w // 4, m.stem_cout
    for b in m.blocks:
        hh, ww = h, w
        for slot, r, ci, co, st, _ in block_convs(b):
            if slot == 3:
                out.append((n * (h // b.stride) * (w // b.stride), co, ci, True))
            else:
                hh, ww = hh // st, ww // st
                out.append((n * hh * ww, co, r * r * ci, True))
        h, w, c = h // b.stride, w // b.stride, b.cout
    return out


def conv_flops_forward(net: NetDesc) -> float:
    """2*M*Ngemm*Kgemm summed over every convolution of every module (one forward pass)."""
    return float(sum(2.0 * M * Nn * Kk for m in net.modules for (M, Nn, Kk, _) in module_conv_shapes(m)))


def conv_flops_step(net: NetDesc) -> float:
    """Forward + wgrad for every conv, + dgrad for every conv except an image-facing stem."""
    tot = 0.0
    for m in net.modules:
        for (M, Nn, Kk, dg) in module_conv_shapes(m):
            tot += 2.0 * M * Nn * Kk * (3.0 if dg else 2.0)
    return tot
