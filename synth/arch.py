"""Shape descriptions of the synthetic SuperNet families and of a subnet cfg.

A spec lists, in forward order, every weight tensor of the max-size SuperNet
(name, shape, fan-in) and every SubnetNorm layer (name, max channels), plus the
choice sets a subnet control tuple (D, E, W [, kernel, resolution]) is drawn
from.  Names are the join key between these generators, the oracle's wiring and
the HIP library's weight-blob layout.  No forward arithmetic lives here.

Tensor layouts (row-major):
  conv      [C_out_max][R][S][C_in_max]
  depthwise [R][S][C_max]
  linear    [out_max][in_max]
  bias / LayerNorm gamma, beta  [C_max]
"""
from dataclasses import dataclass, field
from typing import List, Tuple

MAX_STAGES = 8
MAX_DEPTH = 16


def round_channels(x: float) -> int:
    """Ratio -> channel-count rule: nearest multiple of 8, at least 8."""
    return max(8, 8 * int((x + 4.0) // 8))


@dataclass(frozen=True)
class TensorDesc:
    name: str
    shape: Tuple[int, ...]
    kind: str          # conv | dw | linear | bias | ln_gamma | ln_beta
    fan_in: int


@dataclass
class SubnetCfg:
    """One resolved subnet: integers only (ratios already turned into counts)."""
    subnet_id: int
    n_stages: int
    depth: List[int]
    stage_out_ch: List[int]                 # [0] = stem, [1+s] = stage s
    block_mid_ch: List[List[int]]           # [stage][block]
    block_aux_ch: List[List[int]]           # transformer FFN width, else 0
    block_kernel: List[List[int]]           # depthwise kernel (3|5|7), else 0
    in_h: int
    in_w: int

    def key(self):
        return (tuple(self.depth), tuple(self.stage_out_ch),
                tuple(map(tuple, self.block_mid_ch)),
                tuple(map(tuple, self.block_aux_ch)),
                tuple(map(tuple, self.block_kernel)), self.in_h, self.in_w)


# --------------------------------------------------------------------------
# Tiny conv SuperNet (fp32)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class TinySpec:
    family: str = "tiny"
    dtype: str = "fp32"
    n_classes: int = 10
    in_ch: int = 3
    stem_ch: int = 16
    stage_ch: Tuple[int, ...] = (32, 64, 128)
    max_depth: Tuple[int, ...] = (2, 2, 2)
    depth_choices: Tuple[int, ...] = (1, 2)
    width_choices: Tuple[float, ...] = (0.5, 0.75, 1.0)
    res_choices: Tuple[int, ...] = (32,)

    @property
    def n_stages(self):
        return len(self.stage_ch)

    def tensors(self) -> List[TensorDesc]:
        t = [TensorDesc("stem.w", (self.stem_ch, 3, 3, self.in_ch), "conv", 9 * self.in_ch)]
        prev = self.stem_ch
        for s, c in enumerate(self.stage_ch):
            for j in range(self.max_depth[s]):
                cin = prev if j == 0 else c
                t.append(TensorDesc(f"s{s}.b{j}.w", (c, 3, 3, cin), "conv", 9 * cin))
            prev = c
        t.append(TensorDesc("head.w", (self.n_classes, prev), "linear", prev))
        t.append(TensorDesc("head.b", (self.n_classes,), "bias", prev))
        return t

    def norms(self) -> List[Tuple[str, int]]:
        n = [("stem.sn", self.stem_ch)]
        for s, c in enumerate(self.stage_ch):
            for j in range(self.max_depth[s]):
                n.append((f"s{s}.b{j}.sn", c))
        return n


# --------------------------------------------------------------------------
# ResNet-50-shaped elastic bottleneck SuperNet (bf16)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class ResNetSpec:
    family: str = "resnet"
    dtype: str = "bf16"
    n_classes: int = 1000
    in_ch: int = 3
    stem_ch: int = 64
    stage_ch: Tuple[int, ...] = (256, 512, 1024, 2048)
    stage_stride: Tuple[int, ...] = (1, 2, 2, 2)
    max_depth: Tuple[int, ...] = (4, 6, 8, 6)
    depth_minus: Tuple[int, ...] = (0, 1, 2)
    expand_choices: Tuple[float, ...] = (0.2, 0.25, 0.35)
    width_choices: Tuple[float, ...] = (0.65, 0.8, 1.0)
    res_choices: Tuple[int, ...] = (160, 192, 224)

    @property
    def n_stages(self):
        return len(self.stage_ch)

    def max_mid(self, s: int) -> int:
        return round_channels(max(self.expand_choices) * self.stage_ch[s])

    def tensors(self) -> List[TensorDesc]:
        t = [TensorDesc("stem.w", (self.stem_ch, 7, 7, self.in_ch), "conv", 49 * self.in_ch)]
        prev = self.stem_ch
        for s, c in enumerate(self.stage_ch):
            m = self.max_mid(s)
            for j in range(self.max_depth[s]):
                cin = prev if j == 0 else c
                p = f"s{s}.b{j}."
                t.append(TensorDesc(p + "conv1.w", (m, 1, 1, cin), "conv", cin))
                t.append(TensorDesc(p + "conv2.w", (m, 3, 3, m), "conv", 9 * m))
                t.append(TensorDesc(p + "conv3.w", (c, 1, 1, m), "conv", m))
                if j == 0:
                    t.append(TensorDesc(p + "short.w", (c, 1, 1, cin), "conv", cin))
            prev = c
        t.append(TensorDesc("head.w", (self.n_classes, prev), "linear", prev))
        t.append(TensorDesc("head.b", (self.n_classes,), "bias", prev))
        return t

    def norms(self) -> List[Tuple[str, int]]:
        n = [("stem.sn", self.stem_ch)]
        for s, c in enumerate(self.stage_ch):
            m = self.max_mid(s)
            for j in range(self.max_depth[s]):
                p = f"s{s}.b{j}."
                n += [(p + "sn1", m), (p + "sn2", m), (p + "sn3", c)]
                if j == 0:
                    n.append((p + "sn_short", c))
        return n


# --------------------------------------------------------------------------
# MobileNetV3-shaped elastic SuperNet (bf16)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class MBV3Spec:
    family: str = "mbv3"
    dtype: str = "bf16"
    n_classes: int = 1000
    in_ch: int = 3
    stem_ch: int = 16
    stage_ch: Tuple[int, ...] = (24, 40, 80, 112, 160)
    stage_stride: Tuple[int, ...] = (2, 2, 2, 1, 2)
    stage_se: Tuple[bool, ...] = (False, True, False, True, True)
    stage_act: Tuple[str, ...] = ("relu", "relu", "hswish", "hswish", "hswish")
    max_depth: Tuple[int, ...] = (4, 4, 4, 4, 4)
    depth_choices: Tuple[int, ...] = (2, 3, 4)
    expand_choices: Tuple[int, ...] = (3, 4, 6)
    kernel_choices: Tuple[int, ...] = (3, 5, 7)
    res_choices: Tuple[int, ...] = (160, 192, 224)
    tail_ch: int = 960
    fc_ch: int = 1280
    init_gain: float = 1.0      # weights N(0, init_gain / fan_in), see weights.py

    @property
    def n_stages(self):
        return len(self.stage_ch)

    def block_in(self, s: int, j: int) -> int:
        if j > 0:
            return self.stage_ch[s]
        return self.stem_ch if s == 0 else self.stage_ch[s - 1]

    def max_mid(self, s: int, j: int) -> int:
        return round_channels(max(self.expand_choices) * self.block_in(s, j))

    def max_sq(self, s: int, j: int) -> int:
        return round_channels(self.max_mid(s, j) / 4)

    def tensors(self) -> List[TensorDesc]:
        c0 = self.stem_ch
        t = [TensorDesc("stem.w", (c0, 3, 3, self.in_ch), "conv", 9 * self.in_ch),
             TensorDesc("first.dw.w", (3, 3, c0), "dw", 9),
             TensorDesc("first.pw.w", (c0, 1, 1, c0), "conv", c0)]
        for s, c in enumerate(self.stage_ch):
            for j in range(self.max_depth[s]):
                cin, m, q = self.block_in(s, j), self.max_mid(s, j), self.max_sq(s, j)
                p = f"s{s}.b{j}."
                t.append(TensorDesc(p + "expand.w", (m, 1, 1, cin), "conv", cin))
                t.append(TensorDesc(p + "dw.w", (7, 7, m), "dw", 49))
                if self.stage_se[s]:
                    t.append(TensorDesc(p + "se.fc1.w", (q, m), "linear", m))
                    t.append(TensorDesc(p + "se.fc1.b", (q,), "bias", m))
                    t.append(TensorDesc(p + "se.fc2.w", (m, q), "linear", q))
                    t.append(TensorDesc(p + "se.fc2.b", (m,), "bias", q))
                t.append(TensorDesc(p + "project.w", (c, 1, 1, m), "conv", m))
        last = self.stage_ch[-1]
        t.append(TensorDesc("tail.w", (self.tail_ch, 1, 1, last), "conv", last))
        t.append(TensorDesc("fc1.w", (self.fc_ch, self.tail_ch), "linear", self.tail_ch))
        t.append(TensorDesc("fc1.b", (self.fc_ch,), "bias", self.tail_ch))
        t.append(TensorDesc("head.w", (self.n_classes, self.fc_ch), "linear", self.fc_ch))
        t.append(TensorDesc("head.b", (self.n_classes,), "bias", self.fc_ch))
        return t

    def norms(self) -> List[Tuple[str, int]]:
        c0 = self.stem_ch
        n = [("stem.sn", c0), ("first.sn1", c0), ("first.sn2", c0)]
        for s, c in enumerate(self.stage_ch):
            for j in range(self.max_depth[s]):
                m = self.max_mid(s, j)
                p = f"s{s}.b{j}."
                n += [(p + "sn1", m), (p + "sn2", m), (p + "sn3", c)]
        n.append(("tail.sn", self.tail_ch))
        return n


# --------------------------------------------------------------------------
# Elastic-width Transformer encoder SuperNet (bf16)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class TransformerSpec:
    family: str = "transformer"
    dtype: str = "bf16"
    n_classes: int = 1000
    hidden: int = 768
    n_heads: int = 12
    head_dim: int = 64
    ffn: int = 3072
    max_layers: int = 12
    seq_len: int = 128
    depth_choices: Tuple[int, ...] = (6, 8, 10, 12)
    ratio_choices: Tuple[float, ...] = (0.25, 0.5, 0.75, 1.0)

    @property
    def n_stages(self):
        return 1

    def tensors(self) -> List[TensorDesc]:
        h, a, f = self.hidden, self.n_heads * self.head_dim, self.ffn
        t = []
        for i in range(self.max_layers):
            p = f"l{i}."
            for nm in ("q", "k", "v"):
                t.append(TensorDesc(p + nm + ".w", (a, h), "linear", h))
                t.append(TensorDesc(p + nm + ".b", (a,), "bias", h))
            t.append(TensorDesc(p + "o.w", (h, a), "linear", a))
            t.append(TensorDesc(p + "o.b", (h,), "bias", a))
            t.append(TensorDesc(p + "ln1.g", (h,), "ln_gamma", h))
            t.append(TensorDesc(p + "ln1.b", (h,), "ln_beta", h))
            t.append(TensorDesc(p + "ffn1.w", (f, h), "linear", h))
            t.append(TensorDesc(p + "ffn1.b", (f,), "bias", h))
            t.append(TensorDesc(p + "ffn2.w", (h, f), "linear", f))
            t.append(TensorDesc(p + "ffn2.b", (h,), "bias", f))
            t.append(TensorDesc(p + "ln2.g", (h,), "ln_gamma", h))
            t.append(TensorDesc(p + "ln2.b", (h,), "ln_beta", h))
        t.append(TensorDesc("head.w", (self.n_classes, h), "linear", h))
        t.append(TensorDesc("head.b", (self.n_classes,), "bias", h))
        return t

    def norms(self) -> List[Tuple[str, int]]:
        return []      # LayerNorm computes its statistics per token at run time
