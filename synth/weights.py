"""Random-init SuperNet weights, SubnetNorm statistics and request inputs.

Distributions (second parameter of N(.,.) is a variance):
  conv / depthwise / linear weights  N(0, gain / fan_in), fan_in at max size; gain = 2 except
                                     for the MBV3 family, whose spec sets gain = 1: with gain 2
                                     its un-rectified project -> expand pairs compound to 1e4-scale
                                     activations that saturate the squeeze-excite hard-sigmoid
                                     gates, and the forward becomes ill-conditioned (a one-ulp input
                                     change moves the logits by > 10 %)
  biases                             N(0, 0.01)
  SubnetNorm per (subnet, layer):    mean N(0, 0.1), var U(0.5, 1.5),
                                     gamma U(0.5, 1.5), beta N(0, 0.1)
  LayerNorm gamma U(0.5, 1.5), beta N(0, 0.1) (shared by all subnets)
  inputs                             U(-1, 1) (tiny) or N(0, 1)
For a bf16 family the weight and input values are drawn in fp32 and rounded to
bf16 once here (round-to-nearest-even, torch's conversion), then handed out as
fp32 arrays holding bf16-representable values; biases, statistics and LayerNorm
parameters stay fp32.
"""
import numpy as np
import torch

from .rng import keyed_rng

STAT_FIELDS = ("mean", "var", "gamma", "beta")


def to_bf16_values(a: np.ndarray) -> np.ndarray:
    """fp32 array -> fp32 array whose values are bf16-representable (RNE)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def make_weights(spec, seed: int) -> dict:
    out = {}
    gain = float(getattr(spec, "init_gain", 2.0))
    for td in spec.tensors():
        g = keyed_rng(seed, "w:" + td.name)
        if td.kind in ("conv", "dw", "linear"):
            a = g.standard_normal(td.shape, dtype=np.float32) * np.float32(np.sqrt(gain / td.fan_in))
            if spec.dtype == "bf16":
                a = to_bf16_values(a)
        elif td.kind == "bias":
            a = g.standard_normal(td.shape, dtype=np.float32) * np.float32(0.1)
        elif td.kind == "ln_gamma":
            a = g.uniform(0.5, 1.5, td.shape).astype(np.float32)
        elif td.kind == "ln_beta":
            a = g.standard_normal(td.shape, dtype=np.float32) * np.float32(np.sqrt(0.1))
        else:
            raise ValueError(td.kind)
        out[td.name] = np.ascontiguousarray(a, dtype=np.float32)
    return out


def make_stats(spec, n_subnets: int, seed: int) -> dict:
    """name -> fp32 [n_subnets][4][C_max], fields in STAT_FIELDS order."""
    out = {}
    for name, c in spec.norms():
        g = keyed_rng(seed, "sn:" + name)
        a = np.empty((n_subnets, 4, c), dtype=np.float32)
        a[:, 0] = g.standard_normal((n_subnets, c)) * np.sqrt(0.1)
        a[:, 1] = g.uniform(0.5, 1.5, (n_subnets, c))
        a[:, 2] = g.uniform(0.5, 1.5, (n_subnets, c))
        a[:, 3] = g.standard_normal((n_subnets, c)) * np.sqrt(0.1)
        out[name] = a
    return out


def make_inputs(spec, n: int, in_h: int, in_w: int, seed: int, tag: str = "x") -> np.ndarray:
    """Request inputs: NHWC images, or [n][seq][hidden] token embeddings."""
    g = keyed_rng(seed, f"in:{tag}:{n}:{in_h}:{in_w}")
    if spec.family == "transformer":
        a = g.standard_normal((n, spec.seq_len, spec.hidden), dtype=np.float32)
    elif spec.family == "tiny":
        a = g.uniform(-1.0, 1.0, (n, in_h, in_w, spec.in_ch)).astype(np.float32)
    else:
        a = g.standard_normal((n, in_h, in_w, spec.in_ch), dtype=np.float32)
    if spec.dtype == "bf16":
        a = to_bf16_values(a)
    return a
