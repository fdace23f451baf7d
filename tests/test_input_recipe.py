"""Facts about the synthetic input recipe that the parity bars rest on (no GPU needed).

The benchmark configs ask for weights N(0, 2/fan_in).  The MBV3-shaped family is drawn with
N(0, 1/fan_in) instead; this file shows why on the oracle alone: with gain 2 the deepest cfg of the
benchmark SuperNet is so ill-conditioned that the oracle's own bf16-storage forward and its fp64
forward disagree by far more than the 2e-2 parity bar, so no implementation could be held to that
bar; with gain 1 the two agree to a few bf16 ulps over the whole cfg range.
"""
import dataclasses

import numpy as np
import pytest

import oracle
import synth
from helpers import rel_err


def _storage_vs_exact(spec, ci, n_cfgs=16):
    W = synth.make_weights(spec, 2312)
    S = synth.make_stats(spec, n_cfgs, 2312)
    C = synth.enumerate_cfgs(spec, n_cfgs, 16733)
    c = C[ci]
    x = synth.make_inputs(spec, 2, c.in_h, c.in_w, 7)
    lo = oracle.forward(spec, W, S, c, x, "bf16")
    hi = oracle.forward(spec, W, S, c, x, "f64")
    return float(rel_err(lo, hi).max()), float(np.abs(hi).max()), c


def test_mbv3_gain_2_is_ill_conditioned_at_max_depth_and_gain_1_is_not():
    spec1 = synth.MBV3Spec()
    assert spec1.init_gain == 1.0                       # what every MBV3 test and the benchmark use
    spec2 = dataclasses.replace(spec1, init_gain=2.0)
    e2, mag2, c = _storage_vs_exact(spec2, 15)
    assert tuple(c.depth) == tuple(spec1.max_depth)     # the last cfg is the full-depth one
    e1, mag1, _ = _storage_vs_exact(spec1, 15)
    # gain 2: storage rounding alone moves the logits by > 10 % and they reach 1e4..1e5
    assert e2 > 0.10 and mag2 > 1e3, (e2, mag2)
    # gain 1: well inside the parity bar, logits of order one
    assert e1 < 1e-2 and mag1 < 100, (e1, mag1)


@pytest.mark.parametrize("ci", [0, 8])
def test_mbv3_gain_only_matters_for_the_deep_cfgs(ci):
    """The shallower cfgs are well conditioned under either gain: the change of recipe is about the
    full-depth cfg, not a way to loosen every comparison."""
    for gain in (1.0, 2.0):
        e, _, _ = _storage_vs_exact(dataclasses.replace(synth.MBV3Spec(), init_gain=gain), ci)
        assert e < 2e-2, (gain, ci, e)


def test_other_families_keep_gain_2():
    for spec in (synth.TinySpec(), synth.ResNetSpec(), synth.TransformerSpec()):
        assert float(getattr(spec, "init_gain", 2.0)) == 2.0
    # and the ResNet-shaped max cfg is well conditioned with it (small shape: same wiring, seconds on the CPU)
    spec = synth.ResNetSpec(n_classes=24, stem_ch=16, stage_ch=(32, 64, 96, 128), max_depth=(3, 3, 4, 3),
                            res_choices=(40, 48, 57))
    e, _, _ = _storage_vs_exact(spec, 7, n_cfgs=8)
    assert e < 1e-2, e
