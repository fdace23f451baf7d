"""Pins of the oracle's SubnetNorm calibration (no GPU): the library's training-mode batch norm,
closed forms of what a calibrated layer must output, and the consistency of "calibrate, then serve"."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import synth
from oracle import primitives as P
from tests.test_oracle_pins import SPECS, _setup

CONV_SPECS = [s for s in SPECS if s[0].family != "transformer"]


def test_calibrating_norm_matches_torch_batch_norm_in_training_mode():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, 5, 4, 8)) * 2.0 + 0.7
    table = np.zeros((4, 4, 12), np.float32)
    table[:, 2] = rng.uniform(0.5, 1.5, (4, 12))
    table[:, 3] = rng.standard_normal((4, 12))
    before = table.copy()
    y = P.subnet_norm(x, P.CalibrationTable(table), 2)
    xt = torch.from_numpy(x).permute(0, 3, 1, 2)
    rm, rv = torch.zeros(8, dtype=torch.float64), torch.ones(8, dtype=torch.float64)
    ref = F.batch_norm(xt, rm, rv, torch.from_numpy(table[2, 2, :8].astype(np.float64)),
                       torch.from_numpy(table[2, 3, :8].astype(np.float64)), training=True, momentum=1.0, eps=P.EPS)
    ref = ref.permute(0, 2, 3, 1).numpy()
    assert np.abs(y - ref).max() < 1e-5                      # fp32 storage of the statistics is the only difference
    assert np.abs(table[2, 0, :8] - rm.numpy()).max() < 1e-6  # running mean with momentum 1 = batch mean
    n = 3 * 5 * 4
    assert np.abs(table[2, 1, :8] * n / (n - 1) - rv.numpy()).max() < 1e-5   # torch's running var is the unbiased one
    # only (row 2, mean / var, leading 8 channels) were written
    mask = np.ones_like(table, bool)
    mask[2, 0:2, :8] = False
    assert np.array_equal(table[mask], before[mask])


def test_calibrated_layer_output_has_mean_beta_and_scale_gamma():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((4, 6, 6, 16)) * np.linspace(0.5, 3.0, 16) + np.linspace(-2, 2, 16)
    table = np.zeros((1, 4, 16), np.float32)
    table[0, 2] = rng.uniform(0.5, 1.5, 16)
    table[0, 3] = rng.standard_normal(16)
    y = P.subnet_norm(x, P.CalibrationTable(table), 0).reshape(-1, 16)
    g, b = table[0, 2].astype(np.float64), table[0, 3].astype(np.float64)
    v = table[0, 1].astype(np.float64)
    assert np.abs(y.mean(axis=0) - b).max() < 1e-5
    assert np.abs(y.std(axis=0) - g * np.sqrt(v / (v + P.EPS))).max() < 1e-5


@pytest.mark.parametrize("spec,n,bs", CONV_SPECS, ids=[s[0].family for s in CONV_SPECS])
def test_calibrate_then_serve_reproduces_the_calibration_forward(spec, n, bs):
    W, S, C = _setup(spec, n)
    for c in (C[0], C[len(C) // 2], C[-1]):
        x = synth.make_inputs(spec, max(bs, 3), c.in_h, c.in_w, 9)
        new, logits = oracle.calibrate(spec, W, S, c, x)
        again = oracle.forward(spec, W, new, c, x)
        assert np.array_equal(logits, again)
        # other subnets' rows, gamma and beta are untouched; the calibrated rows did change
        changed = 0
        for name in S:
            keep = np.ones(S[name].shape, bool)
            keep[c.subnet_id, 0:2] = False
            assert np.array_equal(new[name][keep], S[name][keep])
            changed += not np.array_equal(new[name][c.subnet_id, 0:2], S[name][c.subnet_id, 0:2])
        assert changed >= 3
        # the input statistics table was not modified in place
        S2 = synth.make_stats(spec, n, 2312)
        assert all(np.array_equal(S[k], S2[k]) for k in S)


def test_layers_of_skipped_blocks_keep_their_rows():
    """LayerSelect: a block the subnet does not run is never calibrated."""
    spec, n, bs = CONV_SPECS[0]
    W, S, C = _setup(spec, n)
    c = min(C, key=lambda c: sum(c.depth))
    x = synth.make_inputs(spec, 3, c.in_h, c.in_w, 10)
    new, _ = oracle.calibrate(spec, W, S, c, x)
    skipped = [name for name in S if name.startswith("s") and ".b" in name
               and int(name.split(".b")[1].split(".")[0]) >= c.depth[int(name[1:].split(".")[0])]]
    assert skipped
    for name in skipped:
        assert np.array_equal(new[name], S[name]), name


def test_calibration_in_the_first_layer_by_hand():
    """First SubnetNorm of the tiny net: mean / variance of the sliced stem conv output, computed here
    with the independent brute-force convolution."""
    from oracle import brute
    spec, n, bs = [s for s in CONV_SPECS if s[0].family == "tiny"][0]
    W, S, C = _setup(spec, n)
    c = C[1]
    x = synth.make_inputs(spec, 2, c.in_h, c.in_w, 12)
    new, _ = oracle.calibrate(spec, W, S, c, x, "f64")
    k = c.stage_out_ch[0]
    xs = np.asarray(x, np.float64)
    y = brute.conv2d(xs, W["stem.w"][:k, :, :, :xs.shape[-1]], 1, 1).reshape(-1, k)   # the slice, copied out
    assert np.abs(new["stem.sn"][c.subnet_id, 0, :k] - y.mean(axis=0)).max() < 1e-6
    assert np.abs(new["stem.sn"][c.subnet_id, 1, :k] - y.var(axis=0)).max() < 1e-6
