"""Pins of the CPU oracle against things other than itself (no GPU needed).

What fixes each part: definitional Python loops on tiny inputs, PyTorch CPU
library ops, algebraic special cases, and the invariants SubNetAct states
(in place == extracted; max cfg == full SuperNet; skipped block == identity;
SubnetNorm uses the chosen subnet's row).
"""
import copy

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import synth
from oracle import brute
from oracle import primitives as P


def rng(i):
    return np.random.default_rng(1000 + i)


# ------------------------------------------------------------------ strided sums vs brute force
@pytest.mark.parametrize("k,stride,h,w", [(1, 1, 5, 4), (1, 2, 5, 5), (3, 1, 5, 6), (3, 2, 7, 5),
                                          (5, 2, 6, 7), (7, 2, 9, 8), (7, 1, 4, 4)])
def test_conv_sliced_vs_brute(k, stride, h, w):
    g = rng(k * 10 + stride)
    kmax, cmax, rmax = 6, 5, 7 if k > 3 else k
    wt = g.standard_normal((kmax, rmax, rmax, cmax)).astype(np.float32)
    ca, ka = 3, 4
    x = g.standard_normal((2, h, w, ca))
    y = P.conv2d_sliced(x, wt, ka, k, stride)
    o = (rmax - k) // 2
    yb = brute.conv2d(x, wt[:ka, o:o + k, o:o + k, :ca], stride, k // 2)
    assert y.shape == yb.shape
    np.testing.assert_allclose(y, yb, rtol=0, atol=1e-12)


@pytest.mark.parametrize("k,stride", [(3, 1), (3, 2), (5, 1), (5, 2), (7, 1), (7, 2)])
def test_depthwise_centre_slice_vs_brute(k, stride):
    g = rng(k + stride)
    wt = g.standard_normal((7, 7, 6)).astype(np.float32)
    x = g.standard_normal((2, 7, 6, 4))
    y = P.depthwise_sliced(x, wt, k, stride)
    o = (7 - k) // 2
    yb = brute.depthwise(x, wt[o:o + k, o:o + k, :4], stride, k // 2)
    np.testing.assert_allclose(y, yb, rtol=0, atol=1e-12)


def test_linear_sliced_vs_brute():
    g = rng(3)
    wt = g.standard_normal((9, 11)).astype(np.float32)
    b = g.standard_normal(9).astype(np.float32)
    x = g.standard_normal((5, 7))
    y = P.linear_sliced(x, wt, 6, b)
    np.testing.assert_allclose(y, brute.linear(x, wt[:6, :7], b[:6]), rtol=0, atol=1e-12)


def test_maxpool_vs_brute():
    x = rng(4).standard_normal((2, 7, 6, 3))
    np.testing.assert_array_equal(P.maxpool_3x3_s2(x), brute.maxpool_3x3_s2(x))
    xe = rng(5).standard_normal((1, 8, 8, 2))
    np.testing.assert_array_equal(P.maxpool_3x3_s2(xe), brute.maxpool_3x3_s2(xe))


# ------------------------------------------------------------------ library routines
@pytest.mark.parametrize("k,stride,h", [(1, 1, 14), (1, 2, 14), (3, 1, 15), (3, 2, 14), (7, 2, 33)])
def test_conv_vs_torch(k, stride, h):
    g = rng(20 + k)
    wt = g.standard_normal((40, k, k, 24)).astype(np.float32)
    x = g.standard_normal((3, h, h + 1, 16))
    y = P.conv2d_sliced(x, wt, 32, k, stride)
    yt = F.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2),
                  torch.from_numpy(wt[:32, :, :, :16].copy()).double().permute(0, 3, 1, 2),
                  stride=stride, padding=k // 2).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(y, yt, rtol=0, atol=1e-11)


def test_depthwise_vs_torch():
    g = rng(30)
    wt = g.standard_normal((7, 7, 24)).astype(np.float32)
    x = g.standard_normal((2, 13, 12, 16))
    for k in (3, 5, 7):
        for st in (1, 2):
            o = (7 - k) // 2
            wk = torch.from_numpy(wt[o:o + k, o:o + k, :16].copy()).double().permute(2, 0, 1).unsqueeze(1)
            yt = F.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), wk, stride=st, padding=k // 2, groups=16)
            np.testing.assert_allclose(P.depthwise_sliced(x, wt, k, st), yt.permute(0, 2, 3, 1).numpy(),
                                       rtol=0, atol=1e-12)


def test_conv_1x1_is_matrix_product():
    g = rng(31)
    wt = g.standard_normal((12, 1, 1, 10)).astype(np.float32)
    x = g.standard_normal((2, 4, 5, 8))
    y = P.conv2d_sliced(x, wt, 9, 1, 1)
    ref = x.reshape(-1, 8) @ wt[:9, 0, 0, :8].astype(np.float64).T
    np.testing.assert_allclose(y.reshape(-1, 9), ref, rtol=0, atol=1e-12)


def test_conv_delta_kernel_is_identity():
    x = rng(32).standard_normal((1, 6, 7, 4))
    for kmax in (3, 7):
        wt = np.zeros((4, kmax, kmax, 4), dtype=np.float32)
        for c in range(4):
            wt[c, kmax // 2, kmax // 2, c] = 1.0
        for k in range(1, kmax + 1, 2):
            np.testing.assert_array_equal(P.conv2d_sliced(x, wt, 4, k, 1), x)


def test_pool_and_norm_closed_forms():
    x = np.full((2, 5, 3, 4), 2.5)
    np.testing.assert_allclose(P.global_avg_pool(x), 2.5)
    st = np.zeros((3, 4, 6), dtype=np.float32)
    st[:, 0] = [[0.5] * 6, [0.0] * 6, [1.0] * 6]           # mean
    st[:, 1] = [[4.0] * 6, [1.0 - 1e-5] * 6, [0.25] * 6]   # var
    st[:, 2] = [[2.0] * 6, [1.0] * 6, [3.0] * 6]           # gamma
    st[:, 3] = [[-1.0] * 6, [0.0] * 6, [0.5] * 6]          # beta
    y0 = P.subnet_norm(x, st, 0)
    np.testing.assert_allclose(y0, 2.0 * (2.5 - 0.5) / np.sqrt(4.0 + 1e-5) - 1.0, rtol=1e-12)
    xr = rng(33).standard_normal((2, 5, 3, 4))
    np.testing.assert_allclose(P.subnet_norm(xr, st, 1), xr, rtol=0, atol=1e-7)   # identity row
    y2 = P.subnet_norm(x, st, 2)
    np.testing.assert_allclose(y2, 3.0 * (2.5 - 1.0) / np.sqrt(0.25 + 1e-5) + 0.5, rtol=1e-12)
    # against the library's inference-mode batch norm
    s = synth.make_stats(synth.TinySpec(), 4, 5)["s1.b0.sn"]
    xx = rng(34).standard_normal((2, 3, 3, 48))
    t = torch.from_numpy
    ref = F.batch_norm(t(xx).permute(0, 3, 1, 2), t(s[2, 0, :48]).double(), t(s[2, 1, :48]).double(),
                       t(s[2, 2, :48]).double(), t(s[2, 3, :48]).double(), False, eps=1e-5)
    np.testing.assert_allclose(P.subnet_norm(xx, s, 2), ref.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-12)


def test_activation_closed_forms():
    v = np.array([-4.0, -3.0, -1.0, 0.0, 1.0, 3.0, 5.0])
    np.testing.assert_allclose(P.hardswish(v), [0, 0, -1 * 2 / 6, 0, 4 / 6, 3, 5])
    np.testing.assert_allclose(P.hardsigmoid(v), [0, 0, 2 / 6, 0.5, 4 / 6, 1, 1])
    np.testing.assert_allclose(P.relu(v), [0, 0, 0, 0, 1, 3, 5])
    assert P.gelu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(P.gelu(np.array([1.0, -1.0])), [0.8413447460685429, -0.15865525393145707], rtol=1e-12)
    x = rng(35).standard_normal((4, 9))
    np.testing.assert_allclose(P.gelu(x), F.gelu(torch.from_numpy(x)).numpy(), atol=1e-14)
    np.testing.assert_allclose(P.softmax(x).sum(-1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(P.softmax(x), F.softmax(torch.from_numpy(x), -1).numpy(), atol=1e-15)
    y = P.layer_norm(x, np.ones(9, np.float32), np.zeros(9, np.float32), eps=0.0)
    np.testing.assert_allclose(y.mean(-1), 0, atol=1e-14)
    np.testing.assert_allclose(y.var(-1), 1, rtol=1e-12)
    gm, bt = rng(36).standard_normal(9).astype(np.float32), rng(37).standard_normal(9).astype(np.float32)
    ref = F.layer_norm(torch.from_numpy(x), (9,), torch.from_numpy(gm).double(), torch.from_numpy(bt).double(), 1e-5)
    np.testing.assert_allclose(P.layer_norm(x, gm, bt), ref.numpy(), atol=1e-13)


def test_round_bf16():
    a = rng(38).standard_normal(20000).astype(np.float32) * np.float32(37.0)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(P.round_bf16(a.astype(np.float64)), ref)
    # ties go to the even mantissa: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert P.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert P.round_bf16(np.array([1.0 + 2.0 ** -7 + 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert P.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -30]))[0] == 1.0 + 2.0 ** -7
    # one rounding, not two: this value rounds up in one step, but to 1.0 via fp32 first
    v = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert P.round_bf16(np.array([v]))[0] == 1.0 + 2.0 ** -7
    np.testing.assert_array_equal(P.round_bf16(np.array([0.0, -0.0, 3.0, -2.5])), [0.0, -0.0, 3.0, -2.5])
    np.testing.assert_array_equal(P.round_fp32(np.array([1.0 + 2.0 ** -30])), [1.0])


# ------------------------------------------------------------------ WeightSlice
def test_weightslice_ignores_weights_outside_the_slice():
    g = rng(40)
    wt = g.standard_normal((16, 7, 7, 12)).astype(np.float32)
    x = g.standard_normal((1, 6, 6, 8))
    base = P.conv2d_sliced(x, wt, 10, 3, 1)
    w2 = wt.copy()
    w2[10:] += 5.0                       # unused output channels
    w2[:, :, :, 8:] -= 3.0               # unused input channels
    w2[:, :2] = 9.0; w2[:, 5:] = 9.0     # rows outside the centre window
    w2[:, :, :2] = 9.0; w2[:, :, 5:] = 9.0
    np.testing.assert_array_equal(P.conv2d_sliced(x, w2, 10, 3, 1), base)
    w3 = wt.copy()
    w3[9, 3, 3, 7] += 1.0                # last element inside the slice
    assert np.abs(P.conv2d_sliced(x, w3, 10, 3, 1) - base).max() > 1e-3
    w4 = wt.copy()
    w4[0, 2, 4, 0] += 1.0                # corner of the 3x3 window
    assert np.abs(P.conv2d_sliced(x, w4, 10, 3, 1) - base).max() > 1e-3


# ------------------------------------------------------------------ whole-network invariants
SMALL_RESNET = synth.ResNetSpec(n_classes=12, stem_ch=16, stage_ch=(32, 64, 96, 128),
                                max_depth=(3, 3, 4, 3), res_choices=(40, 48, 57))
SMALL_TF = synth.TransformerSpec(n_classes=7, hidden=64, n_heads=4, head_dim=16, ffn=128,
                                 max_layers=4, seq_len=9, depth_choices=(2, 3, 4))
SPECS = [(synth.TinySpec(), 8, 3), (SMALL_RESNET, 6, 2), (synth.MBV3Spec(res_choices=(40, 48, 57)), 5, 2),
         (SMALL_TF, 6, 2)]


def _setup(spec, n):
    W = synth.make_weights(spec, 2312)
    S = synth.make_stats(spec, n, 2312)
    C = synth.enumerate_cfgs(spec, n, 16733)
    return W, S, C


@pytest.mark.parametrize("spec,n,bs", SPECS, ids=[s[0].family for s in SPECS])
@pytest.mark.parametrize("mode", ["f64", "native"])
def test_inplace_equals_extracted_subnet(spec, n, bs, mode):
    """Serving in place gives what the statically extracted subnet gives."""
    W, S, C = _setup(spec, n)
    mode = spec.dtype if mode == "native" else mode
    for c in C:
        x = synth.make_inputs(spec, bs, c.in_h, c.in_w, 7)
        a = oracle.forward(spec, W, S, c, x, mode)
        T, N = oracle.extract_subnet(spec, W, S, c)
        b = oracle.standalone_forward(spec, T, N, x, mode)
        scale = np.abs(b).max()
        tol = 1e-11 if mode == "f64" else (2e-7 if mode == "fp32" else 2e-3)
        assert np.abs(a - b).max() <= tol * scale, (c.subnet_id, np.abs(a - b).max() / scale)


@pytest.mark.parametrize("spec,n,bs", SPECS, ids=[s[0].family for s in SPECS])
def test_max_cfg_equals_full_supernet(spec, n, bs):
    """The largest cfg is the SuperNet itself: run the unsliced tensors as an ordinary network."""
    W, S, C = _setup(spec, n)
    c = C[-1]
    x = synth.make_inputs(spec, bs, c.in_h, c.in_w, 8)
    full_T = {k: v for k, v in W.items()}
    # an elastic depthwise kernel at max size is the stored 7x7 itself, so nothing is cut
    full_N = {k: v[c.subnet_id] for k, v in S.items()}
    b = oracle.standalone_forward(spec, full_T, full_N, x, "f64")
    a = oracle.forward(spec, W, S, c, x, "f64")
    assert np.abs(a - b).max() <= 1e-11 * np.abs(b).max()


def test_skipped_block_is_identity_tiny():
    spec = synth.TinySpec()
    W, S, C = _setup(spec, 8)
    x = synth.make_inputs(spec, 2, 32, 32, 9)
    short = copy.deepcopy(C[0]); short.depth = [1, 1, 1]
    long = copy.deepcopy(short); long.depth = [2, 1, 2]
    W2 = {k: v.copy() for k, v in W.items()}
    S2 = {k: v.copy() for k, v in S.items()}
    for nm in ("s0.b1", "s2.b1"):        # make the extra blocks add exactly zero
        W2[nm + ".w"][:] = 0
        S2[nm + ".sn"][:, 0] = 0; S2[nm + ".sn"][:, 3] = -1.0
    np.testing.assert_array_equal(oracle.forward(spec, W2, S2, long, x), oracle.forward(spec, W2, S2, short, x))
    assert np.abs(oracle.forward(spec, W, S, long, x) - oracle.forward(spec, W, S, short, x)).max() > 1e-3
    # a kept-out block's weights and statistics are never read
    W3 = {k: v.copy() for k, v in W.items()}
    W3["s0.b1.w"][:] = np.nan
    S3 = {k: v.copy() for k, v in S.items()}
    S3["s0.b1.sn"][:] = np.nan
    np.testing.assert_array_equal(oracle.forward(spec, W3, S3, short, x), oracle.forward(spec, W, S, short, x))


def test_skipped_block_is_identity_resnet():
    spec = SMALL_RESNET
    W, S, C = _setup(spec, 6)
    base = copy.deepcopy(C[2])
    s = 2
    d = base.depth[s]
    if d == spec.max_depth[s]:
        base.depth[s] = d = d - 1
        base.block_mid_ch[s][d] = 0
    longer = copy.deepcopy(base)
    longer.depth[s] = d + 1
    longer.block_mid_ch[s][d] = 16
    x = synth.make_inputs(spec, 2, base.in_h, base.in_w, 10)
    W2 = {k: v.copy() for k, v in W.items()}
    S2 = {k: v.copy() for k, v in S.items()}
    W2[f"s{s}.b{d}.conv3.w"][:] = 0      # residual branch contributes exactly zero
    S2[f"s{s}.b{d}.sn3"][:, 0] = 0; S2[f"s{s}.b{d}.sn3"][:, 3] = 0
    for mode in ("f64", "bf16"):
        np.testing.assert_array_equal(oracle.forward(spec, W2, S2, longer, x, mode),
                                      oracle.forward(spec, W2, S2, base, x, mode))
    assert np.abs(oracle.forward(spec, W, S, longer, x) - oracle.forward(spec, W, S, base, x)).max() > 0


@pytest.mark.parametrize("spec,n,bs", SPECS[:3], ids=[s[0].family for s in SPECS[:3]])
def test_subnetnorm_uses_the_chosen_row(spec, n, bs):
    W, S, C = _setup(spec, n)
    c = C[1]
    x = synth.make_inputs(spec, bs, c.in_h, c.in_w, 11)
    a = oracle.forward(spec, W, S, c, x)
    wrong = copy.deepcopy(c); wrong.subnet_id = (c.subnet_id + 1) % n
    assert np.abs(oracle.forward(spec, W, S, wrong, x) - a).max() > 1e-3 * np.abs(a).max()
    S2 = {k: v.copy() for k, v in S.items()}
    for v in S2.values():                # other subnets' rows are never read
        v[np.arange(n) != c.subnet_id] = np.nan
    np.testing.assert_array_equal(oracle.forward(spec, W, S2, c, x), a)


@pytest.mark.parametrize("spec,n,bs", SPECS, ids=[s[0].family for s in SPECS])
def test_requests_are_independent_of_batch_mates(spec, n, bs):
    W, S, C = _setup(spec, n)
    c = C[n // 2]
    x = synth.make_inputs(spec, 3, c.in_h, c.in_w, 12)
    a = oracle.forward(spec, W, S, c, x)
    for r in range(3):
        np.testing.assert_array_equal(oracle.forward(spec, W, S, c, x[r:r + 1]), a[r:r + 1])


def test_tiny_cfg_whole_net_brute_force():
    """Tiny net, smallest cfg, one image: every layer by definitional Python loops."""
    spec = synth.TinySpec(stage_ch=(16, 16, 24), stem_ch=8, res_choices=(8,))
    W, S, C = _setup(spec, 4)
    c = C[1]
    x = synth.make_inputs(spec, 1, 8, 8, 13).astype(np.float64)
    i = c.subnet_id

    def sn(t, name):
        st = S[name][i].astype(np.float64)
        out = np.empty_like(t)
        for ch in range(t.shape[-1]):
            out[..., ch] = st[2, ch] * (t[..., ch] - st[0, ch]) / np.sqrt(st[1, ch] + 1e-5) + st[3, ch]
        return out

    a = np.maximum(sn(brute.conv2d(x, W["stem.w"][:c.stage_out_ch[0]], 1, 1), "stem.sn"), 0)
    for s in range(3):
        co = c.stage_out_ch[1 + s]
        for j in range(c.depth[s]):
            w = W[f"s{s}.b{j}.w"][:co, :, :, :a.shape[-1]]
            y = np.maximum(sn(brute.conv2d(a, w, 2 if j == 0 else 1, 1), f"s{s}.b{j}.sn"), 0)
            a = a + y if j > 0 else y
    pooled = a.sum(axis=(1, 2)) / (a.shape[1] * a.shape[2])
    ref = brute.linear(pooled, W["head.w"][:, :a.shape[-1]], W["head.b"])
    got = oracle.forward(spec, W, S, c, x, "f64")
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-11 * np.abs(ref).max())


def test_oracle_matches_its_frozen_outputs():
    import importlib.util
    import os
    here = os.path.join(os.path.dirname(__file__), "golden")
    sp = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_golden.py"))
    mg = importlib.util.module_from_spec(sp); sp.loader.exec_module(mg)
    stored = [l.split() for l in open(os.path.join(here, "oracle_logits.txt")) if not l.startswith("#")]
    fresh = [r.split() for r in mg.rows()]
    assert len(stored) == len(fresh)
    for a, b in zip(stored, fresh):
        assert a[:2] == b[:2]
        np.testing.assert_allclose([float(v) for v in a[2:]], [float(v) for v in b[2:]], rtol=1e-9)
