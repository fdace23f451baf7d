"""Parity of the HIP path against the CPU oracle, through the C ABI (needs an MI355X)."""
import copy
import sys

import numpy as np
import pytest

import synth
from helpers import setup, check_parity, rel_err

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def to_dev(torch, spec, x):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if spec.dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.to("cuda:0")


def run_single(torch, net, spec, cfg, x):
    out = net.forward([cfg], np.zeros(len(x), np.int32), to_dev(torch, spec, x))
    torch.cuda.synchronize()
    return out.cpu().numpy()


# ------------------------------------------------------------------ cfg 1: tiny conv net, fp32
def test_tiny_all_cfgs(torch_mod):
    import oracle
    import paper_2312_16733_amd as sna
    torch = torch_mod
    spec = synth.TinySpec()
    W, S, C = setup(spec, 8)
    net = sna.Supernet(spec, W, S, 8, 8)
    worst = 0.0
    for c in C:
        x = synth.make_inputs(spec, 4, c.in_h, c.in_w, 7)
        say("tiny cfg", c.subnet_id, c.depth, c.stage_out_ch)
        got = run_single(torch, net, spec, c, x)
        e, _ = check_parity(got, oracle.forward(spec, W, S, c, x), "fp32", f"tiny cfg {c.subnet_id}")
        worst = max(worst, e)
    say("tiny worst rel err", worst)
    net.close()


# ------------------------------------------------------------------ cfg 2: ResNet-shaped, bf16
SMALL_RESNET = synth.ResNetSpec(n_classes=24, stem_ch=16, stage_ch=(32, 64, 96, 128),
                                max_depth=(3, 3, 4, 3), res_choices=(40, 48, 57))


def test_resnet_small_supernet_all_cfgs(torch_mod):
    """Small supernet: odd resolutions, ragged tiles, every cfg, batch 3."""
    import oracle
    import paper_2312_16733_amd as sna
    torch = torch_mod
    spec = SMALL_RESNET
    W, S, C = setup(spec, 8)
    net = sna.Supernet(spec, W, S, 8, 8)
    for c in C:
        x = synth.make_inputs(spec, 3, c.in_h, c.in_w, 7)
        say("resnet-small cfg", c.subnet_id, c.depth, c.stage_out_ch, c.in_h)
        got = run_single(torch, net, spec, c, x)
        e, und = check_parity(got, oracle.forward(spec, W, S, c, x), "bf16", f"small cfg {c.subnet_id}")
        say("   rel err %.3e undecided %d" % (e, und))
    net.close()


@pytest.fixture(scope="module")
def resnet_full(torch_mod):
    import paper_2312_16733_amd as sna
    spec = synth.ResNetSpec()
    W, S, C = setup(spec, 16)
    net = sna.Supernet(spec, W, S, 16, 64)
    yield spec, W, S, C, net
    net.close()


@pytest.mark.parametrize("ci,batch", [(0, 1), (0, 16), (5, 2), (9, 1), (12, 3), (15, 1), (15, 2)])
def test_resnet_full_supernet(torch_mod, resnet_full, ci, batch):
    import oracle
    torch = torch_mod
    spec, W, S, C, net = resnet_full
    c = C[ci]
    x = synth.make_inputs(spec, batch, c.in_h, c.in_w, 11)
    say("resnet cfg", ci, "batch", batch, "res", c.in_h, c.depth, c.stage_out_ch)
    got = run_single(torch, net, spec, c, x)
    e, und = check_parity(got, oracle.forward(spec, W, S, c, x), "bf16", f"resnet cfg {ci} b{batch}")
    say("   rel err %.3e undecided %d" % (e, und))


def test_resnet_every_benchmark_cfg(torch_mod, resnet_full):
    """All 16 benchmark cfgs at full size against the oracle at batch 1, and the smallest, median and
    largest at batch 16 (every request of the batch)."""
    import oracle
    torch = torch_mod
    spec, W, S, C, net = resnet_full
    worst = 0.0
    for ci, c in enumerate(C):
        for batch in ((1, 16) if ci in (0, len(C) // 2, len(C) - 1) else (1,)):
            x = synth.make_inputs(spec, batch, c.in_h, c.in_w, 60 + batch)
            say("resnet every-cfg: cfg", ci, "batch", batch, "res", c.in_h)
            got = run_single(torch, net, spec, c, x)
            e, und = check_parity(got, oracle.forward(spec, W, S, c, x), "bf16", f"resnet cfg {ci} b{batch}")
            worst = max(worst, e)
    say("resnet every-cfg worst rel err %.3e" % worst)


def test_resnet_batch64_sampled(torch_mod, resnet_full):
    """Full batch 64 in the benchmark's launch configuration; the oracle checks sampled requests
    one by one (per-request results do not depend on batch mates)."""
    import oracle
    torch = torch_mod
    spec, W, S, C, net = resnet_full
    for ci in (0, 7, 11, 15):
        c = C[ci]
        x = synth.make_inputs(spec, 64, c.in_h, c.in_w, 12)
        say("resnet b64 cfg", ci)
        got = run_single(torch, net, spec, c, x)
        assert np.all(np.isfinite(got))
        for r in (0, 37, 63):
            check_parity(got[r:r + 1], oracle.forward(spec, W, S, c, x[r:r + 1]), "bf16", f"b64 cfg {ci} req {r}")
        # batch independence on the GPU itself: request 5 alone gives the same bits
        alone = run_single(torch, net, spec, c, x[5:6])
        np.testing.assert_array_equal(alone[0], got[5])


# ------------------------------------------------------------------ cfg 4: mixed-subnet batch
def test_mixed_batch_equals_single_subnet_runs(torch_mod, resnet_full):
    import oracle
    torch = torch_mod
    spec, W, S, _, net = resnet_full
    C = synth.enumerate_cfgs(spec, 16, 16733, fixed_res=224)
    route = synth.zipf_assignment(64, 16, 4)
    x = synth.make_inputs(spec, 64, 224, 224, 13)
    say("mixed batch: groups", np.bincount(route, minlength=16).tolist())
    got = net.forward(C, route, to_dev(torch, spec, x))
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    for ci in sorted(set(route.tolist())):
        idx = np.nonzero(route == ci)[0]
        single = run_single(torch, net, spec, C[ci], x[idx])
        np.testing.assert_array_equal(got[idx], single, err_msg=f"cfg {ci}")
    # and against the oracle: the first request routed to each distinct cfg, plus the last request
    for r in sorted({int(np.nonzero(route == ci)[0][0]) for ci in set(route.tolist())} | {63}):
        say("mixed batch: request", r, "cfg", int(route[r]), "against the oracle")
        check_parity(got[r:r + 1], oracle.forward(spec, W, S, C[route[r]], x[r:r + 1]), "bf16", f"mixed req {r}")


def test_mixed_batch_mixed_resolutions_small(torch_mod):
    import oracle
    import paper_2312_16733_amd as sna
    torch = torch_mod
    spec = SMALL_RESNET
    W, S, C = setup(spec, 8)
    net = sna.Supernet(spec, W, S, 8, 16)
    route = np.array([3, 0, 3, 7, 1, 0, 7, 7, 5, 3, 0], dtype=np.int32)
    xs = [synth.make_inputs(spec, 1, C[ci].in_h, C[ci].in_w, 100 + r) for r, ci in enumerate(route)]
    flat = np.concatenate([a.ravel() for a in xs])
    got = net.forward(C, route, to_dev(torch, spec, flat))
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    for r, ci in enumerate(route):
        check_parity(got[r:r + 1], oracle.forward(spec, W, S, C[ci], xs[r]), "bf16", f"req {r} cfg {ci}")
    net.close()


# ------------------------------------------------------------------ operator behaviour on the GPU
def test_gpu_subnetnorm_row_and_layerselect(torch_mod, resnet_full):
    torch = torch_mod
    spec, W, S, C, net = resnet_full
    c = C[3]
    x = synth.make_inputs(spec, 1, c.in_h, c.in_w, 14)
    base = run_single(torch, net, spec, c, x)
    wrong = copy.deepcopy(c); wrong.subnet_id = 4
    assert rel_err(run_single(torch, net, spec, wrong, x), base).max() > 1e-2
    deeper = copy.deepcopy(c)
    s = next(i for i in range(4) if c.depth[i] < spec.max_depth[i])
    deeper.block_mid_ch[s][deeper.depth[s]] = 64
    deeper.depth[s] += 1
    assert rel_err(run_single(torch, net, spec, deeper, x), base).max() > 1e-3
    np.testing.assert_array_equal(run_single(torch, net, spec, c, x), base)     # deterministic


def test_error_paths(torch_mod, resnet_full):
    import paper_2312_16733_amd as sna
    torch = torch_mod
    spec, W, S, C, net = resnet_full
    x = to_dev(torch, spec, synth.make_inputs(spec, 1, C[0].in_h, C[0].in_w, 15))
    for field, val, status in [("subnet_id", 99, -5), ("in_h", 4000, -3)]:
        bad = copy.deepcopy(C[0]); setattr(bad, field, val)
        with pytest.raises(sna.SnaError) as ei:
            net.forward([bad], [0], x)
        assert ei.value.status == status
    bad = copy.deepcopy(C[0]); bad.depth[1] = 9
    with pytest.raises(sna.SnaError) as ei:
        net.forward([bad], [0], x)
    assert ei.value.status == -3
    bad = copy.deepcopy(C[0]); bad.block_mid_ch[0][0] = 36
    with pytest.raises(sna.SnaError) as ei:
        net.forward([bad], [0], x)
    assert ei.value.status == -4
    with pytest.raises(sna.SnaError) as ei:
        net.forward([C[0]], [0] * 65, x)
    assert ei.value.status == -6
    with pytest.raises(sna.SnaError) as ei:
        net.forward([C[0]], [1], x)
    assert ei.value.status == -6
    out = net.forward([C[0]], [], x)                      # empty call: nothing to do
    assert out.shape[0] == 0
    got = net.forward([C[0]], [0], x)                     # handle still usable
    torch.cuda.synchronize()
    assert np.all(np.isfinite(got.cpu().numpy()))


# ------------------------------------------------------------------ cfg 3: MBV3-shaped, bf16
@pytest.fixture(scope="module")
def mbv3_full(torch_mod):
    import paper_2312_16733_amd as sna
    spec = synth.MBV3Spec()
    W, S, C = setup(spec, 16)
    net = sna.Supernet(spec, W, S, 16, 64)
    yield spec, W, S, C, net
    net.close()


def test_mbv3_small_resolutions_all_cfgs(torch_mod):
    """Odd, small resolutions: ragged strips in the depthwise kernel, every kernel size and stride."""
    import oracle
    import paper_2312_16733_amd as sna
    torch = torch_mod
    spec = synth.MBV3Spec(res_choices=(40, 48, 57))
    W, S, C = setup(spec, 10)
    net = sna.Supernet(spec, W, S, 10, 8)
    for c in C:
        x = synth.make_inputs(spec, 3, c.in_h, c.in_w, 7)
        say("mbv3-small cfg", c.subnet_id, c.depth, c.in_h, [k[:d] for k, d in zip(c.block_kernel, c.depth)])
        got = run_single(torch, net, spec, c, x)
        e, und = check_parity(got, oracle.forward(spec, W, S, c, x), "bf16", f"mbv3 small cfg {c.subnet_id}")
        say("   rel err %.3e undecided %d" % (e, und))
    net.close()


@pytest.mark.parametrize("ci,batch", [(0, 1), (0, 16), (4, 2), (8, 3), (11, 1), (15, 1), (15, 4)])
def test_mbv3_full_supernet(torch_mod, mbv3_full, ci, batch):
    import oracle
    torch = torch_mod
    spec, W, S, C, net = mbv3_full
    c = C[ci]
    x = synth.make_inputs(spec, batch, c.in_h, c.in_w, 21)
    say("mbv3 cfg", ci, "batch", batch, "res", c.in_h, c.depth)
    got = run_single(torch, net, spec, c, x)
    e, und = check_parity(got, oracle.forward(spec, W, S, c, x), "bf16", f"mbv3 cfg {ci} b{batch}")
    say("   rel err %.3e undecided %d" % (e, und))


def test_mbv3_every_benchmark_cfg(torch_mod, mbv3_full):
    """All 16 benchmark cfgs at full size at batch 1; smallest, median and largest at batch 16."""
    import oracle
    torch = torch_mod
    spec, W, S, C, net = mbv3_full
    worst = 0.0
    for ci, c in enumerate(C):
        for batch in ((1, 16) if ci in (0, len(C) // 2, len(C) - 1) else (1,)):
            x = synth.make_inputs(spec, batch, c.in_h, c.in_w, 70 + batch)
            say("mbv3 every-cfg: cfg", ci, "batch", batch, "res", c.in_h)
            got = run_single(torch, net, spec, c, x)
            e, und = check_parity(got, oracle.forward(spec, W, S, c, x), "bf16", f"mbv3 cfg {ci} b{batch}")
            worst = max(worst, e)
    say("mbv3 every-cfg worst rel err %.3e" % worst)


def test_mbv3_batch64_sampled_and_mixed(torch_mod, mbv3_full):
    import oracle
    torch = torch_mod
    spec, W, S, C, net = mbv3_full
    c = C[9]
    x = synth.make_inputs(spec, 64, c.in_h, c.in_w, 22)
    got = run_single(torch, net, spec, c, x)
    for r in (0, 31, 63):
        check_parity(got[r:r + 1], oracle.forward(spec, W, S, c, x[r:r + 1]), "bf16", f"mbv3 b64 req {r}")
    np.testing.assert_array_equal(run_single(torch, net, spec, c, x[7:8])[0], got[7])
    # mixed-subnet batch with mixed resolutions
    route = synth.zipf_assignment(24, 16, 9)
    xs = [synth.make_inputs(spec, 1, C[ci].in_h, C[ci].in_w, 300 + r) for r, ci in enumerate(route)]
    flat = np.concatenate([a.ravel() for a in xs])
    mixed = net.forward(C, route, to_dev(torch, spec, flat))
    torch.cuda.synchronize()
    mixed = mixed.cpu().numpy()
    for ci in sorted(set(route.tolist())):
        idx = np.nonzero(route == ci)[0]
        single = run_single(torch, net, spec, C[ci], np.concatenate([xs[r] for r in idx]))
        np.testing.assert_array_equal(mixed[idx], single, err_msg=f"cfg {ci}")
    for r in sorted({int(np.nonzero(route == ci)[0][0]) for ci in set(route.tolist())} | {23}):
        check_parity(mixed[r:r + 1], oracle.forward(spec, W, S, C[route[r]], xs[r]), "bf16", f"mbv3 mixed req {r}")


# ------------------------------------------------------------------ cfg 5: transformer, bf16
@pytest.fixture(scope="module")
def tf_full(torch_mod):
    import paper_2312_16733_amd as sna
    spec = synth.TransformerSpec()
    W, S, C = setup(spec, 12)
    net = sna.Supernet(spec, W, S, 12, 32)
    yield spec, W, S, C, net
    net.close()


def run_tf(torch, net, spec, cfgs, route, x):
    hidden = torch.empty((len(route), spec.seq_len, spec.hidden), dtype=torch.bfloat16, device="cuda:0")
    out = net.forward(cfgs, route, to_dev(torch, spec, x), hidden=hidden)
    torch.cuda.synchronize()
    return out.cpu().numpy(), hidden.float().cpu().numpy()


@pytest.mark.parametrize("ci,batch", [(0, 2), (3, 1), (6, 3), (11, 2)])
def test_transformer_full_supernet(torch_mod, tf_full, ci, batch):
    import oracle
    torch = torch_mod
    spec, W, S, C, net = tf_full
    c = C[ci]
    x = synth.make_inputs(spec, batch, c.in_h, c.in_w, 31)
    say("transformer cfg", ci, "batch", batch, "depth", c.depth, c.block_mid_ch[0][:c.depth[0]], c.block_aux_ch[0][:c.depth[0]])
    got, hid = run_tf(torch, net, spec, [c], np.zeros(batch, np.int32), x)
    ref, ref_hid = oracle.forward(spec, W, S, c, x, return_hidden=True)
    e, und = check_parity(got, ref, "bf16", f"transformer cfg {ci}")
    he = np.abs(hid - ref_hid).max() / np.abs(ref_hid).max()
    say("   logits rel err %.3e undecided %d; hidden max err / max %.3e" % (e, und, he))
    assert he <= 2e-2


def test_transformer_every_benchmark_cfg(torch_mod, tf_full):
    """All 12 benchmark cfgs at batch 1 (logits and final hidden states); smallest, median, largest at batch 4."""
    import oracle
    torch = torch_mod
    spec, W, S, C, net = tf_full
    worst = 0.0
    for ci, c in enumerate(C):
        for batch in ((1, 4) if ci in (0, len(C) // 2, len(C) - 1) else (1,)):
            x = synth.make_inputs(spec, batch, c.in_h, c.in_w, 80 + batch)
            say("transformer every-cfg: cfg", ci, "batch", batch, "depth", c.depth[0])
            got, hid = run_tf(torch, net, spec, [c], np.zeros(batch, np.int32), x)
            ref, ref_hid = oracle.forward(spec, W, S, c, x, return_hidden=True)
            e, und = check_parity(got, ref, "bf16", f"transformer cfg {ci} b{batch}")
            assert np.abs(hid - ref_hid).max() <= 2e-2 * np.abs(ref_hid).max(), f"hidden states cfg {ci}"
            worst = max(worst, e)
    say("transformer every-cfg worst rel err %.3e" % worst)


def test_transformer_batch32_sampled_and_mixed(torch_mod, tf_full):
    import oracle
    torch = torch_mod
    spec, W, S, C, net = tf_full
    c = C[5]
    x = synth.make_inputs(spec, 32, c.in_h, c.in_w, 32)
    got, hid = run_tf(torch, net, spec, [c], np.zeros(32, np.int32), x)
    for r in (0, 17, 31):
        check_parity(got[r:r + 1], oracle.forward(spec, W, S, c, x[r:r + 1]), "bf16", f"tf b32 req {r}")
    alone, _ = run_tf(torch, net, spec, [c], np.zeros(1, np.int32), x[9:10])
    np.testing.assert_array_equal(alone[0], got[9])
    route = synth.zipf_assignment(32, 12, 3)
    mixed, mhid = run_tf(torch, net, spec, C, route, x)
    for ci in sorted(set(route.tolist())):
        idx = np.nonzero(route == ci)[0]
        single, shid = run_tf(torch, net, spec, [C[ci]], np.zeros(len(idx), np.int32), x[idx])
        np.testing.assert_array_equal(mixed[idx], single, err_msg=f"cfg {ci}")
        np.testing.assert_array_equal(mhid[idx], shid, err_msg=f"cfg {ci} hidden")
    for r in sorted({int(np.nonzero(route == ci)[0][0]) for ci in set(route.tolist())} | {30}):
        check_parity(mixed[r:r + 1], oracle.forward(spec, W, S, C[route[r]], x[r:r + 1]), "bf16", f"tf mixed req {r}")


def test_transformer_short_sequences(torch_mod):
    """Fewer than 128 tokens and a narrow model: masked keys, ragged query tiles."""
    import oracle
    import paper_2312_16733_amd as sna
    torch = torch_mod
    spec = synth.TransformerSpec(n_classes=16, hidden=128, n_heads=4, head_dim=64, ffn=256, max_layers=3,
                                 seq_len=45, depth_choices=(1, 2, 3))
    W, S, C = setup(spec, 6)
    net = sna.Supernet(spec, W, S, 6, 8)
    for c in C:
        x = synth.make_inputs(spec, 3, c.in_h, c.in_w, 33)
        got, hid = run_tf(torch, net, spec, [c], np.zeros(3, np.int32), x)
        ref, ref_hid = oracle.forward(spec, W, S, c, x, return_hidden=True)
        e, _ = check_parity(got, ref, "bf16", f"short tf cfg {c.subnet_id}")
        say("short tf cfg", c.subnet_id, "rel err %.3e" % e)
        assert np.abs(hid - ref_hid).max() <= 2e-2 * np.abs(ref_hid).max()
    net.close()


# ------------------------------------------------------------------ edge cases
def test_head_width_not_multiple_of_8(torch_mod):
    """n_classes = 10 on a bf16 family: the head leaves the MFMA path (rows of 10 floats are not
    16-byte granular) and runs on the direct kernel; logits rows are scattered with 2-byte copies."""
    import oracle
    import paper_2312_16733_amd as sna
    torch = torch_mod
    spec = synth.ResNetSpec(n_classes=10, stem_ch=16, stage_ch=(32, 64, 96, 128),
                            max_depth=(3, 3, 4, 3), res_choices=(33, 48))
    W, S, C = setup(spec, 6)
    net = sna.Supernet(spec, W, S, 6, 8)
    route = np.array([2, 5, 2, 0, 5], dtype=np.int32)
    xs = [synth.make_inputs(spec, 1, C[ci].in_h, C[ci].in_w, 400 + r) for r, ci in enumerate(route)]
    flat = np.concatenate([a.ravel() for a in xs])
    got = net.forward(C, route, to_dev(torch, spec, flat))
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    for r, ci in enumerate(route):
        check_parity(got[r:r + 1], oracle.forward(spec, W, S, C[ci], xs[r]), "bf16", f"req {r} cfg {ci}")
    net.close()


def test_sixteen_groups_and_too_many(torch_mod):
    """16 distinct cfgs in one call is the grouped-launch limit; a 17th is refused before any launch."""
    import oracle
    import paper_2312_16733_amd as sna
    torch = torch_mod
    spec = synth.TinySpec()
    W, S, C = setup(spec, 20)
    net = sna.Supernet(spec, W, S, 20, 32)
    x = synth.make_inputs(spec, 17, 32, 32, 41)
    route = np.arange(16, dtype=np.int32)
    got = net.forward(C, route, to_dev(torch, spec, x[:16]))
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    for r in range(16):
        check_parity(got[r:r + 1], oracle.forward(spec, W, S, C[r], x[r:r + 1]), "fp32", f"tiny req {r}")
    with pytest.raises(sna.SnaError) as ei:
        net.forward(C, np.arange(17, dtype=np.int32), to_dev(torch, spec, x))
    assert ei.value.status == -6
    net.close()


def test_max_batch_boundary_and_workspace_check(torch_mod):
    import ctypes
    import paper_2312_16733_amd as sna
    torch = torch_mod
    spec = synth.TinySpec()
    W, S, C = setup(spec, 8)
    net = sna.Supernet(spec, W, S, 8, 4)
    x = to_dev(torch, spec, synth.make_inputs(spec, 5, 32, 32, 42))
    out = net.forward([C[3]], [0] * 4, x)            # exactly max_batch
    torch.cuda.synchronize()
    assert np.all(np.isfinite(out.cpu().numpy()))
    with pytest.raises(sna.SnaError) as ei:
        net.forward([C[3]], [0] * 5, x)
    assert ei.value.status == -6
    # a workspace one byte short is refused at load
    ws = sna.lib().sna_workspace_bytes(ctypes.byref(net.arch), 8, 4)
    small = torch.empty(ws - 256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(sna.SnaError) as ei:
        sna.supernet_load(net.arch, net.weights.data_ptr(), net.weights.numel(), net.stats.data_ptr(),
                          net.stats.numel() * 4, 8, 4, small.data_ptr(), small.numel(), 0)
    assert ei.value.status == -7
    net.close()


def test_k_split_modes_give_identical_bits(torch_mod, resnet_full, tf_full):
    """Long reductions are summed in shape-determined chunks; whether one block walks the chunks
    or each chunk has its own blocks plus the reduction kernel must not change a bit."""
    torch = torch_mod
    spec, W, S, C, net = resnet_full
    try:
        for ci, batch in ((15, 3), (8, 16), (0, 64)):
            c = C[ci]
            x = synth.make_inputs(spec, batch, c.in_h, c.in_w, 14)
            outs = []
            for mode in (1, 2, 0, 3, 2):
                net.set_k_split(mode)
                say("k split mode", mode, "resnet cfg", ci, "batch", batch)
                outs.append(run_single(torch, net, spec, c, x))
                outs.append(run_single(torch, net, spec, c, x))       # replay: the tile counters are back at zero
            for o in outs[1:]:
                np.testing.assert_array_equal(outs[0], o)
    finally:
        net.set_k_split(0)
    spec, W, S, C, net = tf_full
    try:
        c = C[11]
        x = synth.make_inputs(spec, 4, c.in_h, c.in_w, 15)
        outs = []
        for mode in (1, 2, 0, 3):
            net.set_k_split(mode)
            say("k split mode", mode, "transformer cfg 11 batch 4")
            outs.append(run_tf(torch, net, spec, [c], np.zeros(4, np.int32), x))
        for o in outs[1:]:
            np.testing.assert_array_equal(outs[0][0], o[0])
            np.testing.assert_array_equal(outs[0][1], o[1])
    finally:
        net.set_k_split(0)


def test_tuned_tile_variants_do_not_change_bits(torch_mod):
    """sna_subnet_tune measures tile variants (and whether to spread K chunks over blocks) per layer
    shape; the choice must not change the result, and the tuned forward still matches the oracle."""
    import oracle
    import paper_2312_16733_amd as sna
    torch = torch_mod
    spec = synth.ResNetSpec()
    W, S, C = setup(spec, 16)
    net = sna.Supernet(spec, W, S, 16, 64)
    try:
        for ci, batch in ((3, 2), (15, 1), (9, 16)):
            c = C[ci]
            x = synth.make_inputs(spec, batch, c.in_h, c.in_w, 16)
            before = run_single(torch, net, spec, c, x)
            n0 = net.tuned_count()
            say("tune resnet cfg", ci, "batch", batch)
            tuned_out = net.tune([c], np.zeros(batch, np.int32), to_dev(torch, spec, x))
            torch.cuda.synchronize()
            assert net.tuned_count() > n0
            after = run_single(torch, net, spec, c, x)
            np.testing.assert_array_equal(before, tuned_out.cpu().numpy())
            np.testing.assert_array_equal(before, after)
            check_parity(after[:1], oracle.forward(spec, W, S, c, x[:1]), "bf16", f"tuned cfg {ci}")
    finally:
        net.close()


def test_replayed_launch_list_follows_the_callers_buffers(torch_mod, resnet_full):
    """The second call with the same cfgs and routing replays a recorded launch list; inputs, logits
    (and a different routing) must still be honoured."""
    torch = torch_mod
    spec, W, S, C, net = resnet_full
    c = C[4]
    xa = synth.make_inputs(spec, 3, c.in_h, c.in_w, 21)
    xb = synth.make_inputs(spec, 3, c.in_h, c.in_w, 22)
    r = np.zeros(3, np.int32)
    da, db = to_dev(torch, spec, xa), to_dev(torch, spec, xb)
    la = net.forward([c], r, da).cpu().numpy()          # builds the list
    lb = net.forward([c], r, db).cpu().numpy()          # replays it on other buffers
    la2 = net.forward([c], r, da).cpu().numpy()
    np.testing.assert_array_equal(la, la2)
    assert not np.array_equal(la, lb)
    out = torch.zeros((3, spec.n_classes), dtype=torch.float32, device="cuda:0")
    net.forward([c], r, db, logits=out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), lb)
    # same cfg list, other routing: request 1 goes to another cfg of the same resolution
    C2 = synth.enumerate_cfgs(spec, 16, 16733, fixed_res=c.in_h)
    xa2 = synth.make_inputs(spec, 3, c.in_h, c.in_h, 21)
    d2 = to_dev(torch, spec, xa2)
    m1 = net.forward(C2, np.array([2, 5, 2], np.int32), d2).cpu().numpy()
    m2 = net.forward(C2, np.array([2, 2, 5], np.int32), d2).cpu().numpy()
    m1b = net.forward(C2, np.array([2, 5, 2], np.int32), d2).cpu().numpy()
    np.testing.assert_array_equal(m1, m1b)
    np.testing.assert_array_equal(m1[0], m2[0])
    assert not np.array_equal(m1[1], m2[1])


def test_replayed_launch_list_other_families(torch_mod, mbv3_full, tf_full):
    """Replay of a recorded launch list on the MBV3- and transformer-shaped families: other input and
    output buffers on the second call, hidden states wanted or not."""
    torch = torch_mod
    spec, W, S, C, net = mbv3_full
    c = C[6]
    r = np.zeros(3, np.int32)
    xa = to_dev(torch, spec, synth.make_inputs(spec, 3, c.in_h, c.in_w, 91))
    xb = to_dev(torch, spec, synth.make_inputs(spec, 3, c.in_h, c.in_w, 92))
    la = net.forward([c], r, xa).cpu().numpy()
    lb = net.forward([c], r, xb).cpu().numpy()          # replay on another input buffer
    out = torch.zeros((3, spec.n_classes), dtype=torch.float32, device="cuda:0")
    net.forward([c], r, xa, logits=out)                 # replay into another logits buffer
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), la)
    assert not np.array_equal(la, lb)
    net.set_tile_variant(-1)                            # drops the recorded lists: a fresh list must agree
    np.testing.assert_array_equal(net.forward([c], r, xb).cpu().numpy(), lb)
    spec, W, S, C, net = tf_full
    c = C[4]
    r = np.zeros(2, np.int32)
    xa, xb = synth.make_inputs(spec, 2, c.in_h, c.in_w, 93), synth.make_inputs(spec, 2, c.in_h, c.in_w, 94)
    a1 = run_tf(torch, net, spec, [c], r, xa)
    b1 = run_tf(torch, net, spec, [c], r, xb)           # replay: new inputs, new hidden buffer
    a2 = run_tf(torch, net, spec, [c], r, xa)
    np.testing.assert_array_equal(a1[0], a2[0]); np.testing.assert_array_equal(a1[1], a2[1])
    assert not np.array_equal(a1[0], b1[0])
    nohid = net.forward([c], r, to_dev(torch, spec, xb)).cpu().numpy()      # other key: no hidden states
    np.testing.assert_array_equal(nohid, b1[0])
    net.set_tile_variant(-1)
    b2 = run_tf(torch, net, spec, [c], r, xb)
    np.testing.assert_array_equal(b1[0], b2[0]); np.testing.assert_array_equal(b1[1], b2[1])


def test_binding_rejects_short_buffers(torch_mod, resnet_full):
    """A tensor shorter than the routed requests need must never reach the kernels."""
    torch = torch_mod
    spec, W, S, C, net = resnet_full
    c = C[2]
    x = to_dev(torch, spec, synth.make_inputs(spec, 2, c.in_h, c.in_w, 95))
    with pytest.raises(ValueError):
        net.forward([c], [0, 0, 0], x)                  # three requests, two images
    small = torch.zeros((1, spec.n_classes), dtype=torch.float32, device="cuda:0")
    with pytest.raises(ValueError):
        net.forward([c], [0, 0], x, logits=small)
    with pytest.raises(ValueError):
        net.calibrate(c, x.flatten()[:-8].reshape(-1))


def test_tuning_table_round_trip_and_rejects_bad_lines(torch_mod):
    import paper_2312_16733_amd as sna
    torch = torch_mod
    spec = synth.ResNetSpec()
    W, S, C = setup(spec, 16)
    net = sna.Supernet(spec, W, S, 16, 8)
    other = sna.Supernet(spec, W, S, 16, 8)
    try:
        c = C[6]
        x = synth.make_inputs(spec, 2, c.in_h, c.in_w, 23)
        net.tune([c], np.zeros(2, np.int32), to_dev(torch, spec, x))
        torch.cuda.synchronize()
        text = net.tuning_export()
        lines = [ln for ln in text.splitlines() if ln]
        assert len(lines) == net.tuned_count() and all(ln[0] in "vs" and len(ln.split()) == 9 for ln in lines)
        other.tuning_import("# comment\n" + text)
        assert other.tuned_count() == net.tuned_count()
        assert sorted(other.tuning_export().splitlines()) == sorted(lines)
        a = run_single(torch, net, spec, c, x)
        b = run_single(torch, other, spec, c, x)
        np.testing.assert_array_equal(a, b)
        # a line without the twin count (the older form) is one twin
        other.tuning_import("v 24 24 24 1 1 1 0\n")
        assert "v 24 24 24 1 1 1 1 0" in other.tuning_export().splitlines()
        n0 = other.tuned_count()
        for bad in ("v 1 2 3\n", "v 64 64 64 1 1 1 999\n", "x 1 2 3 4 5 6 0\n", "s 1 2 3 4 5 0 7\n", "v 64 64 64 1 1 1 0 0\n",
                    "v 64 64 64 1 1 1 1 0 5\n"):
            with pytest.raises(sna.SnaError):
                other.tuning_import(text + bad)
            assert other.tuned_count() == n0
    finally:
        net.close()
        other.close()


def test_every_tile_variant_gives_the_same_bits(torch_mod, resnet_full, tf_full):
    """Each tile variant of the matrix kernel (plain and wave-specialised, every tile shape) forced onto
    every layer: ragged rows and columns, chunked reductions, split reductions; same bits as the default."""
    import paper_2312_16733_amd as sna
    torch = torch_mod
    nv = sna.lib().sna_tile_variant_count()
    assert nv >= 7
    spec, W, S, C, net = resnet_full
    cases = [(C[15], 2), (C[3], 5)]
    try:
        for c, batch in cases:
            x = synth.make_inputs(spec, batch, c.in_h, c.in_w, 24)
            ref = run_single(torch, net, spec, c, x)
            for mode in (0, 2, 3):
                net.set_k_split(mode)
                for v in range(nv):
                    net.set_tile_variant(v)
                    say("tile variant", v, "k split mode", mode, "batch", batch)
                    np.testing.assert_array_equal(run_single(torch, net, spec, c, x), ref, err_msg=f"variant {v} mode {mode}")
    finally:
        net.set_tile_variant(-1)
        net.set_k_split(0)
    spec, W, S, C, net = tf_full
    try:
        c = C[7]
        x = synth.make_inputs(spec, 3, c.in_h, c.in_w, 25)
        ref = run_tf(torch, net, spec, [c], np.zeros(3, np.int32), x)
        for v in range(nv):
            net.set_tile_variant(v)
            got = run_tf(torch, net, spec, [c], np.zeros(3, np.int32), x)
            np.testing.assert_array_equal(got[0], ref[0], err_msg=f"variant {v}")
            np.testing.assert_array_equal(got[1], ref[1], err_msg=f"variant {v} hidden")
    finally:
        net.set_tile_variant(-1)


def test_per_launch_profile_lists_every_launch(torch_mod, resnet_full):
    """sna_profile_read_launches: one line per launch of the forward, in order, each with a time, a class
    name and (matrix kernel) the active shapes; the class totals of sna_profile_read cover the same launches."""
    torch = torch_mod
    spec, W, S, C, net = resnet_full
    c = C[3]
    x = synth.make_inputs(spec, 3, c.in_h, c.in_w, 31)
    ref = run_single(torch, net, spec, c, x)
    net.profile_enable(True)
    try:
        got = run_single(torch, net, spec, c, x)
        lines = net.profile_read_launches().strip().split("\n")
        classes = net.profile_read()
    finally:
        net.profile_enable(False)
    np.testing.assert_array_equal(ref, got)
    assert len(lines) == net.last_forward_info()[1] == sum(v["launches"] for v in classes.values())
    total = 0.0
    for line in lines:
        us, cls = line.split(" ")[:2]
        assert float(us) > 0 and cls in classes
        total += float(us)
    assert abs(total * 1e-3 - sum(v["ms"] for v in classes.values())) < 1e-3 * len(lines)
    first_conv = next(l for l in lines if "igemm_conv_linear" in l)
    assert "tile=" in first_conv and f"C={c.stage_out_ch[0]} " in first_conv
    assert net.profile_read_launches() == ""


def test_supernet_profiler_table_has_the_scheduler_properties(torch_mod, resnet_full):
    """The latency table the profiler measures with the real kernels: positive entries, latency rising
    with the batch and with the subnet (the properties the paper's scheduler builds its latency buckets
    on), and a slack pick that meets its deadline."""
    from paper_2312_16733_amd import profiler
    torch = torch_mod
    spec, W, S, C, net = resnet_full
    cfgs = [C[0], C[7], C[15]]
    batches = (1, 8, 32)
    dev = torch.device("cuda:0")

    def make_inputs(c, b):
        return torch.from_numpy(synth.make_inputs(spec, b, c.in_h, c.in_w, 41)).to(torch.bfloat16).to(dev)

    say("profiling 3 cfgs x 3 batch sizes")
    table = profiler.profile_latency(net, spec, cfgs, make_inputs, batches, reps=5)
    assert table.shape == (3, 3) and (table > 0).all()
    props = profiler.check_properties(table, slack=0.10)
    assert props["p1_violations"] == 0 and props["p2_violations"] == 0 and props["p3_violations"] == 0, (table, props)
    bks = profiler.latency_buckets(table, batches, 6)
    assert sum(len(b.choices) for b in bks) == 9
    choice = profiler.pick(bks, float(table.max()) * 1.01)
    assert choice is not None and choice[2] <= table.max() * 1.01


# ------------------------------------------------------------------ other seeds than the standing ones
@pytest.mark.parametrize("k", [5, 17, 29])
def test_fresh_seeds_small_shapes(torch_mod, k):
    """Every family at small shapes with weight, cfg and input seeds the other tests do not use, random
    batch sizes 1..6 per cfg, plus one mixed call of 13 requests over the cfgs that share a resolution."""
    import oracle
    import paper_2312_16733_amd as sna
    torch = torch_mod
    cases = [("tiny", synth.TinySpec(), 8, "fp32"),
             ("resnet-small", SMALL_RESNET, 10, "bf16"),
             ("mbv3-small", synth.MBV3Spec(res_choices=(40, 48, 57, 64)), 10, "bf16"),
             ("tf-small", synth.TransformerSpec(n_classes=40, hidden=256, n_heads=4, head_dim=64, ffn=512, max_layers=4,
                                                seq_len=16 + (k * 8) % 113, depth_choices=(2, 3, 4)), 8, "bf16")]
    for j, (name, spec, n_cfg, mode) in enumerate(cases):
        wseed, cseed = 100 * (2 * j + 1) + k, 100 * (2 * j + 2) + k
        W, S, C = setup(spec, n_cfg, wseed=wseed, cseed=cseed)
        net = sna.Supernet(spec, W, S, n_cfg, 16)
        rng = np.random.default_rng(cseed)
        worst = 0.0
        try:
            for c in C:
                b = int(rng.integers(1, 7))
                x = synth.make_inputs(spec, b, c.in_h, c.in_w, int(rng.integers(1, 1000)))
                say(name, "seeds", wseed, cseed, "cfg", c.subnet_id, "batch", b)
                got = run_single(torch, net, spec, c, x)
                e, _ = check_parity(got, oracle.forward(spec, W, S, c, x), mode, f"{name} cfg {c.subnet_id}")
                worst = max(worst, e)
            byres = {}
            for c in C:
                byres.setdefault((c.in_h, c.in_w), []).append(c)
            res, cs = max(byres.items(), key=lambda kv: len(kv[1]))
            if len(cs) > 1:
                route = rng.integers(0, len(cs), 13).astype(np.int32)
                x = synth.make_inputs(spec, 13, res[0], res[1], 77)
                got = net.forward(cs, route, to_dev(torch, spec, x)).cpu().numpy()
                torch.cuda.synchronize()
                for r in range(13):
                    e, _ = check_parity(got[r:r + 1], oracle.forward(spec, W, S, cs[route[r]], x[r:r + 1]), mode,
                                        f"{name} mixed request {r}")
                    worst = max(worst, e)
        finally:
            net.close()
        say("  ", name, "worst rel err %.3e" % worst)


def test_all_variants_on_small_odd_images(torch_mod):
    """Every tile variant, the 3x3 kernel that keeps the activation slab in LDS included, forced onto every
    layer it can run of the small ResNet- and MBV3-shaped SuperNets (images down to 2x2, odd widths, channel
    counts of one, even and odd numbers of 16-byte units, ragged last tiles, tiles that span several images):
    same bits as the default choice."""
    import paper_2312_16733_amd as sna
    torch = torch_mod
    nv = sna.lib().sna_tile_variant_count()
    for name, spec, n_cfg in (("resnet-small", SMALL_RESNET, 8), ("mbv3-small", synth.MBV3Spec(res_choices=(40, 48, 57)), 6)):
        W, S, C = setup(spec, n_cfg)
        net = sna.Supernet(spec, W, S, n_cfg, 16)
        try:
            for c in C:
                for batch in (1, 7):
                    x = synth.make_inputs(spec, batch, c.in_h, c.in_w, 50 + batch)
                    net.set_tile_variant(-1)
                    ref = run_single(torch, net, spec, c, x)
                    for v in range(nv):
                        net.set_tile_variant(v)
                        got = run_single(torch, net, spec, c, x)
                        np.testing.assert_array_equal(got, ref, err_msg=f"{name} cfg {c.subnet_id} batch {batch} variant {v}")
                say(name, "cfg", c.subnet_id, "res", c.in_h, "variants 0..%d: same bits" % (nv - 1))
        finally:
            net.set_tile_variant(-1)
            net.close()


def test_policies_drive_the_library(torch_mod):
    """The event loop with a GpuExecutor: every dispatched batch really runs on the resident SuperNet."""
    import paper_2312_16733_amd as sna
    from paper_2312_16733_amd import profiler, scheduler
    torch = torch_mod
    spec = SMALL_RESNET
    W, S, C = setup(spec, 8, fixed_res=48)
    net = sna.Supernet(spec, W, S, 8, 8)
    try:
        batches = (1, 2, 4, 8)

        def make_inputs(c, b):
            return to_dev(torch, spec, synth.make_inputs(spec, b, c.in_h, c.in_w, 9))

        full = profiler.profile_latency(net, spec, C, make_inputs, batches, reps=3, warmup=1)
        front = profiler.pareto_subset(full)
        front = [front[k] for k in profiler.pareto_subset(full[front], col=0)]
        table = full[front]
        ex = scheduler.GpuExecutor(net, spec, [C[k] for k in front], batches, make_inputs)
        slo_ms = 20.0 * float(table.max())
        arrivals = scheduler.bursty_trace(200.0, 800.0, 4.0, 0.05, 11)
        for pol in (scheduler.SlackFit(table, batches, n_buckets=8), scheduler.MaxBatch(table, batches)):
            ex.calls = 0
            r = scheduler.simulate(pol, arrivals, slo_ms, 1, executor=ex)
            say(pol.name, "attainment", r["slo_attainment"], "forwards", ex.calls, "queries", r["queries"])
            assert r["queries"] == len(arrivals) and ex.calls == len(r["decisions"]) > 0
            assert r["served"] + r["dropped"] == r["queries"]
            assert r["slo_attainment"] > 0.9                   # far below capacity with a generous deadline
        assert ex.busy_ms > 0
    finally:
        net.close()
