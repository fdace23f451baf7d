"""sna_subnet_forward_static (the entry point that allocates nothing) against sna_subnet_forward.

Same kernels and launch order, scratch taken from the library's static device array instead of the
handle's workspace: the logits must have the same bits.  Two calls in a row, the second smaller, so
that stale contents of the shared array from the first call cannot leak into the second.
"""
import sys

import numpy as np
import pytest

import synth
from helpers import setup, check_parity

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _dev(torch, spec, x):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if spec.dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.to("cuda:0")


def _pair(torch, net, spec, cfgs, route, x, hidden=False):
    """(workspace entry point, static entry point) logits [and hidden states] for one call."""
    outs = []
    for static in (False, True):
        logits = torch.full((len(route), spec.n_classes), float("nan"), dtype=torch.float32, device="cuda:0")
        hid = None
        if hidden:
            hid = torch.zeros((len(route), spec.seq_len, spec.hidden), dtype=torch.bfloat16, device="cuda:0")
        net.forward(cfgs, route, x, logits=logits, hidden=hid, static=static)
        torch.cuda.synchronize()
        outs.append((logits.cpu().numpy(), None if hid is None else hid.float().cpu().numpy()))
    return outs


def test_static_scratch_forward_matches_workspace_forward():
    import torch
    import oracle
    import paper_2312_16733_amd as sna
    assert torch.cuda.is_available()
    assert sna.lib().sna_static_scratch_bytes() == 256 << 20

    # ResNet-50-shaped SuperNet at full size: batch 3 of the largest cfg, then batch 1 of a smaller one
    spec = synth.ResNetSpec()
    W, S, C = setup(spec, 16)
    net = sna.Supernet(spec, W, S, 16, 64)
    try:
        for ci, batch in ((15, 3), (4, 1)):
            c = C[ci]
            xh = synth.make_inputs(spec, batch, c.in_h, c.in_w, 201 + batch)
            say("static scratch: resnet cfg", ci, "batch", batch)
            (a, _), (b, _) = _pair(torch, net, spec, [c], np.zeros(batch, np.int32), _dev(torch, spec, xh))
            assert np.all(np.isfinite(b))
            np.testing.assert_array_equal(a, b)
            check_parity(b, oracle.forward(spec, W, S, c, xh), "bf16", f"static resnet cfg {ci}")
        # replayed launch list of the static flavour, then the workspace flavour again: still the same bits
        c = C[4]
        xh = synth.make_inputs(spec, 1, c.in_h, c.in_w, 202)
        (a, _), (b, _) = _pair(torch, net, spec, [c], np.zeros(1, np.int32), _dev(torch, spec, xh))
        np.testing.assert_array_equal(a, b)
        # a mixed call through the static array (gathered requests, scattered logits), smaller again
        Cm = synth.enumerate_cfgs(spec, 16, 16733, fixed_res=160)
        route = np.array([3, 0, 3], dtype=np.int32)
        xh = synth.make_inputs(spec, 3, 160, 160, 203)
        (a, _), (b, _) = _pair(torch, net, spec, Cm, route, _dev(torch, spec, xh))
        np.testing.assert_array_equal(a, b)
        # beyond the static array: refused with a clear error before anything runs, handle still usable
        c = C[15]
        big = _dev(torch, spec, synth.make_inputs(spec, 32, c.in_h, c.in_w, 204))
        with pytest.raises(sna.SnaError) as ei:
            net.forward([c], np.zeros(32, np.int32), big, static=True)
        assert ei.value.status == -7 and "static scratch" in str(ei.value)
        ok = net.forward([c], np.zeros(32, np.int32), big)
        torch.cuda.synchronize()
        assert np.all(np.isfinite(ok.cpu().numpy()))
        # not while per-launch profiling is on (that path creates events)
        net.profile_enable(True)
        try:
            with pytest.raises(sna.SnaError) as ei:
                net.forward([c], np.zeros(1, np.int32), big, static=True)
            assert ei.value.status == -6
        finally:
            net.profile_enable(False)
    finally:
        net.close()

    # the other families, each a larger call followed by a smaller one
    cases = [(synth.TinySpec(), 8, "fp32", (4, 2)),
             (synth.MBV3Spec(), 16, "bf16", (4, 1)),
             (synth.TransformerSpec(), 12, "bf16", (4, 2))]
    for spec, n_cfgs, mode, batches in cases:
        W, S, C = setup(spec, n_cfgs)
        net = sna.Supernet(spec, W, S, n_cfgs, 8)
        try:
            for k, batch in enumerate(batches):
                c = C[-1 - 3 * k]
                xh = synth.make_inputs(spec, batch, c.in_h, c.in_w, 210 + batch)
                say("static scratch:", spec.family, "cfg", c.subnet_id, "batch", batch)
                (a, ha), (b, hb) = _pair(torch, net, spec, [c], np.zeros(batch, np.int32), _dev(torch, spec, xh),
                                         hidden=spec.family == "transformer")
                np.testing.assert_array_equal(a, b)
                if ha is not None:
                    np.testing.assert_array_equal(ha, hb)
                check_parity(b, oracle.forward(spec, W, S, c, xh), mode, f"static {spec.family}")
        finally:
            net.close()
