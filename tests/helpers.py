"""Shared test plumbing: seeded problem set-up and the parity metric."""
import numpy as np

import synth

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def setup(spec, n_cfgs, wseed=2312, cseed=16733, fixed_res=None):
    W = synth.make_weights(spec, wseed)
    S = synth.make_stats(spec, n_cfgs, wseed)
    C = synth.enumerate_cfgs(spec, n_cfgs, cseed, fixed_res=fixed_res)
    return W, S, C


def rel_err(got, ref):
    """Per request: max_k |g_k - o_k| / max(max_k |o_k|, 1e-6)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return np.abs(got - ref).max(axis=-1) / np.maximum(np.abs(ref).max(axis=-1), 1e-6)


def check_parity(got, ref, dtype, what="", tol=None):
    """Tolerance on the logits plus identical argmax wherever the oracle's top-1 / top-2 gap
    exceeds twice the tolerance (inside that margin either class is a correct answer).  `tol`
    replaces the dtype's bar where a test derives its own."""
    tol = TOL[dtype] if tol is None else tol
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    e = rel_err(got, ref)
    assert e.max() <= tol, f"{what}: max rel err {e.max():.3e} > {tol}"
    srt = np.sort(ref, axis=-1)
    gap = srt[:, -1] - srt[:, -2]
    decided = gap > 2 * tol * np.abs(ref).max(axis=-1)
    same = got.argmax(-1) == ref.argmax(-1)
    assert np.all(same | ~decided), f"{what}: argmax differs on a decided request"
    return float(e.max()), int((~decided).sum())
