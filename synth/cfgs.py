"""Seeded enumeration of subnet control tuples and of request->cfg routing.

A cfg list is {global min, global max} plus seeded uniform draws from the
family's choice sets, de-duplicated and ordered smallest to largest by
multiply-accumulate count per request; subnet ids are positions in that list.
Ratios (E, W) are resolved to channel counts here, once, with round_channels().
"""
import numpy as np

from .arch import SubnetCfg, round_channels
from .rng import keyed_rng


def _out(h, k, s):
    return (h + 2 * (k // 2) - k) // s + 1


def _blank(spec, n_stages):
    z = lambda: [[0] * max(spec.max_depth) for _ in range(n_stages)]
    return z(), z(), z()


# ---------------------------------------------------------------- per family
def _tiny_cfg(spec, depth, widths, res):
    mid, aux, ker = _blank(spec, spec.n_stages)
    out = [spec.stem_ch] + [int(round(w * c)) for w, c in zip(widths, spec.stage_ch)]
    return SubnetCfg(0, spec.n_stages, list(depth), out, mid, aux, ker, res, res)


def _resnet_cfg(spec, depth, widths, expands, res):
    """widths: stem + one per stage; expands[s][j] for every max-depth slot."""
    mid, aux, ker = _blank(spec, spec.n_stages)
    out = [round_channels(widths[0] * spec.stem_ch)]
    for s, c in enumerate(spec.stage_ch):
        out.append(round_channels(widths[1 + s] * c))
        for j in range(spec.max_depth[s]):
            mid[s][j] = round_channels(expands[s][j] * out[1 + s]) if j < depth[s] else 0
    return SubnetCfg(0, spec.n_stages, list(depth), out, mid, aux, ker, res, res)


def _mbv3_cfg(spec, depth, expands, kernels, res):
    mid, aux, ker = _blank(spec, spec.n_stages)
    out = [spec.stem_ch] + list(spec.stage_ch)
    for s in range(spec.n_stages):
        for j in range(depth[s]):
            mid[s][j] = round_channels(expands[s][j] * spec.block_in(s, j))
            aux[s][j] = round_channels(mid[s][j] / 4) if spec.stage_se[s] else 0
            ker[s][j] = kernels[s][j]
    return SubnetCfg(0, spec.n_stages, list(depth), out, mid, aux, ker, res, res)


def _tf_cfg(spec, depth, head_r, ffn_r):
    mid = [[0] * spec.max_layers]
    aux = [[0] * spec.max_layers]
    ker = [[0] * spec.max_layers]
    for j in range(depth):
        mid[0][j] = int(round(head_r[j] * spec.n_heads)) * spec.head_dim
        aux[0][j] = int(round(ffn_r[j] * spec.ffn))
    return SubnetCfg(0, 1, [depth], [spec.hidden, spec.hidden], mid, aux, ker, spec.seq_len, 1)


def _draw(spec, g, pick):
    """pick(choices) returns one element; used for min / max / random cfgs."""
    f = spec.family
    if f == "tiny":
        return _tiny_cfg(spec, [pick(spec.depth_choices) for _ in spec.stage_ch],
                         [pick(spec.width_choices) for _ in spec.stage_ch],
                         pick(spec.res_choices))
    if f == "resnet":
        depth = [pick(tuple(sorted(m - d for d in spec.depth_minus))) for m in spec.max_depth]
        widths = [pick(spec.width_choices) for _ in range(1 + spec.n_stages)]
        ex = [[pick(spec.expand_choices) for _ in range(m)] for m in spec.max_depth]
        return _resnet_cfg(spec, depth, widths, ex, pick(spec.res_choices))
    if f == "mbv3":
        depth = [pick(spec.depth_choices) for _ in spec.stage_ch]
        ex = [[pick(spec.expand_choices) for _ in range(m)] for m in spec.max_depth]
        ke = [[pick(spec.kernel_choices) for _ in range(m)] for m in spec.max_depth]
        return _mbv3_cfg(spec, depth, ex, ke, pick(spec.res_choices))
    if f == "transformer":
        depth = pick(spec.depth_choices)
        hr = [pick(spec.ratio_choices) for _ in range(spec.max_layers)]
        fr = [pick(spec.ratio_choices) for _ in range(spec.max_layers)]
        return _tf_cfg(spec, depth, hr, fr)
    raise ValueError(f)


def subnet_macs(spec, cfg: SubnetCfg) -> int:
    """Multiply-accumulates of one request through the launched layers only."""
    f = spec.family
    macs = 0
    if f == "tiny":
        h = cfg.in_h
        macs += h * h * 9 * spec.in_ch * cfg.stage_out_ch[0]
        cin = cfg.stage_out_ch[0]
        for s in range(spec.n_stages):
            c = cfg.stage_out_ch[1 + s]
            for j in range(cfg.depth[s]):
                if j == 0:
                    h = _out(h, 3, 2)
                macs += h * h * 9 * cin * c
                cin = c
        return macs + cin * spec.n_classes
    if f == "resnet":
        h = _out(cfg.in_h, 7, 2)
        macs += h * h * 49 * spec.in_ch * cfg.stage_out_ch[0]
        h = _out(h, 3, 2)
        cin = cfg.stage_out_ch[0]
        for s in range(spec.n_stages):
            c = cfg.stage_out_ch[1 + s]
            for j in range(cfg.depth[s]):
                st = spec.stage_stride[s] if j == 0 else 1
                m = cfg.block_mid_ch[s][j]
                ho = _out(h, 3, st)
                macs += h * h * cin * m + ho * ho * 9 * m * m + ho * ho * m * c
                if j == 0:
                    macs += ho * ho * cin * c
                h, cin = ho, c
        return macs + cin * spec.n_classes
    if f == "mbv3":
        h = _out(cfg.in_h, 3, 2)
        c0 = spec.stem_ch
        macs += h * h * 9 * spec.in_ch * c0 + h * h * 9 * c0 + h * h * c0 * c0
        cin = c0
        for s in range(spec.n_stages):
            c = spec.stage_ch[s]
            for j in range(cfg.depth[s]):
                st = spec.stage_stride[s] if j == 0 else 1
                m, k, q = cfg.block_mid_ch[s][j], cfg.block_kernel[s][j], cfg.block_aux_ch[s][j]
                ho = _out(h, k, st)
                macs += h * h * cin * m + ho * ho * k * k * m + 2 * m * q + ho * ho * m * c
                h, cin = ho, c
        macs += h * h * cin * spec.tail_ch
        return macs + spec.tail_ch * spec.fc_ch + spec.fc_ch * spec.n_classes
    if f == "transformer":
        S, H = spec.seq_len, spec.hidden
        for j in range(cfg.depth[0]):
            a, ff = cfg.block_mid_ch[0][j], cfg.block_aux_ch[0][j]
            macs += S * (3 * H * a + a * H + 2 * H * ff) + 2 * S * S * a
        return macs + H * spec.n_classes
    raise ValueError(f)


def enumerate_cfgs(spec, n: int, seed: int, fixed_res=None):
    g = keyed_rng(seed, f"cfgs:{spec.family}")
    cfgs = [_draw(spec, g, lambda ch: min(ch)), _draw(spec, g, lambda ch: max(ch))]
    seen = {c.key() for c in cfgs}
    guard = 0
    while len(cfgs) < n and guard < 100 * n:
        guard += 1
        c = _draw(spec, g, lambda ch: ch[int(g.integers(len(ch)))])
        if c.key() not in seen:
            seen.add(c.key())
            cfgs.append(c)
    if fixed_res is not None:
        for c in cfgs:
            c.in_h = c.in_w = fixed_res
    cfgs.sort(key=lambda c: subnet_macs(spec, c))
    for i, c in enumerate(cfgs):
        c.subnet_id = i
    return cfgs


def zipf_assignment(n_requests: int, n_cfgs: int, seed: int, a: float = 1.1) -> np.ndarray:
    """request -> cfg index: P(rank k) ~ k^-a, ranks mapped by a seeded permutation."""
    g = keyed_rng(seed, f"zipf:{n_requests}:{n_cfgs}")
    p = np.arange(1, n_cfgs + 1, dtype=np.float64) ** (-a)
    p /= p.sum()
    perm = g.permutation(n_cfgs)
    ranks = g.choice(n_cfgs, size=n_requests, p=p)
    return perm[ranks].astype(np.int32)
