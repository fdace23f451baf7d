"""Oracle forward of a subnet served in place -- TEST INFRASTRUCTURE.

forward(spec, weights, stats, cfg, x, mode) runs subnet `cfg` directly on the
max-size SuperNet tensors, using the three SubNetAct operators exactly as their
paragraphs describe them:

  LayerSelect  the per-stage depth D becomes one boolean per block; a block is
               either applied to its input or its input is passed on unchanged.
  WeightSlice  E / W arrive as channel counts; conv / linear layers use the
               leading output and input channels of the shared weights (and the
               centre window of an elastic depthwise kernel) with no copy.
  SubnetNorm   normalisation uses the statistics stored for (subnet id, layer).

`mode` names the storage precision of activations: every tensor a layer hands
to the next one is rounded once to that format ("fp32", "bf16") or not at all
("f64"); all arithmetic in between is float64.  Logits are returned unrounded.
The block wiring of each family and the places where activations are stored
are this build's reading; the paper names the families only.
"""
import numpy as np

from . import primitives as P


def layer_select(run: bool, layer, x):
    """LayerSelect: apply the wrapped layer, or forward the input unchanged."""
    return layer(x) if run else x


def depth_to_flags(depth: int, max_depth: int):
    """Depth D of a stage -> per-block booleans: keep the leading D blocks."""
    return [j < depth for j in range(max_depth)]


# ------------------------------------------------------------------ tiny conv net
def _tiny(spec, W, S, cfg, x, rd):
    i = cfg.subnet_id
    a = rd(P.relu(P.subnet_norm(P.conv2d_sliced(x, W["stem.w"], cfg.stage_out_ch[0], 3, 1),
                                S["stem.sn"], i)))
    for s in range(spec.n_stages):
        c = cfg.stage_out_ch[1 + s]
        flags = depth_to_flags(cfg.depth[s], spec.max_depth[s])
        for j, run in enumerate(flags):
            def block(t, s=s, j=j, c=c):
                y = P.relu(P.subnet_norm(
                    P.conv2d_sliced(t, W[f"s{s}.b{j}.w"], c, 3, 2 if j == 0 else 1),
                    S[f"s{s}.b{j}.sn"], i))
                return rd(t + y) if j > 0 else rd(y)      # block 0 changes shape: no residual
            a = layer_select(run, block, a)
    pooled = rd(P.global_avg_pool(a))
    return P.linear_sliced(pooled, W["head.w"], spec.n_classes, W["head.b"])


# ------------------------------------------------------------------ ResNet bottlenecks
def _resnet(spec, W, S, cfg, x, rd):
    i = cfg.subnet_id
    a = rd(P.relu(P.subnet_norm(P.conv2d_sliced(x, W["stem.w"], cfg.stage_out_ch[0], 7, 2),
                                S["stem.sn"], i)))
    a = P.maxpool_3x3_s2(a)
    for s in range(spec.n_stages):
        c = cfg.stage_out_ch[1 + s]
        flags = depth_to_flags(cfg.depth[s], spec.max_depth[s])
        for j, run in enumerate(flags):
            def block(t, s=s, j=j, c=c):
                p = f"s{s}.b{j}."
                st = spec.stage_stride[s] if j == 0 else 1
                m = cfg.block_mid_ch[s][j]
                u = rd(P.relu(P.subnet_norm(P.conv2d_sliced(t, W[p + "conv1.w"], m, 1, 1), S[p + "sn1"], i)))
                u = rd(P.relu(P.subnet_norm(P.conv2d_sliced(u, W[p + "conv2.w"], m, 3, st), S[p + "sn2"], i)))
                u = P.subnet_norm(P.conv2d_sliced(u, W[p + "conv3.w"], c, 1, 1), S[p + "sn3"], i)
                if j == 0:
                    sc = rd(P.subnet_norm(P.conv2d_sliced(t, W[p + "short.w"], c, 1, st), S[p + "sn_short"], i))
                else:
                    sc = t
                return rd(P.relu(u + sc))
            a = layer_select(run, block, a)
    pooled = rd(P.global_avg_pool(a))
    return P.linear_sliced(pooled, W["head.w"], spec.n_classes, W["head.b"])


# ------------------------------------------------------------------ MobileNetV3-shaped
def _mbv3(spec, W, S, cfg, x, rd):
    i = cfg.subnet_id
    c0 = spec.stem_ch
    a = rd(P.hardswish(P.subnet_norm(P.conv2d_sliced(x, W["stem.w"], c0, 3, 2), S["stem.sn"], i)))
    u = rd(P.relu(P.subnet_norm(P.depthwise_sliced(a, W["first.dw.w"], 3, 1), S["first.sn1"], i)))
    a = rd(a + P.subnet_norm(P.conv2d_sliced(u, W["first.pw.w"], c0, 1, 1), S["first.sn2"], i))
    for s in range(spec.n_stages):
        c = spec.stage_ch[s]
        act = P.ACT[spec.stage_act[s]]
        flags = depth_to_flags(cfg.depth[s], spec.max_depth[s])
        for j, run in enumerate(flags):
            def block(t, s=s, j=j, c=c, act=act):
                p = f"s{s}.b{j}."
                st = spec.stage_stride[s] if j == 0 else 1
                m, k = cfg.block_mid_ch[s][j], cfg.block_kernel[s][j]
                u = rd(act(P.subnet_norm(P.conv2d_sliced(t, W[p + "expand.w"], m, 1, 1), S[p + "sn1"], i)))
                u = rd(act(P.subnet_norm(P.depthwise_sliced(u, W[p + "dw.w"], k, st), S[p + "sn2"], i)))
                if spec.stage_se[s]:
                    q = cfg.block_aux_ch[s][j]
                    z = P.global_avg_pool(u)
                    z = P.relu(P.linear_sliced(z, W[p + "se.fc1.w"], q, W[p + "se.fc1.b"]))
                    g = P.hardsigmoid(P.linear_sliced(z, W[p + "se.fc2.w"], m, W[p + "se.fc2.b"]))
                    u = rd(u * g[:, None, None, :])
                y = P.subnet_norm(P.conv2d_sliced(u, W[p + "project.w"], c, 1, 1), S[p + "sn3"], i)
                return rd(t + y) if (st == 1 and t.shape[-1] == c) else rd(y)
            a = layer_select(run, block, a)
    a = rd(P.hardswish(P.subnet_norm(P.conv2d_sliced(a, W["tail.w"], spec.tail_ch, 1, 1), S["tail.sn"], i)))
    z = rd(P.global_avg_pool(a))
    z = rd(P.hardswish(P.linear_sliced(z, W["fc1.w"], spec.fc_ch, W["fc1.b"])))
    return P.linear_sliced(z, W["head.w"], spec.n_classes, W["head.b"])


# ------------------------------------------------------------------ Transformer encoder
def _transformer(spec, W, S, cfg, x, rd, return_hidden=False):
    b, sl, h = x.shape
    d = spec.head_dim
    flags = depth_to_flags(cfg.depth[0], spec.max_layers)
    for j, run in enumerate(flags):
        def block(t, j=j):
            p = f"l{j}."
            a, f = cfg.block_mid_ch[0][j], cfg.block_aux_ch[0][j]
            nh = a // d
            q = rd(P.linear_sliced(t, W[p + "q.w"], a, W[p + "q.b"])).reshape(b, sl, nh, d)
            k = rd(P.linear_sliced(t, W[p + "k.w"], a, W[p + "k.b"])).reshape(b, sl, nh, d)
            v = rd(P.linear_sliced(t, W[p + "v.w"], a, W[p + "v.b"])).reshape(b, sl, nh, d)
            scores = np.einsum("bihd,bjhd->bhij", q, k) / np.sqrt(float(d))
            prob = rd(P.softmax(scores))
            ctx = rd(np.einsum("bhij,bjhd->bihd", prob, v).reshape(b, sl, a))
            u = rd(t + P.linear_sliced(ctx, W[p + "o.w"], h, W[p + "o.b"]))
            t1 = rd(P.layer_norm(u, W[p + "ln1.g"], W[p + "ln1.b"]))
            g = rd(P.gelu(P.linear_sliced(t1, W[p + "ffn1.w"], f, W[p + "ffn1.b"])))
            u = rd(t1 + P.linear_sliced(g, W[p + "ffn2.w"], h, W[p + "ffn2.b"]))
            return rd(P.layer_norm(u, W[p + "ln2.g"], W[p + "ln2.b"]))
        x = layer_select(run, block, x)
    logits = P.linear_sliced(x[:, 0, :], W["head.w"], spec.n_classes, W["head.b"])
    return (logits, x) if return_hidden else logits


_FAMILY = {"tiny": _tiny, "resnet": _resnet, "mbv3": _mbv3, "transformer": _transformer}


def forward(spec, weights, stats, cfg, x, mode=None, **kw):
    """Logits [n][n_classes] (float64) of subnet `cfg` for inputs x."""
    mode = mode or spec.dtype
    rd = P.ROUND[mode]
    return _FAMILY[spec.family](spec, weights, stats, cfg, rd(x), rd, **kw)


def calibrate(spec, weights, stats, cfg, x, mode=None):
    """SubnetNorm calibration of subnet `cfg` on the batch x: one forward in which every SubnetNorm
    layer the subnet runs takes its mean / variance row from the activations it sees (gamma and beta
    stay).  Returns (copy of stats with row cfg.subnet_id filled in, logits of that forward).
    A later forward(spec, weights, new_stats, cfg, x) reproduces these logits exactly."""
    new = {k: np.array(v, copy=True) for k, v in stats.items()}
    wrapped = {k: P.CalibrationTable(v) for k, v in new.items()}
    logits = forward(spec, weights, wrapped, cfg, x, mode)
    return new, logits
