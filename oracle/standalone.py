"""Extract-then-run oracle: the plain definition of a subnet -- TEST INFRASTRUCTURE.

SubNetAct is exact: serving a subnet in place must give what prior work gets by
statically extracting that subnet from the SuperNet and deploying it alone
(section "Weight-Shared Supernets"; opening of the SubNetAct section).  This
module is that definition written out:

  extract_subnet()      copies the active slice of every kept layer (and the
                        subnet's own row of normalisation statistics) into fresh
                        dense tensors; skipped blocks simply do not exist in it.
  standalone_forward()  runs the resulting ordinary network with PyTorch CPU
                        library ops in float64.  It never sees the cfg: which
                        blocks exist and every channel count are read off the
                        extracted tensors themselves.

It shares no arithmetic with inplace.py except the storage-rounding helpers.
"""
import numpy as np
import torch
import torch.nn.functional as F

from . import primitives as P


# ------------------------------------------------------------------ extraction
def _conv(w, k_out, c_in, k=None):
    r = w.shape[1]
    k = r if k is None else k
    o = (r - k) // 2
    return np.array(w[:k_out, o:o + k, o:o + k, :c_in], dtype=np.float32, copy=True)


def extract_subnet(spec, weights, stats, cfg):
    """-> (tensors, norms): dense copies of exactly what subnet `cfg` uses."""
    T, N = {}, {}
    i = cfg.subnet_id

    def norm(name, c):
        N[name] = np.array(stats[name][i, :, :c], dtype=np.float32, copy=True)

    f = spec.family
    if f == "tiny":
        cin = cfg.stage_out_ch[0]
        T["stem.w"] = _conv(weights["stem.w"], cin, spec.in_ch); norm("stem.sn", cin)
        for s in range(spec.n_stages):
            c = cfg.stage_out_ch[1 + s]
            for j in range(cfg.depth[s]):
                T[f"s{s}.b{j}.w"] = _conv(weights[f"s{s}.b{j}.w"], c, cin); norm(f"s{s}.b{j}.sn", c)
                cin = c
        T["head.w"] = weights["head.w"][:, :cin].copy(); T["head.b"] = weights["head.b"].copy()
    elif f == "resnet":
        cin = cfg.stage_out_ch[0]
        T["stem.w"] = _conv(weights["stem.w"], cin, spec.in_ch); norm("stem.sn", cin)
        for s in range(spec.n_stages):
            c = cfg.stage_out_ch[1 + s]
            for j in range(cfg.depth[s]):
                p, m = f"s{s}.b{j}.", cfg.block_mid_ch[s][j]
                T[p + "conv1.w"] = _conv(weights[p + "conv1.w"], m, cin); norm(p + "sn1", m)
                T[p + "conv2.w"] = _conv(weights[p + "conv2.w"], m, m); norm(p + "sn2", m)
                T[p + "conv3.w"] = _conv(weights[p + "conv3.w"], c, m); norm(p + "sn3", c)
                if j == 0:
                    T[p + "short.w"] = _conv(weights[p + "short.w"], c, cin); norm(p + "sn_short", c)
                cin = c
        T["head.w"] = weights["head.w"][:, :cin].copy(); T["head.b"] = weights["head.b"].copy()
    elif f == "mbv3":
        for nm in ("stem.w", "first.dw.w", "first.pw.w", "tail.w", "fc1.w", "fc1.b", "head.w", "head.b"):
            T[nm] = weights[nm].copy()
        for nm in ("stem.sn", "first.sn1", "first.sn2", "tail.sn"):
            norm(nm, stats[nm].shape[-1])
        cin = spec.stem_ch
        for s in range(spec.n_stages):
            c = spec.stage_ch[s]
            for j in range(cfg.depth[s]):
                p = f"s{s}.b{j}."
                m, k, q = cfg.block_mid_ch[s][j], cfg.block_kernel[s][j], cfg.block_aux_ch[s][j]
                T[p + "expand.w"] = _conv(weights[p + "expand.w"], m, cin); norm(p + "sn1", m)
                o = (7 - k) // 2
                T[p + "dw.w"] = weights[p + "dw.w"][o:o + k, o:o + k, :m].copy(); norm(p + "sn2", m)
                if spec.stage_se[s]:
                    T[p + "se.fc1.w"] = weights[p + "se.fc1.w"][:q, :m].copy()
                    T[p + "se.fc1.b"] = weights[p + "se.fc1.b"][:q].copy()
                    T[p + "se.fc2.w"] = weights[p + "se.fc2.w"][:m, :q].copy()
                    T[p + "se.fc2.b"] = weights[p + "se.fc2.b"][:m].copy()
                T[p + "project.w"] = _conv(weights[p + "project.w"], c, m); norm(p + "sn3", c)
                cin = c
    elif f == "transformer":
        for j in range(cfg.depth[0]):
            p = f"l{j}."
            a, ff = cfg.block_mid_ch[0][j], cfg.block_aux_ch[0][j]
            for nm in ("q", "k", "v"):
                T[p + nm + ".w"] = weights[p + nm + ".w"][:a].copy()
                T[p + nm + ".b"] = weights[p + nm + ".b"][:a].copy()
            T[p + "o.w"] = weights[p + "o.w"][:, :a].copy(); T[p + "o.b"] = weights[p + "o.b"].copy()
            T[p + "ffn1.w"] = weights[p + "ffn1.w"][:ff].copy(); T[p + "ffn1.b"] = weights[p + "ffn1.b"][:ff].copy()
            T[p + "ffn2.w"] = weights[p + "ffn2.w"][:, :ff].copy(); T[p + "ffn2.b"] = weights[p + "ffn2.b"].copy()
            for nm in ("ln1.g", "ln1.b", "ln2.g", "ln2.b"):
                T[p + nm] = weights[p + nm].copy()
        T["head.w"] = weights["head.w"].copy(); T["head.b"] = weights["head.b"].copy()
    else:
        raise ValueError(f)
    return T, N


# ------------------------------------------------------------------ dense library forward
def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.float64)


def _rd(rd):
    return lambda t: torch.from_numpy(rd(t.contiguous().numpy()))


def _conv2d(x, w, stride):
    """x NCHW float64; w stored [K][R][S][C]."""
    return F.conv2d(x, _t(w).permute(0, 3, 1, 2), stride=stride, padding=w.shape[1] // 2)


def _dw(x, w, stride):
    """w stored [R][S][C]."""
    c = w.shape[2]
    return F.conv2d(x, _t(w).permute(2, 0, 1).unsqueeze(1), stride=stride, padding=w.shape[0] // 2, groups=c)


def _bn(x, n):
    n = _t(n)
    return F.batch_norm(x, n[0], n[1], n[2], n[3], training=False, eps=P.EPS)


def _nblocks(T, s):
    j = 0
    while any(k.startswith(f"s{s}.b{j}.") for k in T):
        j += 1
    return j


def standalone_forward(spec, T, N, x, mode=None, return_hidden=False):
    """Run the extracted network.  `spec` supplies only family constants that
    no subnet changes (strides, activation kind, which stages carry SE)."""
    rd = _rd(P.ROUND[mode or spec.dtype])
    f = spec.family
    if f == "transformer":
        return _standalone_transformer(spec, T, rd(_t(x)), rd, return_hidden)
    a = rd(_t(x).permute(0, 3, 1, 2))
    if f == "tiny":
        a = rd(F.relu(_bn(_conv2d(a, T["stem.w"], 1), N["stem.sn"])))
        for s in range(spec.n_stages):
            for j in range(_nblocks(T, s)):
                y = F.relu(_bn(_conv2d(a, T[f"s{s}.b{j}.w"], 2 if j == 0 else 1), N[f"s{s}.b{j}.sn"]))
                a = rd(a + y) if j > 0 else rd(y)
        z = rd(a.mean(dim=(2, 3)))
    elif f == "resnet":
        a = rd(F.relu(_bn(_conv2d(a, T["stem.w"], 2), N["stem.sn"])))
        a = F.max_pool2d(a, 3, 2, 1)
        for s in range(spec.n_stages):
            for j in range(_nblocks(T, s)):
                p = f"s{s}.b{j}."
                st = spec.stage_stride[s] if j == 0 else 1
                u = rd(F.relu(_bn(_conv2d(a, T[p + "conv1.w"], 1), N[p + "sn1"])))
                u = rd(F.relu(_bn(_conv2d(u, T[p + "conv2.w"], st), N[p + "sn2"])))
                u = _bn(_conv2d(u, T[p + "conv3.w"], 1), N[p + "sn3"])
                sc = rd(_bn(_conv2d(a, T[p + "short.w"], st), N[p + "sn_short"])) if (p + "short.w") in T else a
                a = rd(F.relu(u + sc))
        z = rd(a.mean(dim=(2, 3)))
    elif f == "mbv3":
        a = rd(F.hardswish(_bn(_conv2d(a, T["stem.w"], 2), N["stem.sn"])))
        u = rd(F.relu(_bn(_dw(a, T["first.dw.w"], 1), N["first.sn1"])))
        a = rd(a + _bn(_conv2d(u, T["first.pw.w"], 1), N["first.sn2"]))
        for s in range(spec.n_stages):
            act = F.relu if spec.stage_act[s] == "relu" else F.hardswish
            for j in range(_nblocks(T, s)):
                p = f"s{s}.b{j}."
                st = spec.stage_stride[s] if j == 0 else 1
                u = rd(act(_bn(_conv2d(a, T[p + "expand.w"], 1), N[p + "sn1"])))
                u = rd(act(_bn(_dw(u, T[p + "dw.w"], st), N[p + "sn2"])))
                if (p + "se.fc1.w") in T:
                    zz = u.mean(dim=(2, 3))
                    zz = F.relu(F.linear(zz, _t(T[p + "se.fc1.w"]), _t(T[p + "se.fc1.b"])))
                    g = F.hardsigmoid(F.linear(zz, _t(T[p + "se.fc2.w"]), _t(T[p + "se.fc2.b"])))
                    u = rd(u * g[:, :, None, None])
                y = _bn(_conv2d(u, T[p + "project.w"], 1), N[p + "sn3"])
                a = rd(a + y) if (st == 1 and a.shape[1] == y.shape[1]) else rd(y)
        a = rd(F.hardswish(_bn(_conv2d(a, T["tail.w"], 1), N["tail.sn"])))
        z = rd(a.mean(dim=(2, 3)))
        z = rd(F.hardswish(F.linear(z, _t(T["fc1.w"]), _t(T["fc1.b"]))))
    else:
        raise ValueError(f)
    return F.linear(z, _t(T["head.w"]), _t(T["head.b"])).numpy()


def _standalone_transformer(spec, T, x, rd, return_hidden):
    b, sl, h = x.shape
    d = spec.head_dim
    j = 0
    while f"l{j}.q.w" in T:
        p = f"l{j}."
        lin = lambda t, nm: F.linear(t, _t(T[p + nm + ".w"]), _t(T[p + nm + ".b"]))
        nh = T[p + "q.w"].shape[0] // d
        q = rd(lin(x, "q")).view(b, sl, nh, d).transpose(1, 2)
        k = rd(lin(x, "k")).view(b, sl, nh, d).transpose(1, 2)
        v = rd(lin(x, "v")).view(b, sl, nh, d).transpose(1, 2)
        prob = rd(F.softmax(q @ k.transpose(-1, -2) / float(d) ** 0.5, dim=-1))
        ctx = rd((prob @ v).transpose(1, 2).reshape(b, sl, nh * d))
        u = rd(x + lin(ctx, "o"))
        x = rd(F.layer_norm(u, (h,), _t(T[p + "ln1.g"]), _t(T[p + "ln1.b"]), eps=1e-5))
        g = rd(F.gelu(lin(x, "ffn1")))
        u = rd(x + lin(g, "ffn2"))
        x = rd(F.layer_norm(u, (h,), _t(T[p + "ln2.g"]), _t(T[p + "ln2.b"]), eps=1e-5))
        j += 1
    logits = F.linear(x[:, 0, :], _t(T["head.w"]), _t(T["head.b"])).numpy()
    return (logits, x.numpy()) if return_hidden else logits
