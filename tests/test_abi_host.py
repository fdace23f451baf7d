"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and its layout queries / architecture validation behave."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2312_16733_amd as sna
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SPECS = [synth.TinySpec(), synth.ResNetSpec(), synth.MBV3Spec(), synth.TransformerSpec()]


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "subnetact.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(sna_[a-z_]+)\s*\(", hdr))
    assert {"sna_supernet_load", "sna_subnet_forward", "sna_supernet_free"} <= names
    L = ctypes.CDLL(sna.library_path())
    for n in sorted(names):
        assert hasattr(L, n), n


@pytest.mark.parametrize("spec", SPECS, ids=[s.family for s in SPECS])
def test_layout_matches_the_family_description(spec):
    a = sna.arch_desc_from_spec(spec)
    tis = sna.tensor_infos(a)
    want = spec.tensors()
    assert [t.name.decode() for t in tis] == [t.name for t in want]
    end = 0
    for ti, td in zip(tis, want):
        nd = {0: 4, 1: 3, 2: 2, 3: 1}[ti.kind]
        assert tuple(ti.dims[:nd]) == tuple(td.shape)
        assert ti.offset % 256 == 0 and ti.offset >= end
        end = ti.offset + ti.bytes
    assert sna.lib().sna_weights_bytes(ctypes.byref(a)) >= end
    nis = sna.norm_infos(a)
    assert [(n.name.decode(), n.channels) for n in nis] == list(spec.norms())
    off = 0
    for n in nis:
        assert n.offset == off
        off += n.channels
    assert sna.lib().sna_stats_row_len(ctypes.byref(a)) == off


def test_pack_weights_places_bf16_bits():
    spec = synth.MBV3Spec()
    a = sna.arch_desc_from_spec(spec)
    W = synth.make_weights(spec, 1)
    blob = sna.pack_weights(a, W)
    ti = [t for t in sna.tensor_infos(a) if t.name == b"s2.b1.dw.w"][0]
    raw = blob[ti.offset:ti.offset + ti.bytes].view(np.uint16).astype(np.uint32) << 16
    np.testing.assert_array_equal(raw.view(np.float32).reshape(W["s2.b1.dw.w"].shape), W["s2.b1.dw.w"])
    W["stem.w"][0, 0, 0, 0] = np.float32(1.0 + 2.0 ** -12)     # not a bf16 value
    with pytest.raises(ValueError):
        sna.pack_weights(a, W)


def test_bad_architectures_are_rejected():
    L = sna.lib()
    a = sna.arch_desc_from_spec(synth.ResNetSpec())
    a.stage_ch[1] = 500                     # not a multiple of 8
    assert L.sna_tensor_count(ctypes.byref(a)) == -2
    assert b"stage_ch" in L.sna_last_error()
    a = sna.arch_desc_from_spec(synth.ResNetSpec())
    a.dtype = 0
    assert L.sna_weights_bytes(ctypes.byref(a)) == -2
    a = sna.arch_desc_from_spec(synth.TransformerSpec())
    a.head_dim = 32
    assert L.sna_workspace_bytes(ctypes.byref(a), 4, 4) == -2
    a = sna.arch_desc_from_spec(synth.TinySpec())
    assert L.sna_workspace_bytes(ctypes.byref(a), 0, 4) == -6
    assert L.sna_supernet_load(None, None, 0, None, 0, 1, 1, None, 0, None, None) == -1


def test_workspace_grows_with_batch():
    a = sna.arch_desc_from_spec(synth.ResNetSpec())
    w1 = sna.lib().sna_workspace_bytes(ctypes.byref(a), 16, 1)
    w64 = sna.lib().sna_workspace_bytes(ctypes.byref(a), 16, 64)
    assert 0 < w1 < w64


@pytest.mark.parametrize("family", ["resnet", "mbv3", "transformer"])
def test_shipped_tuning_tables_are_well_formed(family):
    """The tables `bench.py --save-tuning` wrote: every line is a tile-variant ("v") or K-split ("s")
    entry with 7 key fields (the last: same-shaped problems sharing the launch) and a value the library accepts (an import would drop anything else)."""
    path = os.path.join(os.path.dirname(sna.library_path()), "tuned", f"gfx950_{family}.txt")
    nv = sna.lib().sna_tile_variant_count()
    assert nv >= 7
    seen, n = set(), 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        assert f[0] in ("v", "s") and len(f) == 9, line
        key = tuple(int(x) for x in f[1:8])
        val = int(f[8])
        m, k, c, taps, stride, parts, twins = key
        assert 1 <= twins <= 16, line
        assert m >= 1 and k >= 8 and k % 8 == 0 and c >= 8 and c % 8 == 0 and taps in (1, 9, 49) and stride in (1, 2, 128), line
        assert (0 <= val < nv and parts >= 1) if f[0] == "v" else (val in (0, 1) and parts == 0), line
        assert (f[0], key) not in seen, line
        seen.add((f[0], key))
        n += 1
    assert n > 20
