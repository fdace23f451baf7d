"""Writes tests/golden/oracle_logits.txt from the CPU oracle alone.

The paper prints no logits or worked forward example, so these stored values
are not the paper's: they freeze the oracle's own output on small seeded cases
so that a later change to its arithmetic cannot pass unnoticed.  Run:
    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle   # noqa: E402
import synth    # noqa: E402

CASES = [("tiny", synth.TinySpec(), 8, [0, 3, 7]),
         ("resnet_small", synth.ResNetSpec(n_classes=12, stem_ch=16, stage_ch=(32, 64, 96, 128),
                                           max_depth=(3, 3, 4, 3), res_choices=(40, 48, 57)), 6, [0, 5]),
         ("mbv3_small", synth.MBV3Spec(res_choices=(40, 48, 57)), 5, [0, 4])]


def rows():
    for name, spec, n, picks in CASES:
        W = synth.make_weights(spec, 2312)
        S = synth.make_stats(spec, n, 2312)
        C = synth.enumerate_cfgs(spec, n, 16733)
        for i in picks:
            x = synth.make_inputs(spec, 1, C[i].in_h, C[i].in_w, 7)
            y = oracle.forward(spec, W, S, C[i], x)[0, :6]
            yield f"{name} {i} " + " ".join(f"{v:.10e}" for v in y)


if __name__ == "__main__":
    with open(os.path.join(os.path.dirname(__file__), "oracle_logits.txt"), "w") as f:
        f.write("# case cfg_index first-6-logits (oracle.forward, native storage mode); see make_golden.py\n")
        for r in rows():
            f.write(r + "\n")
