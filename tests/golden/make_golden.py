"""Writes tests/golden/tiny_vit_oracle.txt: sampled outputs of the CPU oracle on a small seeded model.

The paper prints no numeric model output, so no fixture here comes from the paper.  This file is a
regression pin of the oracle itself: it calls only `oracle/` (and the seeded input generator) and stores
a few dozen fp64 values; tests/test_oracle_golden.py recomputes and compares them, so an accidental
change to the oracle's arithmetic shows up even where the library-layer pins do not look.

Run from the repository root:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import vpe_inputs as vi  # noqa: E402
from oracle import model  # noqa: E402

SPEC = vi.ModelSpec("golden", dim=64, depth=4, heads=1, mlp_hidden=128, registers=1, img_h=42, img_w=56, dtype="f32",
                    taps=(1, 2, 3, 4), head_ch=64, seg_classes=5, det_classes=6)
SEED, IMG_SEED = 4242, 4343


def sample():
    w = vi.make_backbone_weights(SPEC, SEED)
    img = vi.make_image(SPEC.img_h, SPEC.img_w, IMG_SEED)
    feats = model.encode_image(SPEC, w, img)
    seg = model.seg_head(SPEC, vi.make_head_weights(SPEC, vi.HEAD_SEG, SEED), feats)
    det = model.det_head(SPEC, vi.make_head_weights(SPEC, vi.HEAD_DET, SEED), feats)
    dep = model.depth_head(SPEC, vi.make_head_weights(SPEC, vi.HEAD_DEPTH, SEED), feats)
    dpt = model.dpt_head(SPEC, vi.make_head_weights(SPEC, vi.HEAD_DPT, SEED), feats, return_stages=True)
    out = {}
    for k, f in enumerate(feats):
        out[f"feat{k}"] = f.ravel()[::97][:8]
    out["seg_logits"] = seg["logits"].ravel()[::7][:8]
    out["det_logits"] = det["logits"].ravel()[::5][:8]
    out["det_box"] = det["box"].ravel()[::3][:8]
    out["depth_pre_relu"] = dep["pre_relu"].ravel()[::131][:8]
    out["dpt_l3"] = dpt["l"][3].ravel()[::11][:8]
    out["dpt_path0"] = dpt["paths"][-1].ravel()[::1201][:8]
    out["dpt_pre_relu"] = dpt["pre_relu"].ravel()[::131][:8]
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_vit_oracle.txt")
    with open(path, "w") as f:
        f.write("# written by tests/golden/make_golden.py from oracle/ only (no paper values exist for this path)\n")
        for name, vals in sample().items():
            f.write(name + " " + " ".join(repr(float(v)) for v in vals) + "\n")
    print("wrote", path)
