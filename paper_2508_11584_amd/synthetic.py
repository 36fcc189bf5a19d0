"""Engines on seeded synthetic weights: the glue between the input generators (`vpe_inputs`) and the binding.

Used by the benchmark, the smoke check and the tests to build a `vpe.Engine` for a `vpe_inputs.ModelSpec`.
Holds no arithmetic: it draws the weights, packs them into the blobs the C ABI takes and calls `vpe_create`
through the binding.
"""
from __future__ import annotations

import vpe_inputs as vi

from . import binding as vpe

KIND = {"seg": vi.HEAD_SEG, "depth": vi.HEAD_DEPTH, "det": vi.HEAD_DET, "dpt": vi.HEAD_DPT}


def head_cfgs(spec, seed, kinds, every_n=None):
    """Returns ([vpe.HeadCfg...], [weight dict...]) for the named heads.  The i-th repetition of a kind draws
    its weights from seed + 1000 i, so several heads of one kind are different heads."""
    cfgs, dicts, seen = [], [], {}
    for i, k in enumerate(kinds):
        rep = seen.get(k, 0)
        seen[k] = rep + 1
        hw = vi.make_head_weights(spec, KIND[k], seed + 1000 * rep)
        dicts.append(hw)
        classes = spec.seg_classes if k == "seg" else spec.det_classes if k == "det" else 0
        cfgs.append(vpe.HeadCfg(kind=KIND[k], weights=vi.pack_head(spec, KIND[k], hw), classes=classes,
                                channels=0 if k == "seg" else spec.head_ch,
                                every_n=1 if every_n is None else every_n[i]))
    return cfgs, dicts


def make_engine(spec, seed, kinds=("seg", "depth", "det"), every_n=None, ring_slots=2, flags=0, weights=None,
                torch_workspace=True, encoder_lanes=1, head_streams=0):
    """Returns (engine, backbone weight dict, [head weight dicts])."""
    w = weights if weights is not None else vi.make_backbone_weights(spec, seed)
    hc, hd = head_cfgs(spec, seed, kinds, every_n)
    eng = vpe.Engine(dim=spec.dim, depth=spec.depth, heads=spec.heads, mlp_hidden=spec.mlp_hidden,
                     mlp_kind=spec.mlp_kind, registers=spec.registers, img_h=spec.img_h, img_w=spec.img_w,
                     batch=spec.batch, dtype=vpe.VPE_BF16 if spec.dtype == "bf16" else vpe.VPE_F32,
                     taps=spec.taps, ring_slots=ring_slots, flags=flags, ln_eps=spec.ln_eps,
                     encoder_lanes=encoder_lanes, head_streams=head_streams,
                     weights=vi.pack_backbone(spec, w), head_cfgs=hc, torch_workspace=torch_workspace)
    return eng, w, hd
