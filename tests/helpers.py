"""Shared test plumbing: build an engine and oracle weights from one ModelSpec and seed."""
from __future__ import annotations

import numpy as np

import paper_2508_11584_amd as vpe
import vpe_inputs as vi

KIND = {"seg": vi.HEAD_SEG, "depth": vi.HEAD_DEPTH, "det": vi.HEAD_DET, "dpt": vi.HEAD_DPT}


def head_cfgs(spec, seed, kinds, every_n=None):
    """Returns ([vpe.HeadCfg...], [weight dict...]) for the named heads."""
    cfgs, dicts = [], []
    for i, k in enumerate(kinds):
        hw = vi.make_head_weights(spec, KIND[k], seed)
        dicts.append(hw)
        classes = spec.seg_classes if k == "seg" else spec.det_classes if k == "det" else 0
        cfgs.append(vpe.HeadCfg(kind=KIND[k], weights=vi.pack_head(spec, KIND[k], hw), classes=classes,
                                channels=0 if k == "seg" else spec.head_ch,
                                every_n=1 if every_n is None else every_n[i]))
    return cfgs, dicts


def make_engine(spec, seed, kinds=("seg", "depth", "det"), every_n=None, ring_slots=2, flags=0, weights=None,
                torch_workspace=True, encoder_lanes=1, head_streams=0):
    w = weights if weights is not None else vi.make_backbone_weights(spec, seed)
    hc, hd = head_cfgs(spec, seed, kinds, every_n)
    eng = vpe.Engine(dim=spec.dim, depth=spec.depth, heads=spec.heads, mlp_hidden=spec.mlp_hidden,
                     mlp_kind=spec.mlp_kind, registers=spec.registers, img_h=spec.img_h, img_w=spec.img_w,
                     batch=spec.batch, dtype=vpe.VPE_BF16 if spec.dtype == "bf16" else vpe.VPE_F32,
                     taps=spec.taps, ring_slots=ring_slots, flags=flags, ln_eps=spec.ln_eps, encoder_lanes=encoder_lanes, head_streams=head_streams,
                     weights=vi.pack_backbone(spec, w), head_cfgs=hc, torch_workspace=torch_workspace)
    return eng, w, hd


def relerr(got, ref) -> float:
    """max |got - ref| / max |ref| over one tensor (the gate's error measure)."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-300))


def depth_err(got, ref) -> float:
    """Depth error: max |got - depth| / max |depth before its final ReLU|.  ReLU is 1-Lipschitz, so this
    bounds the error of the un-clipped signal; normalising by max |depth| itself would blow up on the
    (random-weight) maps that the ReLU clips almost everywhere."""
    got = np.asarray(got, dtype=np.float64)
    return float(np.max(np.abs(got - ref["depth"])) / max(np.max(np.abs(ref["pre_relu"])), 1e-300))
